// Vocabulary pass of the Power-SMC step (Alg. 1 "sample" and "update"; Eq. "inc"; Cor. 1) for gfx950, with the row
// finalizer (Sec. 5.3 boundary reweight + Eq. "inc") and, on request, the per-prompt resampling (Eq. "ess"; Alg. 1)
// folded into the tail of the same launch.
//
// One read of every logit of every row produces, per row:
//   log Z_1 = LSE_v(l_v), log Z_beta = LSE_v(beta l_v), and the Gumbel-max draw argmax_v(beta l_v + g_v),
// from which log p(y), log q(y) and the increment alpha log p(y) - log q(y) follow.
//
// The work is HBM-bound streaming; there is no contraction here, hence no MFMA.  A row is split over
// n_split workgroups of 256, 512 or 1024 threads; every thread streams 16-byte vectors.  The two sums are kept per
// lane against a wave-uniform power-of-two reference, so a rising running maximum rescales them exactly.
//
// Exact lazy Gumbel-max: g is bounded, g in [kGumbelMin, kGumbelMax].  An entry whose best possible key
// beta*l_v + kGumbelMax is below a key that some entry is already known to reach cannot be the argmax, so it
// draws no random number.  The threshold on l_v ("thr") only ever rises; it comes from the wave's running maximum,
// from the key that the entry holding a new running maximum really reaches (its variate is drawn at once, for the
// bound alone), from keys already scored, and from one LDS word per workgroup that all its waves raise with an LDS atomic max
// and read without waiting -- a stale value only makes the filter more conservative, never wrong.  The filter works
// on whole 16-byte vectors: a lane whose vector holds an entry at or above thr appends the vector as loaded (16 bytes
// + its index) to a per-wave LDS ring -- one compare and one ballot per vector, not per entry.  Scoring is deferred
// to the end of the slice, when the bound is known best, and takes 64 queued vectors at a time: every lane re-tests
// the entries of one vector against the bound as it stands then and draws Philox blocks only for the quads that still
// hold a possible winner.  The result is the same argmax as scoring every entry.  The "dense" instantiation scores
// every entry in place.
//
// Tail.  The workgroup that writes the last slice of a row (a ticket per row) merges the row's slices in fp64,
// re-ranks the finalists with fp64 keys, and applies the boundary reweight and the increment.  With resampling
// folded in, the wave that finalizes the last row of a prompt (a ticket per prompt) goes on to normalise the
// prompt's weights and resample it.  Tickets return to zero by themselves, so the launch can be replayed.  What is handed
// over behind a ticket (a slice's record, a row's weight) is written and read at agent scope, and the ticket is taken once
// those writes have completed; no cache is written back or invalidated for it.
#pragma once
#include "weights_device.hpp"

namespace psmc {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

typedef unsigned int vec16 __attribute__((ext_vector_type(4)));    // one 16-byte global load

template <int DT> struct Elems;
template <> struct Elems<SMC_BF16> { static constexpr int kPerVec = 8; };
template <> struct Elems<SMC_F32>  { static constexpr int kPerVec = 4; };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <int DT>
__device__ __forceinline__ void unpack(const uint4& raw, float (&x)[Elems<DT>::kPerVec])
{
    if constexpr (DT == SMC_BF16) {
        x[0] = bf16_lo(raw.x); x[1] = bf16_hi(raw.x); x[2] = bf16_lo(raw.y); x[3] = bf16_hi(raw.y);
        x[4] = bf16_lo(raw.z); x[5] = bf16_hi(raw.z); x[6] = bf16_lo(raw.w); x[7] = bf16_hi(raw.w);
    } else {
        x[0] = __uint_as_float(raw.x); x[1] = __uint_as_float(raw.y);
        x[2] = __uint_as_float(raw.z); x[3] = __uint_as_float(raw.w);
    }
}

template <int DT>
__device__ __forceinline__ float vec_max(const float (&x)[Elems<DT>::kPerVec])
{
    if constexpr (DT == SMC_BF16)
        return fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    else
        return fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
}

template <int DT>
__device__ __forceinline__ float load_scalar(const void* row, int64_t i)
{
    if constexpr (DT == SMC_BF16) return __uint_as_float((uint32_t)((const uint16_t*)row)[i] << 16);
    else return ((const float*)row)[i];
}

// e^P for small integer P by multiplication
template <int P> __device__ __forceinline__ float ipow(float e)
{
    if constexpr (P == 1) return e;
    else if constexpr (P == 2) return e * e;
    else if constexpr (P == 3) return e * e * e;
    else if constexpr (P == 4) { float a = e * e; return a * a; }
    else if constexpr (P == 5) { float a = e * e; return a * a * e; }
    else if constexpr (P == 6) { float a = e * e; return a * a * a; }
    else { float a = e * e; a = a * a; return a * a; }   // P == 8
}

struct Cand { float l, g; int32_t i; };

// value known to be equal on every lane -> scalar register
__device__ __forceinline__ float uniform(float v)
{
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(v)));
}

// is candidate (l,g,i) ahead of (bl,bg,bi)?  Keys compared through differences so that no large
// common term is rounded; equal keys go to the lower index.
__device__ __forceinline__ bool ahead(float beta, float l, float g, int32_t i, float bl, float bg, int32_t bi)
{
    if (bi < 0) return true;
    const float d = fmaf(beta, l - bl, g - bg);
    return d > 0.0f || (d == 0.0f && i < bi);
}

struct LaneTop2 {
    Cand a, b;
    __device__ __forceinline__ void init() { a = Cand{0.f, 0.f, -1}; b = Cand{0.f, 0.f, -1}; }
    __device__ __forceinline__ void offer(float beta, float l, float g, int32_t i)
    {
        if (ahead(beta, l, g, i, a.l, a.g, a.i)) { b = a; a = Cand{l, g, i}; }
        else if (ahead(beta, l, g, i, b.l, b.g, b.i)) { b = Cand{l, g, i}; }
    }
};

// Best two of one candidate per lane (index < 0: none) by fp32 key relative to `ref`; ties to the lower lane.
// Returns the lanes holding the best and the runner-up (-1: none).  `ka` / `kb` are the lane's first and second key.
__device__ __forceinline__ void wave_best_two(float ka, float kb, bool has_a, int& lane_best, int& lane_second,
                                              bool& second_is_b)
{
    const float NEG = -3.4e38f;
    const int lane = lane_id();
    ka = has_a ? ka : NEG;
    const float best = wave_max_f32(ka);
    const unsigned long long who = __ballot(ka == best && has_a);
    lane_best = who ? __ffsll((long long)who) - 1 : -1;
    const float mine = lane == lane_best ? kb : ka;
    const float k2 = wave_max_f32(mine);
    const unsigned long long who2 = __ballot(mine == k2 && k2 > NEG);
    lane_second = who2 ? __ffsll((long long)who2) - 1 : -1;
    second_is_b = lane_second == lane_best;
}

// Workgroup summary: per-wave sums (each against its own power-of-two reference) and per-lane best-two candidates
// are merged and written as this slice's Partial, to global memory and to `lds_copy` (for a row of one slice the
// finalizer reads it from there).  m_wave is the wave's reference for comparing keys across lanes.
// Data that one workgroup hands to another inside a launch (a slice's record, a row's weight) is written and read
// with agent-scope accesses: they go to the level of the memory system that all compute units share, so that a ticket
// taken after the writes have completed (an explicit wait for the wave's vector memory operations) publishes them.  A release at agent
// scope would do as well, but it writes back -- and the matching acquire invalidates -- whole caches, which every row
// would then do to the logit stream of its neighbours.
template <typename T> __device__ __forceinline__ void store_shared(T* p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ T load_shared(const T* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Takes a ticket after this lane's earlier stores have completed; returns its number (lane 0's, on every lane).
__device__ __forceinline__ int take_ticket(int32_t* ticket)
{
    // The fence keeps the compiler from moving the stores behind the ticket; by itself it waits for nothing at this
    // scope.  The wait is spelled out: vmcnt(0) -- every vector memory operation of this wave, the agent-scope stores
    // among them, has been acknowledged (s_waitcnt encoding of this family: vmcnt in bits 3:0 and 15:14, expcnt 6:4
    // and lgkmcnt 11:8 left at their maxima, i.e. not waited for).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    int tk = 0;
    if (lane_id() == 0) tk = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_amdgcn_readfirstlane(tk);
}

template <int NW>
__device__ __forceinline__ void block_epilogue(float beta, float m_wave, float M1, float Mb, float s1, float sb,
                                               const LaneTop2 top, unsigned long long n_scored,
                                               unsigned long long n_drains, Partial* __restrict__ out, Partial* lds_copy)
{
    static_assert(2 * NW <= kWave, "one wave merges two candidates per wave");
    __shared__ float red_f[NW][5];
    __shared__ float red_cl[NW][2], red_cg[NW][2];
    __shared__ int32_t red_ci[NW][2];
    __shared__ uint32_t red_n[NW][2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float NEG = -3.4e38f;

    s1 = wave_sum_f32(s1);
    sb = wave_sum_f32(sb);
    {
        const float ka = fmaf(beta, top.a.l - m_wave, top.a.g);
        const float kb = top.b.i >= 0 ? fmaf(beta, top.b.l - m_wave, top.b.g) : NEG;
        int lb, l2; bool sec_b;
        wave_best_two(ka, kb, top.a.i >= 0, lb, l2, sec_b);
        if (lane == lb) { red_cl[wave][0] = top.a.l; red_cg[wave][0] = top.a.g; red_ci[wave][0] = top.a.i; }
        if (lane == l2) {
            red_cl[wave][1] = sec_b ? top.b.l : top.a.l; red_cg[wave][1] = sec_b ? top.b.g : top.a.g;
            red_ci[wave][1] = sec_b ? top.b.i : top.a.i;
        }
        const int sc = wave_sum_i32((int)n_scored);
        if (lane == 0) {
            if (lb < 0) red_ci[wave][0] = -1;
            if (l2 < 0) red_ci[wave][1] = -1;
            red_f[wave][0] = M1; red_f[wave][1] = s1; red_f[wave][2] = Mb; red_f[wave][3] = sb; red_f[wave][4] = m_wave;
            red_n[wave][0] = (uint32_t)sc; red_n[wave][1] = (uint32_t)n_drains;
        }
    }
    __syncthreads();
    if (wave == 0) {
        // sums: lane w < NW holds wave w
        const bool hw = lane < NW;
        const float wM1 = hw ? red_f[lane][0] : -INFINITY, wMb = hw ? red_f[lane][2] : -INFINITY;
        const float gM1 = wave_max_f32(wM1), gMb = wave_max_f32(wMb);
        const float gm = wave_max_f32(hw ? red_f[lane][4] : -3.0e38f);
        // a wave that saw nothing but masked (-inf) entries has reference -inf and sum 0; when every wave of the
        // slice is like that the difference of the references is not a number, hence the explicit zero
        const float t1 = wave_sum_f32(hw && wM1 > -INFINITY ? red_f[lane][1] * fast_exp2(wM1 - gM1) : 0.f);
        const float tb = wave_sum_f32(hw && wMb > -INFINITY ? red_f[lane][3] * fast_exp2(wMb - gMb) : 0.f);
        const uint32_t nsc = (uint32_t)wave_sum_i32(hw ? (int)red_n[lane][0] : 0);
        const uint32_t ndr = (uint32_t)wave_sum_i32(hw ? (int)red_n[lane][1] : 0);
        // candidates: lane c < 2*NW holds candidate (c & 1) of wave (c >> 1)
        const bool hc = lane < 2 * NW;
        const float cl = hc ? red_cl[lane >> 1][lane & 1] : 0.f, cg = hc ? red_cg[lane >> 1][lane & 1] : 0.f;
        const int32_t ci = hc ? red_ci[lane >> 1][lane & 1] : -1;
        const float key = fmaf(beta, cl - gm, cg);
        int lb, l2; bool sec_b;
        wave_best_two(key, NEG, ci >= 0, lb, l2, sec_b);
        const int sb_lane = lb < 0 ? 0 : lb, s2_lane = (l2 < 0 || sec_b) ? 0 : l2;
        const float l1v = read_lane(cl, sb_lane), g1v = read_lane(cg, sb_lane); const int32_t i1v = read_lane(ci, sb_lane);
        const float l2v = read_lane(cl, s2_lane), g2v = read_lane(cg, s2_lane); const int32_t i2v = read_lane(ci, s2_lane);
        if (lane == 0) {
            Partial p;
            p.M1 = gM1; p.s1 = t1; p.Mb = gMb; p.sb = tb;
            p.l1 = l1v; p.g1 = g1v; p.i1 = lb < 0 ? -1 : i1v;
            p.l2 = l2v; p.g2 = g2v; p.i2 = (l2 < 0 || sec_b) ? -1 : i2v;
            p.n_scored = (int32_t)nsc; p.n_drains = (int32_t)ndr;
            if (out) {                                  // a row of several slices: another workgroup may read the record
                store_shared(&out->M1, p.M1); store_shared(&out->s1, p.s1); store_shared(&out->Mb, p.Mb); store_shared(&out->sb, p.sb);
                store_shared(&out->l1, p.l1); store_shared(&out->g1, p.g1); store_shared(&out->i1, p.i1);
                store_shared(&out->l2, p.l2); store_shared(&out->g2, p.g2); store_shared(&out->i2, p.i2);
                store_shared(&out->n_scored, p.n_scored); store_shared(&out->n_drains, p.n_drains);
            }
            *lds_copy = p;
        }
    }
}

// order-preserving map float -> int for atomicMax on a shared lower bound
__device__ __forceinline__ int enc_bound(float f) { const int i = __float_as_int(f); return i >= 0 ? i : i ^ 0x7FFFFFFF; }
__device__ __forceinline__ float dec_bound(int i) { return __int_as_float(i >= 0 ? i : i ^ 0x7FFFFFFF); }

// Scalars of one step as the kernels see them: by value, or -- when the context keeps its step on the device -- from the
// device-resident counter and exponent schedule, so that a captured launch advances when it is replayed.
struct StepScalars { uint32_t step; double alpha_t, alpha_prev, beta; };

__device__ __forceinline__ StepScalars step_scalars(const StepArgs& a)
{
    StepScalars s{a.step, a.alpha_t, a.alpha_prev, a.beta};
    if (a.d_step) {
        const int t = *a.d_step;
        s.step = (uint32_t)t;
        const int last = a.n_sched - 1;
        s.alpha_t = a.d_sched[t < last ? t : last];
        s.alpha_prev = a.d_sched[t - 1 < last ? (t > 0 ? t - 1 : 0) : last];
        if (a.tau_by_value <= 0.0) s.beta = s.alpha_t;
    }
    return s;
}

// ------------------------------------------------------------------------------------------------
// Row finalizer (a0 + a2) by one wave.  Merges the row's partials in fp64, re-ranks the finalists of the
// Gumbel-max draw with fp64 keys beta*l + g (ties to the lower index), then applies the boundary reweight of
// exponent bridging (Sec. 5.3) and the increment alpha*log p(y) - log q(y) (Eq. "inc").
// pp: the row's n_split partial records (global memory, or LDS for a row of one slice).
// What the finalizer needs of a row's state.  Read when the kernel starts, long before it is used: a dependent global read
// at the end of the kernel would wait behind the whole chip's logit stream.
struct RowState { double logW, cumlogp; int32_t* hist; };

__device__ __forceinline__ RowState load_row_state(const StepArgs& a, uint32_t row)
{
    RowState r;
    r.logW = a.logW[row];
    r.cumlogp = a.cumlogp[row];
    r.hist = a.histAB ? a.histAB[a.parity[row]] : nullptr;
    return r;
}

__device__ inline void finalize_row(const StepArgs& a, const StepScalars& sc, uint32_t row, const Partial* pp, int n_split,
                                    const RowState& rs)
{
    const int lane = lane_id();
    const double beta = sc.beta, alpha_t = sc.alpha_t, alpha_prev = sc.alpha_prev;
    const uint32_t step = sc.step;

    // lane c takes what it needs of the records: the sums of slice c, candidate (c & 1) of slice (c >> 1).  A row of one
    // slice reads this workgroup's own record (LDS); records of other workgroups are read at agent scope.
    Partial mine{}, cand{};
    mine.M1 = -INFINITY; mine.Mb = -INFINITY; cand.i1 = -1; cand.i2 = -1;
    if (n_split == 1) {
        if (lane < 2) { mine = pp[0]; cand = mine; }
    } else {
        if (lane < n_split) {
            const Partial* q = pp + lane;
            mine.M1 = load_shared(&q->M1); mine.s1 = load_shared(&q->s1); mine.Mb = load_shared(&q->Mb); mine.sb = load_shared(&q->sb);
            mine.n_scored = load_shared(&q->n_scored); mine.n_drains = load_shared(&q->n_drains);
        }
        if (lane < 2 * n_split) {
            const Partial* q = pp + (lane >> 1);
            if (lane & 1) { cand.i2 = load_shared(&q->i2); cand.l2 = load_shared(&q->l2); cand.g2 = load_shared(&q->g2); }
            else { cand.i1 = load_shared(&q->i1); cand.l1 = load_shared(&q->l1); cand.g1 = load_shared(&q->g1); }
        }
    }

    // sums: the references are integer powers of two, so bringing a slice to the common reference is exact
    double M1 = -1e300, Mb = -1e300, s1 = 0.0, sb = 0.0;
    if (lane < n_split) { M1 = mine.M1; Mb = mine.Mb; s1 = mine.s1; sb = mine.sb; }
    const double gM1 = wave_max_f64(M1), gMb = wave_max_f64(Mb);
    const double S1 = wave_sum_f64(lane < n_split && M1 > -1e300 ? ldexp(s1, (int)fmax(M1 - gM1, -2000.0)) : 0.0);
    const double Sb = wave_sum_f64(lane < n_split && Mb > -1e300 ? ldexp(sb, (int)fmax(Mb - gMb, -2000.0)) : 0.0);
    constexpr double LN2 = 0.69314718055994530942;
    // the two logarithms side by side on two lanes (one pass through the fp64 log instead of two in a row)
    const double lg = log((lane & 1) ? Sb : S1);
    const double logZ1 = gM1 * LN2 + read_lane(lg, 0);
    const double logZb = gMb * LN2 + read_lane(lg, 1);

    const int32_t nsc = wave_sum_i32(lane < n_split ? mine.n_scored : 0);
    const int32_t ndr = wave_sum_i32(lane < n_split ? mine.n_drains : 0);

    // finalists: lane c -> candidate (c & 1) of split (c >> 1).  The finalist's logit and fp32 Gumbel variate travel in
    // the partial record (the logit is an exact copy: bf16 and fp32 both fit a float), so no second read of the logits.
    int32_t idx = -1;
    float lf = 0.f, gf = 0.f;
    if (lane < 2 * n_split) {
        idx = (lane & 1) ? cand.i2 : cand.i1;
        lf = (lane & 1) ? cand.l2 : cand.l1;
        gf = (lane & 1) ? cand.g2 : cand.g1;
    }
    if (idx >= a.V) idx = -1;                          // never trust an index outside the row, whatever the partial holds
    const bool has = idx >= 0;
    // fp32 keys relative to the largest finalist logit (differences of logits are exact or nearly so)
    const float lref = wave_max_f32(has ? lf : -3.4e38f);
    const float kf = has ? fmaf((float)beta, lf - lref, gf) : -3.4e38f;
    const float kf1 = wave_max_f32(kf);
    const unsigned long long lead = __ballot(has && kf == kf1);
    const int lead_lane = lead ? __ffsll((long long)lead) - 1 : 0;
    const float kf2 = wave_max_f32(lane == lead_lane ? -3.4e38f : kf);
    int32_t y, second;
    double gap, ly;
    // The fp32 keys carry an error of a few 1e-7; a lead of more than 1e-3 decides the draw.  Closer calls (and rows
    // with no finalist) are re-ranked with fp64 keys beta*l + g from the random stream, ties to the lower index --
    // the arithmetic of the plain definition.
    if (lead != 0ull && (lead & (lead - 1)) == 0ull && kf1 - kf2 > 1.0e-3f) {
        y = read_lane(idx, lead_lane);
        ly = (double)read_lane(lf, lead_lane);
        const unsigned long long runner = __ballot(has && lane != lead_lane && kf == kf2);
        second = runner ? read_lane(idx, __ffsll((long long)runner) - 1) : -1;
        gap = runner ? (double)(kf1 - kf2) : (double)INFINITY;
    } else {
        double key = -INFINITY;
        const double lv = (double)lf;
        if (has) {
            const U4 blk = philox4x32_10((uint32_t)idx >> 2, row, step, 0u, a.key0, a.key1);
            key = beta * lv + gumbel_f64(pick_word(blk, (uint32_t)idx & 3u));
        }
        const double k1 = wave_max_f64(key);
        y = wave_min_i32((has && key == k1) ? idx : 0x7FFFFFFF);       // max key, lowest index among equals
        const double k2 = wave_max_f64((has && idx != y) ? key : -INFINITY);
        const int32_t c2 = wave_min_i32((has && idx != y && key == k2) ? idx : 0x7FFFFFFF);
        second = c2 == 0x7FFFFFFF ? -1 : c2;
        gap = k1 - k2;
        const unsigned long long ymask = __ballot(idx == y);
        ly = read_lane(lv, ymask ? __ffsll((long long)ymask) - 1 : 0);
    }

    if (lane == 0) {
        const bool ok = (y != 0x7FFFFFFF) && isfinite(logZ1) && isfinite(logZb);
        const int32_t tok = ok ? y : 0;
        const double logp = ly - logZ1;
        const double logq = beta * ly - logZb;
        const double delta = alpha_t * logp - logq;
        double w = rs.logW + (alpha_t - alpha_prev) * rs.cumlogp;          // stage boundary on the prefix y_{1:t-1}
        w += delta;
        store_shared(&a.logW[row], w);                  // (the wave that resamples the prompt may belong to another workgroup)
        a.cumlogp[row] = rs.cumlogp + logp;
        a.tokens_out[row] = tok;
        // (a device-resident step may have run past the end of the history)
        if (rs.hist && step >= 1u && step <= (uint32_t)a.T_max) rs.hist[(int64_t)row * a.T_max + (step - 1)] = tok;
        a.d_delta[row] = delta; a.d_logZ1[row] = logZ1; a.d_logZb[row] = logZb;
        a.d_gap[row] = gap;
        a.d_second[row] = second;
        a.d_rowstat[3 * row] = ok ? 0 : 1; a.d_rowstat[3 * row + 1] = nsc; a.d_rowstat[3 * row + 2] = ndr;
        if (a.eos_id >= 0 && ok && tok == a.eos_id) a.done[row] = 1;
    }
}

// Absorbing state (Alg. 1 "if done"; App. D): y_t = EOS, increment 1; the stage-boundary reweight still re-targets
// the particle's prefix (App. B).  One lane.
__device__ inline void finalize_done_row(const StepArgs& a, const StepScalars& sc, uint32_t row)
{
    store_shared(&a.logW[row], a.logW[row] + (sc.alpha_t - sc.alpha_prev) * a.cumlogp[row]);
    a.tokens_out[row] = a.eos_id;
    if (a.histAB && sc.step >= 1u && sc.step <= (uint32_t)a.T_max) {
        int32_t* h = a.histAB[a.parity[row]];
        if (h) h[(int64_t)row * a.T_max + (sc.step - 1)] = a.eos_id;
    }
    a.d_delta[row] = 0.0; a.d_logZ1[row] = 0.0; a.d_logZb[row] = 0.0; a.d_gap[row] = INFINITY; a.d_second[row] = -1;
    a.d_rowstat[3 * row] = 0; a.d_rowstat[3 * row + 1] = 0; a.d_rowstat[3 * row + 2] = 0;
}

// After a row is final: with resampling folded into this launch, the wave that completes a prompt resamples it.
// lds: at least 2*N doubles + one int, free for this wave's use.
__device__ inline void after_row_final(const StepArgs& a, const StepScalars& sc, uint32_t row, unsigned char* lds)
{
    if (!a.fuse_resample) return;
    const int lane = lane_id();
    const int b = (int)row / a.rs.N;
    const int tk = take_ticket(&a.prompt_ticket[b]);   // this row's weight has been written
    if (tk != a.rs.N - 1) return;
    if (lane == 0) store_shared(&a.prompt_ticket[b], 0);   // nobody else touches it until the next step
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); // (keeps the reads below behind the ticket)
    double* sh_a = reinterpret_cast<double*>(lds);
    double* sh_b = sh_a + a.rs.N;
    int* sh_k = reinterpret_cast<int*>(sh_b + a.rs.N);
    resample_prompt(a.rs, a.logW, b, sc.step, sh_a, sh_b, sh_k);
}

}  // namespace

// P > 0: beta is the integer P (sum of e^P by multiplication); P == 0: generic beta (second exp2).
// DENSE: every entry is scored in place (no filter, no ring) -- the plain definition, kept for cross-checks.
// NW: waves per workgroup (4, 8 or 16).
template <int DT, int P, bool DENSE, int NW>
__global__ __launch_bounds__(NW * kWave, 4) void vocab_pass_kernel(const StepArgs a)
{
    constexpr int EPV = Elems<DT>::kPerVec;
    constexpr int QPV = EPV / 4;                       // Philox blocks (four entries each) per vector
    constexpr int UNROLL = 4;                          // 16-byte loads per thread and register set (two sets alternate)
    constexpr int THREADS = NW * kWave;
    constexpr int kRingV = 256;                        // queued vectors per wave (power of two, >= 2 wave-widths)
    constexpr int kRingE = 128;                        // queued single entries per wave (power of two, 2 wave-widths)
    // A drain that finds more than this many entries still above the bound scores its vectors as they are (one Philox
    // block serves the four entries of a quad); fewer are compacted into the entry ring first, so that every lane of
    // a scoring pass has an entry to score.  The two costs meet at about 2.5 entries per lane.
    constexpr int kScoreAsVectors = 160;
    // LDS: the candidate rings while streaming; afterwards the same bytes serve the resampling of a prompt
    constexpr int kRingBytes = DENSE ? 0 : NW * (kRingV * 20 + kRingE * 8);
    constexpr int kTailBytes = 2 * SMC_MAX_PARTICLES * 8 + 16;
    constexpr int kLdsBytes = kRingBytes > kTailBytes ? kRingBytes : kTailBytes;
    __shared__ __align__(16) unsigned char lds[kLdsBytes];
    __shared__ int wg_bound;                           // best "cannot win below this" bound of the whole workgroup
    __shared__ Partial sh_part;                        // this workgroup's partial record, for a row of one slice

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_split = a.n_split;
    const int split = blockIdx.x % n_split;
    const uint32_t row = blockIdx.x / n_split;
    const StepScalars sc = step_scalars(a);
    if (a.eos_id >= 0 && a.done[row]) {                // terminated particle (App. D): its logits are not read
        if (split == 0 && wave == 0) {
            if (lane == 0) finalize_done_row(a, sc, row);
            after_row_final(a, sc, row, lds);
        }
        return;
    }
    uint4* const ring_raw = reinterpret_cast<uint4*>(lds) + (DENSE ? 0 : wave * kRingV);
    uint32_t* const ring_idx = reinterpret_cast<uint32_t*>(lds + (DENSE ? 0 : NW * kRingV * 16)) + (DENSE ? 0 : wave * kRingV);
    uint2* const ring_ent = reinterpret_cast<uint2*>(lds + (DENSE ? 0 : NW * kRingV * 20)) + (DENSE ? 0 : wave * kRingE);
    const char* rowp = (const char*)a.logits + (int64_t)row * a.row_stride_bytes;
    const int V = a.V;
    const uint32_t key0 = a.key0, key1 = a.key1, step = sc.step;
    if (tid == 0) wg_bound = enc_bound(-INFINITY);
    __syncthreads();
    RowState row_state{};
    if (wave == 0) row_state = load_row_state(a, row);    // wave-uniform (scalar) reads, consumed by the tail

    const int nvec_full = V / EPV;                      // vectors wholly inside the row
    const int nvec = (V + EPV - 1) / EPV;
    const int vec_begin = split * a.vecs_per_split;
    const int vec_end = min(vec_begin + a.vecs_per_split, nvec);

    const float beta = (float)sc.beta;
    const float beta_l2e = beta * kLog2e;
    const float window = (kGumbelMax - kGumbelMin + kKeyMargin) / beta;   // in logit units

    constexpr uint32_t kPadWord = DT == SMC_BF16 ? 0xFF80FF80u : 0xFF800000u;      // -inf in every element

    // wave-uniform running state
    float m = -3.0e38f;            // running max of the logits seen by this wave
    // power-of-two references (integers): M1 >= m*log2e, Mb >= m*beta*log2e.  Finite from the start, so that a masked
    // (-inf) entry met before any finite one has a well-defined exponent of -inf
    float M1 = -3.0e38f, Mb = -3.0e38f;
    float thr = -3.4e38f;          // entries below thr cannot win
    float published = -3.4e38f;    // what this wave last wrote to the row's shared bound
    float c1 = 0.f, cb = 0.f;      // c1 = M1 - m*log2e, cb = Mb - m*beta*log2e, both >= 0
    float s1 = 0.f, sb = 0.f;      // per-lane sums relative to the references
    float thr_rel = -3.4e38f;      // the filter bound in the units the stream works in, rounded down: thr - m where the
                                   // stream forms d = x - m (fp32 rows), thr*log2e - M1 where it forms t = x*log2e - M1 (bf16 rows)
    float t_max = -3.4e38f;        // bf16 rows: m in those units, t_max = m*log2e - M1
    int q_head = 0, q_count = 0;   // ring of queued vectors
    int e_head = 0, e_count = 0;   // ring of queued single entries (always < 64 between drains)
    unsigned long long n_scored = 0, n_drains = 0;
    LaneTop2 top; top.init();
    // the lane's highest entry among the vectors that raised the wave's running maximum since the last probe
    float probe_l = -INFINITY;
    uint32_t probe_i = 0u;
    bool probe_pending = false;                        // wave-uniform

    auto lower = [](float b) { return b - fabsf(b) * 4e-7f; };    // a few ulps down: never drop a possible winner

    // thr in units relative to the running maximum, with the rounding of both subtractions on the safe side
    // bf16 rows take the exponent straight from the logit, t = fma(x, log2e, -M1): one instruction less per entry than
    // forming x - m first.  The product is exact inside the fma, so the only error is that of the fp32 constant,
    // 2^(x*kLog2eLow); its bulk 2^(m*kLog2eLow) is a per-wave factor applied to the sums at the end, what remains is
    // below 1e-6 for entries within a hundred units of the maximum (others add nothing).  fp32 rows, whose magnitudes
    // are unbounded and whose stream is bound by HBM anyway, keep the x - m form.
    constexpr bool kDirect = DT == SMC_BF16;
    constexpr double kLog2eLow = 1.4426950408889634074 - (double)kLog2e;

    auto set_thr = [&](float t) __attribute__((always_inline)) {
        thr = fmaxf(thr, t);
        if constexpr (kDirect) thr_rel = fmaf(thr, kLog2e, -M1) - (fabsf(thr) * kLog2e + fabsf(M1)) * 3e-7f;
        else thr_rel = (thr - m) - (fabsf(thr) + fabsf(m)) * 3e-7f;
    };

    auto raise_max = [&](float nm) __attribute__((always_inline)) {                    // nm > m, wave-uniform
        nm = uniform(nm);
        const float nM1 = ceilf(nm * kLog2e);
        const float nMb = P > 0 ? (float)P * nM1 : ceilf(nm * beta_l2e);
        s1 *= fast_exp2(M1 - nM1);                        // exact power of two <= 1 (0 on the first call)
        sb *= fast_exp2(Mb - nMb);
        M1 = nM1; Mb = nMb; m = nm;
        // offsets of the references from the max, in fp64 so that exp2((x-m)*log2e - c1) = exp(x) / 2^M1 holds to
        // fp32 rounding of the SMALL quantity (x-m), not of the large products x*log2e
        c1 = (float)((double)nM1 - (double)nm * 1.4426950408889634074);
        cb = (float)((double)nMb - (double)nm * (double)beta * 1.4426950408889634074);
        t_max = fmaf(m, kLog2e, -M1);
        set_thr(lower(m - window));
    };

    auto publish = [&]() __attribute__((always_inline)) {                              // let the other waves of the workgroup use this wave's bound
        if (thr > published) {
            if (lane == 0) atomicMax(&wg_bound, enc_bound(thr));
            published = thr;
        }
    };
    auto adopt = [&]() __attribute__((always_inline)) {                                // and take theirs (no waiting: stale is only conservative)
        const int seen = __hip_atomic_load(&wg_bound, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        set_thr(uniform(dec_bound(seen)));
    };

    // the bound that the best key found so far implies: entries below it cannot beat that key
    auto tighten = [&]() __attribute__((always_inline)) {
        float bound = top.a.i >= 0 ? top.a.l + (top.a.g - kGumbelMax - kKeyMargin) / beta : -3.4e38f;
        set_thr(lower(wave_max_f32(bound)));
    };

    // A new running maximum alone only gives the bound "its key is at least beta*m + kGumbelMin".  Drawing the variate of
    // that entry (and, in the same instructions, of every other lane's highest entry of the same vectors) replaces
    // kGumbelMin by the key it really reaches, which raises the bound by a few units of 1/beta at once -- while
    // the stream still runs, so that fewer vectors are queued at all.  Only the bound is kept: the entries are scored
    // again with the rest of their vectors, so no candidate is offered twice.
    auto probe = [&]() __attribute__((always_inline)) {
        // Wave-uniform conditions.  Not before the wave has met a finite entry; not when the bound already lies so far
        // above what this wave holds that only a variate beyond the 1 - e^-8 quantile could raise it; and not when hardly
        // any lane holds an entry near the bound -- then the logits are so thin up there that a somewhat higher bound
        // would spare next to nothing.
        const bool wanted = probe_l >= thr;
        if (m > -3.0e38f && beta * (m - thr) > kGumbelMax - 8.0f && __popcll(__ballot(wanted)) >= 3) {
            float b = -3.4e38f;
            if (wanted) {
                const U4 blk = philox4x32_10(probe_i >> 2, row, step, 0u, key0, key1);
                b = probe_l + (gumbel_f32(pick_word(blk, probe_i & 3u)) - kGumbelMax - kKeyMargin) / beta;
            }
            set_thr(lower(wave_max_f32(b)));
        }
        probe_pending = false;
        probe_l = -INFINITY;
    };

    // Scores the entries of one vector that are at or above `bar`: one Philox block per quad that holds such an entry.
    auto score_vector = [&](const float (&x)[EPV], uint32_t vec_index, float bar) __attribute__((always_inline)) {
#pragma unroll
        for (int q4 = 0; q4 < QPV; ++q4) {
            bool need = false;
#pragma unroll
            for (int j = 0; j < 4; ++j) need = need || x[q4 * 4 + j] >= bar;
            if (need) {
                const U4 blk = philox4x32_10(vec_index * QPV + q4, row, step, 0u, key0, key1);
                const uint32_t wd[4] = {blk.x, blk.y, blk.z, blk.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (x[q4 * 4 + j] >= bar) {
                        top.offer(beta, x[q4 * 4 + j], gumbel_f32(wd[j]), (int32_t)(vec_index * EPV + q4 * 4 + j));
                        ++n_scored;
                    }
                }
            }
        }
    };

    // Scores the first k (<= 64) queued single entries, one per lane, and tightens thr from the keys reached.
    auto score_entries = [&](int k) __attribute__((always_inline)) {
        wave_sync();                                    // ring writes of other lanes, same wave
        if (lane < k) {
            const uint2 ent = ring_ent[(e_head + lane) & (kRingE - 1)];
            const uint32_t idx = ent.x;
            const float xv = __uint_as_float(ent.y);
            if (xv >= thr) {
                const U4 blk = philox4x32_10(idx >> 2, row, step, 0u, key0, key1);
                top.offer(beta, xv, gumbel_f32(pick_word(blk, idx & 3u)), (int32_t)idx);
                ++n_scored;
            }
        }
        e_head = (e_head + k) & (kRingE - 1);
        e_count -= k;
        tighten();
    };

    // Takes up to 64 queued vectors (one per lane) off the ring.  Entries still at or above thr are either scored where
    // they are (many: a flat proposal) or compacted into the entry ring, which is scored whenever it holds a full
    // wave-width.
    auto drain = [&](int n) __attribute__((always_inline)) {
        wave_sync();                                    // ring writes of other lanes, same wave
        float x[EPV];
        uint32_t vi = 0u;
        const bool in = lane < n;
        {
            uint4 raw = make_uint4(kPadWord, kPadWord, kPadWord, kPadWord);
            if (in) {
                const int slot = (q_head + lane) & (kRingV - 1);
                raw = ring_raw[slot];
                vi = ring_idx[slot];
            }
            unpack<DT>(raw, x);
        }
        q_head = (q_head + n) & (kRingV - 1);
        q_count -= n;
        ++n_drains;
        int mine = 0;
#pragma unroll
        for (int j = 0; j < EPV; ++j) mine += x[j] >= thr ? 1 : 0;
        const int total = wave_sum_i32(mine);
        if (total > kScoreAsVectors) {
            if (in) score_vector(x, vi, thr);
            tighten();
        } else if (total > 0) {
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                const bool hit = x[j] >= thr;
                const unsigned long long mk = __ballot(hit);
                if (mk) {                               // wave-uniform
                    if (hit) {
                        const int slot = (e_head + e_count + mask_rank(mk)) & (kRingE - 1);
                        ring_ent[slot] = make_uint2(vi * EPV + j, __float_as_uint(x[j]));
                    }
                    e_count += __popcll(mk);
                    if (e_count >= kWave) score_entries(kWave);
                }
            }
        }
    };

    // Drops queued vectors whose entries have all fallen below thr, keeping the order of the rest.
    auto compact = [&]() __attribute__((always_inline)) {
        wave_sync();
        int kept = 0;
        for (int base = 0; base < q_count; base += kWave) {
            const int src = (q_head + base + lane) & (kRingV - 1);
            const bool in = base + lane < q_count;
            uint4 raw = make_uint4(kPadWord, kPadWord, kPadWord, kPadWord);
            uint32_t vi = 0u;
            if (in) { raw = ring_raw[src]; vi = ring_idx[src]; }
            float x[EPV];
            unpack<DT>(raw, x);
            const bool keep = in && vec_max<DT>(x) >= thr;
            const unsigned long long mk = __ballot(keep);
            wave_sync();                                // all lanes have read this chunk before any lane overwrites it
            if (keep) {
                const int dst = (q_head + kept + mask_rank(mk)) & (kRingV - 1);
                ring_raw[dst] = raw;
                ring_idx[dst] = vi;
            }
            kept += __popcll(mk);
        }
        q_count = kept;
    };

    // Before a batch of the stream: leaves at most half of the vector ring occupied (one copy of the drain code, outside
    // the unrolled loop over the batch's vectors).
    auto make_room = [&]() __attribute__((always_inline)) {
        if (q_count > kRingV / 2) {                     // wave-uniform, rare
            compact();
            while (q_count > kRingV / 2) drain(kWave);
        }
    };

    // both sums from d[j] = x[j] - m (fp32 rows) or t[j] = x[j]*log2e - M1 (bf16 rows); the exponents are <= 0 up to rounding
    auto accumulate = [&](const float (&x)[EPV], const float (&d)[EPV]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const float e = kDirect ? fast_exp2(d[j]) : fast_exp2(fmaf(d[j], kLog2e, -c1));
            s1 += e;
            if constexpr (P > 0) sb += ipow<P>(e);
            else if constexpr (kDirect) sb += fast_exp2(fmaf(x[j], beta_l2e, -Mb));
            else sb += fast_exp2(fmaf(d[j], beta_l2e, -cb));
        }
    };
    auto relative = [&](const float (&x)[EPV], float (&d)[EPV]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < EPV; ++j) d[j] = kDirect ? fmaf(x[j], kLog2e, -M1) : x[j] - m;
    };

    // One vector of the stream: running maximum, filter, sums.  The maximum and the filter work on the relative values
    // (which the sums need anyway); only when some lane holds an entry above the running maximum is the maximum itself formed.
    auto stream_vector = [&](const uint4& raw, int vi, bool in_slice) __attribute__((always_inline)) {
        float x[EPV], d[EPV];
        unpack<DT>(raw, x);
        relative(x, d);
        float dm = vec_max<DT>(d);
        if (__ballot(dm > (kDirect ? t_max : 0.f))) {   // wave-uniform, rare
            const float lx = vec_max<DT>(x);
            const float nm = wave_max_f32(lx);
            if (nm > m) {
                raise_max(nm);
                if constexpr (!DENSE) {
                    probe_pending = true;
                    if (in_slice && lx > probe_l) {
                        int jm = EPV - 1;
#pragma unroll
                        for (int j = EPV - 2; j >= 0; --j) jm = x[j] == lx ? j : jm;
                        probe_l = lx;
                        probe_i = (uint32_t)vi * EPV + (uint32_t)jm;
                    }
                }
            }
            relative(x, d);
            dm = vec_max<DT>(d);
        }
        if constexpr (DENSE) {
            if (in_slice) score_vector(x, (uint32_t)vi, -INFINITY);                  // padding has no index to score
        } else {
            // Scoring is deferred: a vector that holds an entry which may still win is only queued here.  By the
            // time the queue is scored the row's bound is far better than what this wave knows now, and most
            // entries drop out.
            const bool hit = dm >= thr_rel;
            const unsigned long long lanes = __ballot(hit);
            if (lanes) {                                                              // wave-uniform branch
                if (q_count <= kRingV - kWave) {
                    if (hit) {
                        const int slot = (q_head + q_count + mask_rank(lanes)) & (kRingV - 1);
                        ring_raw[slot] = raw;
                        ring_idx[slot] = (uint32_t)vi;
                    }
                    q_count += __popcll(lanes);
                } else {
                    // the ring is full although it was at most half full when the batch began: so many entries may still
                    // win (a flat proposal) that scoring the vector where it is costs no more than queueing it would
                    if (hit) score_vector(x, (uint32_t)vi, thr);
                    tighten();
                }
            }
        }
        accumulate(x, d);
    };

    // The main stream covers the vectors that lie wholly inside the row; the ragged last vector of a row (V not a
    // multiple of the vector width) is handled after it.  A batch that lies wholly inside the slice is loaded without
    // any guard; only the last, partial batch pays for clamped addresses and selects (-inf where there is no vector:
    // such an entry adds 0 to the sums and never passes the filter).
    const int full_end = min(vec_end, nvec_full);
    constexpr int kBatch = THREADS * UNROLL;
    // vector u of the batch that starts at b0; `whole`: the batch lies wholly inside the slice (wave-uniform)
    auto load_vec = [&](int b0, int u, bool whole) __attribute__((always_inline)) -> uint4 {
        const int vi = b0 + u * THREADS + tid;
        if (whole) {
            // every logit is read exactly once: non-temporal loads keep the stream out of the caches
            const vec16 r = __builtin_nontemporal_load((const vec16*)(rowp + (int64_t)vi * 16));
            return make_uint4(r.x, r.y, r.z, r.w);
        }
        const int vc = min(vi, full_end - 1);
        uint4 r = *(const uint4*)(rowp + (int64_t)vc * 16);
        const bool pad = vi >= full_end;
        r.x = pad ? kPadWord : r.x; r.y = pad ? kPadWord : r.y;
        r.z = pad ? kPadWord : r.z; r.w = pad ? kPadWord : r.w;
        return r;
    };

    // Two register sets of UNROLL vectors per thread alternate: while one batch is processed the next is in flight.
    auto load_batch = [&](uint4 (&dst)[UNROLL], int b0) __attribute__((always_inline)) {
        const bool whole = b0 + kBatch <= full_end;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) dst[u] = load_vec(b0, u, whole);
    };
    auto stream_batch = [&](const uint4 (&src)[UNROLL], int b0) __attribute__((always_inline)) {
        if constexpr (!DENSE) { publish(); adopt(); make_room(); }   // no waiting: whatever the other waves have found so far
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int vi = b0 + u * THREADS + tid;
            stream_vector(src[u], vi, vi < full_end);
        }
        if constexpr (!DENSE) { if (probe_pending) probe(); }
    };
    uint4 buf_a[UNROLL], buf_b[UNROLL];
    if (vec_begin < full_end) {
        load_batch(buf_a, vec_begin);
        // warm start: the maximum of the wave's first batch gives a useful threshold at once
        // (vectors past the slice were loaded as -inf and are never the lane's highest)
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float x[EPV];
            unpack<DT>(buf_a[u], x);
            const uint32_t vi = (uint32_t)(vec_begin + u * THREADS + tid);
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                if (x[j] > probe_l) { probe_l = x[j]; probe_i = vi * EPV + (uint32_t)j; }
            }
        }
        const float bm = wave_max_f32(probe_l);
        if (bm > m) raise_max(bm);
        probe_pending = true;                            // drawn once the next batch's loads are on their way
    }
    for (int base = vec_begin; base < full_end; base += 2 * kBatch) {
        const bool second = base + kBatch < full_end;
        if (second) load_batch(buf_b, base + kBatch);
        if constexpr (!DENSE) { if (probe_pending) probe(); }      // (the warm start's: behind the loads just issued)
        stream_batch(buf_a, base);
        if (!second) break;
        if (base + 2 * kBatch < full_end) load_batch(buf_a, base + 2 * kBatch);
        stream_batch(buf_b, base + kBatch);
    }
    if (nvec > nvec_full && vec_end == nvec && wave == 0) {                // the ragged tail: lane 0 of wave 0
        float x[EPV], d[EPV];
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const int v = nvec_full * EPV + j;
            x[j] = (lane == 0 && v < V) ? load_scalar<DT>(rowp, v) : -INFINITY;
        }
        const float vm = vec_max<DT>(x);
        if (__ballot(vm > m)) { const float nm = wave_max_f32(vm); if (nm > m) raise_max(nm); }
        // the few entries past the last full vector are scored where they are (-inf padding never reaches the bar)
        if (lane == 0) score_vector(x, (uint32_t)nvec_full, DENSE ? -3.4e38f : thr);
        relative(x, d);
        accumulate(x, d);
    }
    if constexpr (!DENSE) {
        // No barrier here: a wave that is done streaming scores its queue against the bound as the workgroup knows it
        // now, while slower waves still stream -- a few more entries are scored than with the final bound, but the
        // scoring overlaps with the stream instead of following it.
        tighten(); publish(); adopt();
        while (q_count > 0) {
            if (q_count > kWave) compact();
            if (q_count > 0) { drain(min(q_count, kWave)); publish(); adopt(); }
        }
        if (e_count > 0) score_entries(e_count);
        publish();
    }

    if constexpr (kDirect) {
        // the per-wave part of the error of the fp32 constant log2e (see kDirect above)
        if (m > -3.0e38f) {
            s1 *= fast_exp2((float)((double)m * kLog2eLow));
            sb *= fast_exp2((float)((double)m * (double)beta * kLog2eLow));
        }
    }
    Partial* const slot_out = n_split > 1 ? a.partials + (int64_t)row * kMaxSplit + split : nullptr;
    block_epilogue<NW>(beta, m, M1, Mb, s1, sb, top, n_scored, n_drains, slot_out, &sh_part);
    if (wave != 0) return;

    // ---- tail: the wave that completes the row finalizes it ---------------------------------------------------
    const Partial* pp = &sh_part;
    if (n_split > 1) {
        const int tk = take_ticket(&a.row_ticket[row]);    // this slice's record (written by lane 0) is complete
        if (tk != n_split - 1) return;
        if (lane == 0) store_shared(&a.row_ticket[row], 0);    // nobody else touches it until the next step
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); // (keeps the reads of the records behind the ticket)
        pp = a.partials + (int64_t)row * kMaxSplit;
    } else {
        wave_sync();                                   // lane 0's copy of the record in LDS
    }
    finalize_row(a, sc, row, pp, n_split, row_state);
    after_row_final(a, sc, row, lds);
}

// ------------------------------------------------------------------------------------------------
template <int DT, bool DENSE, int NW>
static hipError_t launch_k1(smc_ctx* c, const StepArgs& a, int P)
{
    const dim3 grid((unsigned)(c->R * a.n_split)), block(NW * kWave);
#define PSMC_LAUNCH(PP) hipLaunchKernelGGL((vocab_pass_kernel<DT, PP, DENSE, NW>), grid, block, 0, c->stream, a)
    if constexpr (DENSE) {                              // the cross-check instantiation: generic exponent only
        PSMC_LAUNCH(0);
    } else {
        switch (P) {
            case 1: PSMC_LAUNCH(1); break;
            case 2: PSMC_LAUNCH(2); break;
            case 3: PSMC_LAUNCH(3); break;
            case 4: PSMC_LAUNCH(4); break;
            case 5: PSMC_LAUNCH(5); break;
            case 6: PSMC_LAUNCH(6); break;
            case 8: PSMC_LAUNCH(8); break;
            default: PSMC_LAUNCH(0); break;
        }
    }
#undef PSMC_LAUNCH
    return hipGetLastError();
}


// One logits dtype: picks the instantiation for the workgroup size, the dense / lazy variant and the exponent.
template <int DT>
static hipError_t launch_vocab_dt(smc_ctx* c, const StepArgs& a, int P)
{
    const int nw = c->wg_waves;
    if (c->dense)
        return nw == 16 ? launch_k1<DT, true, 16>(c, a, P) : nw == 8 ? launch_k1<DT, true, 8>(c, a, P) : launch_k1<DT, true, 4>(c, a, P);
    return nw == 16 ? launch_k1<DT, false, 16>(c, a, P) : nw == 8 ? launch_k1<DT, false, 8>(c, a, P) : launch_k1<DT, false, 4>(c, a, P);
}

}  // namespace psmc
