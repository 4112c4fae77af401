// Vocabulary pass of the Power-SMC step (Alg. 1 "sample" and "update"; Eq. "inc"; Cor. 1) for gfx950.
//
// One read of every logit of every row produces, per row:
//   log Z_1 = LSE_v(l_v), log Z_beta = LSE_v(beta l_v), and the Gumbel-max draw argmax_v(beta l_v + g_v),
// from which the row finalizer forms log p(y), log q(y) and the increment alpha log p(y) - log q(y).
//
// The work is HBM-bound streaming; there is no contraction here, hence no MFMA.  A row is split over
// n_split workgroups of 256 or 1024 threads; every thread streams 16-byte vectors.  The two sums are kept per lane
// against a wave-uniform power-of-two reference, so a rising running maximum rescales them exactly.
//
// Exact lazy Gumbel-max: g is bounded, g in [kGumbelMin, kGumbelMax].  An entry whose best possible key
// beta*l_v + kGumbelMax is below a key that some entry is already known to reach cannot be the argmax, so it
// draws no random number.  The threshold on l_v ("thr") only ever rises; it comes from the wave's running maximum,
// from keys already scored, and from one LDS word per workgroup that all its waves raise with an LDS atomic max
// and read without waiting -- a stale value only makes the filter more conservative, never wrong.  Entries at or
// above thr are compacted (ballot + mbcnt) into a per-wave LDS ring; scoring is deferred to the end of the slice,
// when the bound is known best, and runs 64 entries at a time with Philox.  The result is the same argmax as
// scoring every entry.  The "dense" instantiation scores every entry in place.
#include "device_rng.hpp"
#include "smc_internal.hpp"

namespace psmc {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

typedef unsigned int vec16 __attribute__((ext_vector_type(4)));    // one 16-byte global load

template <int DT> struct Elems;
template <> struct Elems<SMC_BF16> { static constexpr int kPerVec = 8; using Scalar = uint16_t; };
template <> struct Elems<SMC_F32>  { static constexpr int kPerVec = 4; using Scalar = float; };

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
// are merged and written as this slice's Partial.  m_wave is the wave's reference for comparing keys across lanes.
template <int NW>
__device__ __forceinline__ void block_epilogue(float beta, float m_wave, float M1, float Mb, float s1, float sb,
                                               const LaneTop2 top, unsigned long long n_scored,
                                               unsigned long long n_drains, Partial* __restrict__ out)
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
        unsigned long long sc = n_scored;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sc += __shfl_xor(sc, o);
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
        uint32_t nsc = hw ? red_n[lane][0] : 0u, ndr = hw ? red_n[lane][1] : 0u;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) { nsc += __shfl_xor(nsc, o); ndr += __shfl_xor(ndr, o); }
        // candidates: lane c < 2*NW holds candidate (c & 1) of wave (c >> 1)
        const bool hc = lane < 2 * NW;
        const float cl = hc ? red_cl[lane >> 1][lane & 1] : 0.f, cg = hc ? red_cg[lane >> 1][lane & 1] : 0.f;
        const int32_t ci = hc ? red_ci[lane >> 1][lane & 1] : -1;
        const float key = fmaf(beta, cl - gm, cg);
        int lb, l2; bool sec_b;
        wave_best_two(key, NEG, ci >= 0, lb, l2, sec_b);
        const int sb_lane = lb < 0 ? 0 : lb, s2_lane = (l2 < 0 || sec_b) ? 0 : l2;
        const float l1v = __shfl(cl, sb_lane), g1v = __shfl(cg, sb_lane); const int32_t i1v = __shfl(ci, sb_lane);
        const float l2v = __shfl(cl, s2_lane), g2v = __shfl(cg, s2_lane); const int32_t i2v = __shfl(ci, s2_lane);
        if (lane == 0) {
            Partial p;
            p.M1 = gM1; p.s1 = t1; p.Mb = gMb; p.sb = tb;
            p.l1 = l1v; p.g1 = g1v; p.i1 = lb < 0 ? -1 : i1v;
            p.l2 = l2v; p.g2 = g2v; p.i2 = (l2 < 0 || sec_b) ? -1 : i2v;
            p.n_scored = (int32_t)nsc; p.n_drains = (int32_t)ndr;
            *out = p;
        }
    }
}

// order-preserving map float -> int for atomicMax on a shared lower bound
__device__ __forceinline__ int enc_bound(float f) { const int i = __float_as_int(f); return i >= 0 ? i : i ^ 0x7FFFFFFF; }
__device__ __forceinline__ float dec_bound(int i) { return __int_as_float(i >= 0 ? i : i ^ 0x7FFFFFFF); }

}  // namespace

// P > 0: beta is the integer P (sum of e^P by multiplication); P == 0: generic beta (second exp2).
// DENSE: every entry is scored in place (no filter, no ring) -- the plain definition, kept for cross-checks.
// NW: waves per workgroup (4 or 16).
template <int DT, int P, bool DENSE, int NW>
__global__ __launch_bounds__(NW * kWave, 4) void vocab_pass_kernel(
    const void* __restrict__ logits, int64_t row_stride_bytes, int V, float beta, uint32_t key0, uint32_t key1,
    uint32_t step, int n_split, int vecs_per_split, Partial* __restrict__ partials, const int32_t* __restrict__ done)
{
    constexpr int EPV = Elems<DT>::kPerVec;
    constexpr int UNROLL = 4;                          // 16-byte vectors per thread and batch (two batches in flight)
    constexpr int THREADS = NW * kWave;
    constexpr int kRing = 1024;                        // candidate ring entries per wave (power of two)
    static_assert(kRing >= 2 * EPV * kWave, "a full vector of candidates must fit beside a partly filled ring");
    // Queueing costs ~6 ps per queued entry, scoring a vector in place ~1.4 ps per entry whatever its content
    // (measured on 2048 bf16 rows), so the two meet where a little under a quarter of the entries qualify, i.e.
    // where a lane's EPV entries include a qualifying one with probability 1 - 0.77^EPV.  A vector with at least
    // this many such lanes is scored in place.  (Deciding once per batch of vectors instead was tried: the
    // threshold rises fast at the start of a slice and the stale decision cost more than the test.)
    constexpr int kScoreInPlace = EPV == 8 ? 56 : 42;
    __shared__ uint2 ring[DENSE ? 1 : NW][DENSE ? 1 : kRing];     // (vocabulary index, logit bits)
    __shared__ int wg_bound;                           // best "cannot win below this" bound of the whole workgroup

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x % n_split;
    const uint32_t row = blockIdx.x / n_split;
    const char* rowp = (const char*)logits + (int64_t)row * row_stride_bytes;
    if (done && done[row]) return;                     // terminated particle (App. D): its logits are not read
    if (tid == 0) wg_bound = enc_bound(-INFINITY);
    __syncthreads();

    const int nvec_full = V / EPV;                      // vectors wholly inside the row
    const int nvec = (V + EPV - 1) / EPV;
    const int vec_begin = split * vecs_per_split;
    const int vec_end = min(vec_begin + vecs_per_split, nvec);

    const float beta_l2e = beta * kLog2e;
    const float window = (kGumbelMax - kGumbelMin + kKeyMargin) / beta;   // in logit units

    // wave-uniform running state
    float m = -3.0e38f;            // running max of the logits seen by this wave
    float M1 = -INFINITY, Mb = -INFINITY;   // power-of-two references (integers): M1 >= m*log2e, Mb >= m*beta*log2e
    float thr = -3.4e38f;          // entries below thr cannot win
    float published = -3.4e38f;    // what this wave last wrote to the row's shared bound
    float c1 = 0.f, cb = 0.f;      // c1 = M1 - m*log2e, cb = Mb - m*beta*log2e, both >= 0
    float s1 = 0.f, sb = 0.f;      // per-lane sums relative to the references
    int q_head = 0, q_count = 0;
    unsigned long long n_scored = 0, n_drains = 0;
    LaneTop2 top; top.init();

    auto lower = [](float b) { return b - fabsf(b) * 4e-7f; };    // a few ulps down: never drop a possible winner

    auto raise_max = [&](float nm) {                    // nm > m, wave-uniform
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
        thr = fmaxf(thr, lower(m - window));
    };

    auto publish = [&]() {                              // let the other waves of the workgroup use this wave's bound
        if (thr > published) {
            if (lane == 0) atomicMax(&wg_bound, enc_bound(thr));
            published = thr;
        }
    };
    auto adopt = [&]() {                                // and take theirs (no waiting: stale is only conservative)
        const int seen = __hip_atomic_load(&wg_bound, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        thr = fmaxf(thr, uniform(dec_bound(seen)));
    };

    // Scores up to 64 ring entries (those still at or above thr) and tightens thr from the keys reached.
    auto drain = [&](int n) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // ring writes of other lanes, same wave
        __builtin_amdgcn_wave_barrier();
        if (lane < n) {
            const int slot = (q_head + lane) & (kRing - 1);
            const uint2 ent = ring[DENSE ? 0 : wave][slot];
            const uint32_t idx = ent.x;
            const float xv = __uint_as_float(ent.y);
            if (xv >= thr) {
                const U4 blk = philox4x32_10(idx >> 2, row, step, 0u, key0, key1);
                top.offer(beta, xv, gumbel_f32(pick_word(blk, idx & 3u)), (int32_t)idx);
                ++n_scored;
            }
        }
        q_head = (q_head + n) & (kRing - 1);
        q_count -= n;
        ++n_drains;
        float bound = top.a.i >= 0 ? top.a.l + (top.a.g - kGumbelMax - kKeyMargin) / beta : -3.4e38f;
        bound = uniform(wave_max_f32(bound));
        thr = fmaxf(thr, lower(bound));
    };

    // Drops ring entries that have fallen below thr, keeping the order of the rest.
    auto compact = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        int kept = 0;
        for (int base = 0; base < q_count; base += kWave) {
            const int src = (q_head + base + lane) & (kRing - 1);
            const bool in = base + lane < q_count;
            const uint2 ent = in ? ring[DENSE ? 0 : wave][src] : make_uint2(0u, 0u);
            const bool keep = in && __uint_as_float(ent.y) >= thr;
            const unsigned long long mk = __ballot(keep);
            __builtin_amdgcn_wave_barrier();            // all lanes have read this chunk before any lane overwrites it
            if (keep) {
                const int dst = (q_head + kept + mask_rank(mk)) & (kRing - 1);
                ring[DENSE ? 0 : wave][dst] = ent;
            }
            kept += __popcll(mk);
        }
        q_count = kept;
    };

    auto process = [&](const float (&x)[EPV], int v0) {
        if constexpr (DENSE) {
            float vm = x[0];
#pragma unroll
            for (int j = 1; j < EPV; ++j) vm = fmaxf(vm, x[j]);
            if (__ballot(vm > m)) { const float nm = wave_max_f32(vm); if (nm > m) raise_max(nm); }
#pragma unroll
            for (int q4 = 0; q4 < EPV / 4; ++q4) {
                const U4 blk = philox4x32_10((uint32_t)(v0 >> 2) + q4, row, step, 0u, key0, key1);
                const uint32_t wd[4] = {blk.x, blk.y, blk.z, blk.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int v = v0 + q4 * 4 + j;
                    if (v < V) top.offer(beta, x[q4 * 4 + j], gumbel_f32(wd[j]), v);
                }
            }
        } else {
            // Scoring is deferred: entries that may still win are only queued here.  By the time the queue is
            // scored the row's bound is far better than what this wave knows now, and most entries drop out.
            if (q_count > kRing - EPV * kWave) {                             // rare: make room for one more vector
                compact();
                while (q_count > kRing - EPV * kWave) drain(min(q_count, kWave));
            }
            // the running maximum first (the sums below need x <= m); thr may sit above m when another wave of the
            // workgroup has seen a larger logit
            float vm = x[0];
#pragma unroll
            for (int j = 1; j < EPV; ++j) vm = fmaxf(vm, x[j]);
            if (__ballot(vm > m)) raise_max(wave_max_f32(vm));
            const unsigned long long lanes = __ballot(vm >= thr);           // lanes that hold a qualifying entry
            if (lanes == 0ull) {
                // nothing in this vector can win: the common case once the threshold has risen
            } else if (__popcll(lanes) >= kScoreInPlace) {                  // wave-uniform
                // So many entries may still win (a flat proposal: small beta, or logits that differ little) that
                // queueing them one by one costs more than scoring the vector where it is, four entries per
                // Philox block.
#pragma unroll
                for (int q4 = 0; q4 < EPV / 4; ++q4) {
                    bool need = false;
#pragma unroll
                    for (int j = 0; j < 4; ++j) need = need || x[q4 * 4 + j] >= thr;
                    if (need) {
                        const U4 blk = philox4x32_10((uint32_t)(v0 >> 2) + q4, row, step, 0u, key0, key1);
                        const uint32_t wd[4] = {blk.x, blk.y, blk.z, blk.w};
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (x[q4 * 4 + j] >= thr) {
                                top.offer(beta, x[q4 * 4 + j], gumbel_f32(wd[j]), v0 + q4 * 4 + j);
                                ++n_scored;
                            }
                        }
                    }
                }
                float bound = top.a.i >= 0 ? top.a.l + (top.a.g - kGumbelMax - kKeyMargin) / beta : -3.4e38f;
                bound = uniform(wave_max_f32(bound));
                thr = fmaxf(thr, lower(bound));
            } else {
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    const bool hit = x[j] >= thr;
                    const unsigned long long mk = __ballot(hit);
                    if (mk) {                                               // wave-uniform
                        if (hit) {
                            const int slot = (q_head + q_count + mask_rank(mk)) & (kRing - 1);
                            ring[wave][slot] = make_uint2((uint32_t)(v0 + j), __float_as_uint(x[j]));
                        }
                        q_count += __popcll(mk);
                    }
                }
            }
        }
        // both sums; every x[j] <= m here, so the exponents are <= 0
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const float d = x[j] - m;
            const float e = fast_exp2(fmaf(d, kLog2e, -c1));
            s1 += e;
            if constexpr (P > 0) sb += ipow<P>(e);
            else sb += fast_exp2(fmaf(d, beta_l2e, -cb));
        }
    };

    // The main stream covers the vectors that lie wholly inside the row; the ragged last vector of a row (V not a
    // multiple of the vector width) is handled after it.  Loads are unconditional (clamped address + select) so that
    // the loop has no divergent branch around a load and the next batch really stays in flight.
    constexpr uint32_t kPadWord = DT == SMC_BF16 ? 0xFF80FF80u : 0xFF800000u;      // -inf in every element
    const int full_end = min(vec_end, nvec_full);
    constexpr int kBatch = THREADS * UNROLL;
    // A batch that lies wholly inside the slice is loaded without any guard; only the last, partial batch pays for
    // clamped addresses and selects (which consume the loaded words at once and so cannot stay in flight).
    auto load_batch = [&](uint4 (&dst)[UNROLL], int b0) {
        if (b0 + kBatch <= full_end) {                                     // uniform
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                // every logit is read exactly once: non-temporal loads keep the stream out of the caches
                const vec16 r = __builtin_nontemporal_load((const vec16*)(rowp + (int64_t)(b0 + u * THREADS + tid) * 16));
                dst[u] = make_uint4(r.x, r.y, r.z, r.w);
            }
        } else {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int vi = b0 + u * THREADS + tid;
                const int vc = min(vi, full_end - 1);
                uint4 r = *(const uint4*)(rowp + (int64_t)vc * 16);
                const bool pad = vi >= full_end;
                r.x = pad ? kPadWord : r.x; r.y = pad ? kPadWord : r.y;
                r.z = pad ? kPadWord : r.z; r.w = pad ? kPadWord : r.w;
                dst[u] = r;
            }
        }
    };

    // while one batch of UNROLL vectors per thread is processed the next is already in flight
    uint4 cur[UNROLL], nxt[UNROLL];
    if (vec_begin < full_end) load_batch(cur, vec_begin);
    bool first = true;
    for (int base = vec_begin; base < full_end; base += kBatch) {
        if (base + kBatch < full_end) load_batch(nxt, base + kBatch);
        if (first) {                 // warm start: the max of the workgroup's first batch gives a useful threshold
            first = false;
            float vm = -INFINITY;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float x[EPV];
                unpack<DT>(cur[u], x);
#pragma unroll
                for (int j = 0; j < EPV; ++j) vm = fmaxf(vm, x[j]);
            }
            vm = wave_max_f32(vm);
            if (vm > m) raise_max(vm);
            if constexpr (!DENSE) { publish(); adopt(); }      // no waiting: whatever the other waves have found so far
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (base + u * THREADS + (wave << 6) < full_end) {             // wave-uniform: wave has data
                float x[EPV];
                unpack<DT>(cur[u], x);
                process(x, (base + u * THREADS + tid) * EPV);
            }
        }
        if constexpr (!DENSE) { publish(); adopt(); }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) cur[u] = nxt[u];
    }
    if (nvec > nvec_full && vec_end == nvec && wave == 0) {                // the ragged tail: lane 0 of wave 0
        float x[EPV];
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const int v = nvec_full * EPV + j;
            x[j] = (lane == 0 && v < V) ? load_scalar<DT>(rowp, v) : -INFINITY;
        }
        process(x, nvec_full * EPV);
    }
    if constexpr (!DENSE) {
        // every wave has streamed its share: the workgroup's bound now reflects the maximum of the whole slice
        __syncthreads();
        adopt();
        while (q_count > 0) {
            compact();
            if (q_count > 0) { drain(min(q_count, kWave)); publish(); adopt(); }
        }
    }

    block_epilogue<NW>(beta, m, M1, Mb, s1, sb, top, n_scored, n_drains, partials + (int64_t)row * kMaxSplit + split);
}

// ------------------------------------------------------------------------------------------------
// Row finalizer (a0 + a2): one wave per row.  Merges the row's partials in fp64, re-ranks the finalists of the
// Gumbel-max draw with fp64 keys beta*l + g (ties to the lower index), then applies the boundary reweight of
// exponent bridging (Sec. 5.3) and the increment alpha*log p(y) - log q(y) (Eq. "inc").
template <int DT>
__global__ __launch_bounds__(kWave) void finalize_rows_kernel(
    const void* __restrict__ logits, int64_t row_stride_bytes, int V, int N, double beta, double alpha_t,
    double alpha_prev, uint32_t key0, uint32_t key1, uint32_t step, int n_split, const Partial* __restrict__ partials,
    double* __restrict__ logW, double* __restrict__ cumlogp, const int32_t* __restrict__ parity,
    int32_t* const* __restrict__ histAB, int T_max, int32_t* __restrict__ tokens_out, double* __restrict__ d_delta,
    double* __restrict__ d_logZ1, double* __restrict__ d_logZb, double* __restrict__ d_gap,
    int32_t* __restrict__ d_second, int32_t* __restrict__ d_rowstat, int eos_id, int32_t* __restrict__ done)
{
    const int lane = threadIdx.x;
    const uint32_t row = blockIdx.x;
    if (eos_id >= 0 && done[row]) {                    // absorbing state (Alg. 1 "if done"; App. D): y_t = EOS, increment 1;
        if (lane == 0) {                               // the stage-boundary reweight still re-targets its prefix (App. B)
            logW[row] += (alpha_t - alpha_prev) * cumlogp[row];
            tokens_out[row] = eos_id;
            if (histAB) {
                int32_t* h = histAB[parity[row]];
                if (h) h[(int64_t)row * T_max + (step - 1)] = eos_id;
            }
            d_delta[row] = 0.0; d_logZ1[row] = 0.0; d_logZb[row] = 0.0; d_gap[row] = INFINITY; d_second[row] = -1;
            d_rowstat[3 * row] = 0; d_rowstat[3 * row + 1] = 0; d_rowstat[3 * row + 2] = 0;
        }
        return;
    }
    const Partial* pp = partials + (int64_t)row * kMaxSplit;

    // sums
    double M1 = -1e300, Mb = -1e300, s1 = 0.0, sb = 0.0;
    if (lane < n_split) { M1 = pp[lane].M1; Mb = pp[lane].Mb; s1 = pp[lane].s1; sb = pp[lane].sb; }
    const double gM1 = wave_max_f64(M1), gMb = wave_max_f64(Mb);
    const double S1 = wave_sum_f64(lane < n_split ? s1 * exp2(M1 - gM1) : 0.0);
    const double Sb = wave_sum_f64(lane < n_split ? sb * exp2(Mb - gMb) : 0.0);
    constexpr double LN2 = 0.69314718055994530942;
    const double logZ1 = gM1 * LN2 + log(S1);
    const double logZb = gMb * LN2 + log(Sb);

    int32_t nsc = 0, ndr = 0;
    if (lane < n_split) { nsc = pp[lane].n_scored; ndr = pp[lane].n_drains; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { nsc += __shfl_xor(nsc, o); ndr += __shfl_xor(ndr, o); }

    // finalists: lane c -> candidate (c & 1) of split (c >> 1)
    int32_t idx = -1;
    if (lane < 2 * n_split) idx = (lane & 1) ? pp[lane >> 1].i2 : pp[lane >> 1].i1;
    if (idx >= V) idx = -1;                            // never read outside the row, whatever the partial holds
    double key = -INFINITY, lv = 0.0;
    if (idx >= 0) {
        // the finalist's logit travels in the partial record (an exact copy: bf16 and fp32 both fit a float), so no
        // second, dependent read of the logits is needed here
        lv = (double)((lane & 1) ? pp[lane >> 1].l2 : pp[lane >> 1].l1);
        const U4 blk = philox4x32_10((uint32_t)idx >> 2, row, step, 0u, key0, key1);
        key = beta * lv + gumbel_f64(pick_word(blk, (uint32_t)idx & 3u));
    }
    // winner: max key, lowest index among equals
    const double k1 = wave_max_f64(key);
    int32_t cand = (idx >= 0 && key == k1) ? idx : 0x7FFFFFFF;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cand = min(cand, __shfl_xor(cand, o));
    const int32_t y = cand;
    const double key2v = (idx >= 0 && idx != y) ? key : -INFINITY;
    const double k2 = wave_max_f64(key2v);
    int32_t cand2 = (idx >= 0 && idx != y && key == k2) ? idx : 0x7FFFFFFF;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cand2 = min(cand2, __shfl_xor(cand2, o));
    const unsigned long long ymask = __ballot(idx == y);
    const int ylane = __ffsll((long long)ymask) - 1;
    const double ly = __shfl(lv, ylane < 0 ? 0 : ylane);

    if (lane == 0) {
        const bool ok = (y != 0x7FFFFFFF) && isfinite(logZ1) && isfinite(logZb);
        const int32_t tok = ok ? y : 0;
        const double logp = ly - logZ1;
        const double logq = beta * ly - logZb;
        const double delta = alpha_t * logp - logq;
        double w = logW[row] + (alpha_t - alpha_prev) * cumlogp[row];      // stage boundary on the prefix y_{1:t-1}
        w += delta;
        logW[row] = w;
        cumlogp[row] += logp;
        tokens_out[row] = tok;
        if (histAB) {
            int32_t* h = histAB[parity[row]];
            if (h) h[(int64_t)row * T_max + (step - 1)] = tok;
        }
        d_delta[row] = delta; d_logZ1[row] = logZ1; d_logZb[row] = logZb;
        d_gap[row] = k1 - k2;
        d_second[row] = cand2 == 0x7FFFFFFF ? -1 : cand2;
        d_rowstat[3 * row] = ok ? 0 : 1; d_rowstat[3 * row + 1] = nsc; d_rowstat[3 * row + 2] = ndr;
        if (eos_id >= 0 && ok && tok == eos_id) done[row] = 1;
    }
}

// ------------------------------------------------------------------------------------------------
template <int DT, bool DENSE, int NW>
static hipError_t launch_k1(smc_ctx* c, const void* logits, int64_t row_stride_bytes, int t, float betaf,
                            int n_split, int vecs_per_split)
{
    const dim3 grid((unsigned)(c->R * n_split)), block(NW * kWave);
    const uint32_t k0 = (uint32_t)c->cfg.seed, k1 = (uint32_t)(c->cfg.seed >> 32);
    const int V = c->cfg.V;
    Partial* pa = c->ws.partials;
    const int32_t* dn = c->cfg.eos_id >= 0 ? c->ws.done : nullptr;
    int P = 0;
    if (betaf == floorf(betaf) && betaf >= 1.f && betaf <= 8.f && betaf != 7.f) P = (int)betaf;
#define PSMC_LAUNCH(PP) hipLaunchKernelGGL((vocab_pass_kernel<DT, PP, DENSE, NW>), grid, block, 0, c->stream, logits, \
                                           row_stride_bytes, V, betaf, k0, k1, (uint32_t)t, n_split, vecs_per_split, pa, dn)
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
#undef PSMC_LAUNCH
    return hipGetLastError();
}

hipError_t launch_vocab_pass(smc_ctx* c, const void* logits, int64_t row_stride, int t, double alpha_t,
                             double alpha_prev, double beta, int32_t* tokens_out)
{
    const int dt = c->cfg.logits_dtype;
    const int esz = dt == SMC_BF16 ? 2 : 4;
    const int epv = 16 / esz;
    const int64_t row_stride_bytes = row_stride * esz;
    const int nvec = (c->cfg.V + epv - 1) / epv;
    // workgroup size: 16 waves when there are few rows (the waves of a workgroup share their bound through LDS),
    // 4 waves when rows alone fill the chip
    const int nw = c->wg_waves;
    const int threads = nw * kWave;
    // split a row into n_split contiguous runs of vectors
    int n_split = c->n_split;
    const int tiles = (nvec + threads - 1) / threads;
    if (n_split > tiles) n_split = tiles;
    // equal shares at vector granularity (whole wave-widths), so that no slice of a row is a tile longer than another
    int vecs_per_split = (nvec + n_split - 1) / n_split;
    vecs_per_split = (vecs_per_split + kWave - 1) / kWave * kWave;
    n_split = (nvec + vecs_per_split - 1) / vecs_per_split;

    hipError_t e;
    const float betaf = (float)beta;
    {
        ScopedKernelTimer timer(c, 0);
#define PSMC_GO(DT, DENSE)                                                                                  \
    (nw == 16 ? launch_k1<DT, DENSE, 16>(c, logits, row_stride_bytes, t, betaf, n_split, vecs_per_split)    \
              : launch_k1<DT, DENSE, 4>(c, logits, row_stride_bytes, t, betaf, n_split, vecs_per_split))
        if (dt == SMC_BF16) e = c->dense ? PSMC_GO(SMC_BF16, true) : PSMC_GO(SMC_BF16, false);
        else e = c->dense ? PSMC_GO(SMC_F32, true) : PSMC_GO(SMC_F32, false);
#undef PSMC_GO
    }
    if (e != hipSuccess) return e;

    const uint32_t k0 = (uint32_t)c->cfg.seed, k1 = (uint32_t)(c->cfg.seed >> 32);
    int32_t* const* hist = c->hist_bound ? (int32_t* const*)c->ws.histAB : nullptr;
    auto& w = c->ws;
    if (dt == SMC_BF16)
        hipLaunchKernelGGL((finalize_rows_kernel<SMC_BF16>), dim3(c->R), dim3(kWave), 0, c->stream, logits,
                           row_stride_bytes, c->cfg.V, c->cfg.N, beta, alpha_t, alpha_prev, k0, k1, (uint32_t)t, n_split,
                           w.partials, w.logW, w.cumlogp, w.parity, hist, c->cfg.T_max, tokens_out, w.d_delta,
                           w.d_logZ1, w.d_logZb, w.d_gap, w.d_second, w.d_rowstat, c->cfg.eos_id, w.done);
    else
        hipLaunchKernelGGL((finalize_rows_kernel<SMC_F32>), dim3(c->R), dim3(kWave), 0, c->stream, logits,
                           row_stride_bytes, c->cfg.V, c->cfg.N, beta, alpha_t, alpha_prev, k0, k1, (uint32_t)t, n_split,
                           w.partials, w.logW, w.cumlogp, w.parity, hist, c->cfg.T_max, tokens_out, w.d_delta,
                           w.d_logZ1, w.d_logZb, w.d_gap, w.d_second, w.d_rowstat, c->cfg.eos_id, w.done);
    return hipGetLastError();
}

}  // namespace psmc
