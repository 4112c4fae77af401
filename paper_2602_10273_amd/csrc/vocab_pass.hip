// Vocabulary pass of the Power-SMC step (Alg. 1 "sample" and "update"; Eq. "inc"; Cor. 1) for gfx950.
//
// One read of every logit of every row produces, per row:
//   log Z_1 = LSE_v(l_v), log Z_beta = LSE_v(beta l_v), and the Gumbel-max draw argmax_v(beta l_v + g_v),
// from which the row finalizer forms log p(y), log q(y) and the increment alpha log p(y) - log q(y).
//
// The work is HBM-bound streaming; there is no contraction here, hence no MFMA.  A row is split over
// n_split workgroups of 256 threads; every thread streams 16-byte vectors.  The two sums are kept per lane
// against a wave-uniform power-of-two reference, so a rising running maximum rescales them exactly.
//
// Exact lazy Gumbel-max: g is bounded, g in [kGumbelMin, kGumbelMax].  An entry whose best possible key
// beta*l_v + kGumbelMax is below a key that some entry is already known to reach cannot be the argmax, so it
// draws no random number.  The threshold on l_v ("thr") only ever rises.  Entries at or above it are compacted
// (ballot + mbcnt) into a per-wave LDS ring and scored 64 at a time with Philox.  The result is the same
// argmax as scoring every entry.  The "dense" instantiation scores every entry in place.
#include "device_rng.hpp"
#include "smc_internal.hpp"

namespace psmc {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kRing = 128;                     // entries per wave ring (count stays below 128: drained at >= 64)

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

}  // namespace

// P > 0: beta is the integer P (sum of e^P by multiplication); P == 0: generic beta (second exp2).
template <int DT, int P, bool DENSE>
__global__ __launch_bounds__(kVocabThreads) void vocab_pass_kernel(
    const void* __restrict__ logits, int64_t row_stride_bytes, int V, float beta, uint32_t key0, uint32_t key1,
    uint32_t step, int n_split, int vecs_per_split, Partial* __restrict__ partials, Counters* __restrict__ counters)
{
    constexpr int EPV = Elems<DT>::kPerVec;
    constexpr int UNROLL = 4;
    __shared__ uint32_t ring_idx[kVocabThreads / kWave][kRing];
    __shared__ float ring_val[kVocabThreads / kWave][kRing];
    __shared__ float red_f[kVocabThreads / kWave][4];
    __shared__ Cand red_c[kVocabThreads / kWave][2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x % n_split;
    const uint32_t row = blockIdx.x / n_split;
    const char* rowp = (const char*)logits + (int64_t)row * row_stride_bytes;

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
    float c1 = 0.f, cb = 0.f;      // c1 = M1 - m*log2e, cb = Mb - m*beta*log2e, both >= 0
    float s1 = 0.f, sb = 0.f;      // per-lane sums relative to the references
    int q_head = 0, q_count = 0;
    unsigned long long n_scored = 0, n_drains = 0;
    LaneTop2 top; top.init();

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
        const float bound = m - window;
        thr = fmaxf(thr, bound - fabsf(bound) * 4e-7f);   // a few ulps down: the test must never drop a possible winner
    };

    auto score = [&](uint32_t idx, float xv) {          // one candidate on this lane
        const U4 blk = philox4x32_10(idx >> 2, row, step, 0u, key0, key1);
        const float g = gumbel_f32(pick_word(blk, idx & 3u));
        top.offer(beta, xv, g, (int32_t)idx);
    };

    auto tighten = [&]() {                              // raise thr from the keys reached so far
        float bound = top.a.i >= 0 ? top.a.l + (top.a.g - kGumbelMax - kKeyMargin) / beta : -3.4e38f;
        bound = uniform(wave_max_f32(bound));
        thr = fmaxf(thr, bound - fabsf(bound) * 4e-7f);
    };

    auto drain = [&](int n) {                           // score n <= 64 ring entries
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // ring writes of other lanes, same wave
        __builtin_amdgcn_wave_barrier();
        if (lane < n) {
            const int slot = (q_head + lane) & (kRing - 1);
            const uint32_t idx = ring_idx[wave][slot];
            const float xv = ring_val[wave][slot];
            if (xv >= thr) { score(idx, xv); ++n_scored; }
        }
        q_head = (q_head + n) & (kRing - 1);
        q_count -= n;
        ++n_drains;
        tighten();
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
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                const bool hit = x[j] >= thr;
                const unsigned long long mk = __ballot(hit);
                if (mk) {                                                   // wave-uniform
                    if (__ballot(x[j] > m)) {
                        const float nm = wave_max_f32(x[j]);
                        raise_max(nm);
                    }
                    // re-test against the possibly raised threshold, then compact into the ring
                    const bool keep = x[j] >= thr;
                    const unsigned long long mk2 = __ballot(keep);
                    if (keep) {
                        const int slot = (q_head + q_count + mask_rank(mk2)) & (kRing - 1);
                        ring_idx[wave][slot] = (uint32_t)(v0 + j);
                        ring_val[wave][slot] = x[j];
                    }
                    q_count += __popcll(mk2);
                    if (q_count >= kWave) drain(kWave);
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

    auto load_vec = [&](int vi, float (&x)[EPV]) {
        const int v0 = vi * EPV;
        if (vi < nvec_full) {
            const uint4 raw = *(const uint4*)(rowp + (int64_t)vi * 16);
            unpack<DT>(raw, x);
        } else {
#pragma unroll
            for (int j = 0; j < EPV; ++j)
                x[j] = (vi < nvec && v0 + j < V) ? load_scalar<DT>(rowp, v0 + j) : -INFINITY;
        }
    };

    // main stream: UNROLL vectors per thread in flight
    bool first = true;
    for (int base = vec_begin; base < vec_end; base += kVocabThreads * UNROLL) {
        float x[UNROLL][EPV];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int vi = base + u * kVocabThreads + tid;
            if (vi < vec_end) load_vec(vi, x[u]);
            else {
#pragma unroll
                for (int j = 0; j < EPV; ++j) x[u][j] = -INFINITY;
            }
        }
        if (first) {                 // warm start: the max of the first vectors gives a useful threshold at once
            first = false;
            float vm = -INFINITY;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int j = 0; j < EPV; ++j) vm = fmaxf(vm, x[u][j]);
            vm = wave_max_f32(vm);
            if (vm > m) raise_max(vm);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (base + u * kVocabThreads + (wave << 6) < vec_end)          // wave-uniform: wave has data
                process(x[u], (base + u * kVocabThreads + tid) * EPV);
        }
    }
    if constexpr (!DENSE) {
        while (q_count > 0) drain(min(q_count, kWave));
    }

    // ---- wave summary
    s1 = wave_sum_f32(s1);
    sb = wave_sum_f32(sb);
    // wave top-2 by fp32 key relative to the wave max
    const float NEG = -3.4e38f;
    const float ka = top.a.i >= 0 ? fmaf(beta, top.a.l - m, top.a.g) : NEG;
    const float kb = top.b.i >= 0 ? fmaf(beta, top.b.l - m, top.b.g) : NEG;
    const float best = wave_max_f32(ka);
    const unsigned long long who = __ballot(ka == best && top.a.i >= 0);
    const int wlane = who ? __ffsll((long long)who) - 1 : -1;
    const float k2 = wave_max_f32(lane == wlane ? kb : ka);
    const unsigned long long who2 = __ballot((lane == wlane ? kb : ka) == k2 && k2 > NEG);
    const int wlane2 = who2 ? __ffsll((long long)who2) - 1 : -1;
    if (lane == wlane) red_c[wave][0] = top.a;
    if (lane == wlane2) red_c[wave][1] = (lane == wlane) ? top.b : top.a;
    if (lane == 0) {
        if (wlane < 0) red_c[wave][0] = Cand{0.f, 0.f, -1};
        if (wlane2 < 0) red_c[wave][1] = Cand{0.f, 0.f, -1};
        red_f[wave][0] = M1; red_f[wave][1] = s1; red_f[wave][2] = Mb; red_f[wave][3] = sb;
    }
    // counters: one atomic per wave
    {
        unsigned long long sc = n_scored;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sc += __shfl_xor(sc, o);
        if (lane == 0 && counters) {
            atomicAdd(&counters->scored, sc);
            atomicAdd(&counters->drains, n_drains);
        }
    }
    __syncthreads();
    if (tid == 0) {
        constexpr int NW = kVocabThreads / kWave;
        float gM1 = red_f[0][0], gMb = red_f[0][2];
        for (int w = 1; w < NW; ++w) { gM1 = fmaxf(gM1, red_f[w][0]); gMb = fmaxf(gMb, red_f[w][2]); }
        float t1 = 0.f, tb = 0.f;
        for (int w = 0; w < NW; ++w) {
            t1 += red_f[w][1] * fast_exp2(red_f[w][0] - gM1);
            tb += red_f[w][3] * fast_exp2(red_f[w][2] - gMb);
        }
        LaneTop2 t; t.init();
        for (int w = 0; w < NW; ++w)
            for (int k = 0; k < 2; ++k) {
                const Cand c = red_c[w][k];
                if (c.i >= 0) t.offer(beta, c.l, c.g, c.i);
            }
        Partial p;
        p.M1 = gM1; p.s1 = t1; p.Mb = gMb; p.sb = tb;
        p.l1 = t.a.l; p.g1 = t.a.g; p.i1 = t.a.i; p.l2 = t.b.l; p.g2 = t.b.g; p.i2 = t.b.i;
        p.pad0 = 0; p.pad1 = 0;
        partials[(int64_t)row * kMaxSplit + split] = p;
        if (counters && split == 0) atomicAdd(&counters->seen, (unsigned long long)V);
    }
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
    int32_t* __restrict__ d_second, Counters* __restrict__ counters)
{
    const int lane = threadIdx.x;
    const uint32_t row = blockIdx.x;
    const char* rowp = (const char*)logits + (int64_t)row * row_stride_bytes;
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

    // finalists: lane c -> candidate (c & 1) of split (c >> 1)
    int32_t idx = -1;
    if (lane < 2 * n_split) idx = (lane & 1) ? pp[lane >> 1].i2 : pp[lane >> 1].i1;
    double key = -INFINITY, lv = 0.0;
    if (idx >= 0) {
        lv = (double)load_scalar<DT>(rowp, idx);
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
            int32_t* h = histAB[parity[row / N]];
            if (h) h[(int64_t)row * T_max + (step - 1)] = tok;
        }
        d_delta[row] = delta; d_logZ1[row] = logZ1; d_logZb[row] = logZb;
        d_gap[row] = k1 - k2;
        d_second[row] = cand2 == 0x7FFFFFFF ? -1 : cand2;
        if (!ok) atomicAdd(&counters->bad_rows, 1ull);
    }
}

// ------------------------------------------------------------------------------------------------
template <int DT, bool DENSE>
static hipError_t launch_k1(smc_ctx* c, const void* logits, int64_t row_stride_bytes, int t, float betaf,
                            int n_split, int vecs_per_split)
{
    const dim3 grid((unsigned)(c->R * n_split)), block(kVocabThreads);
    const uint32_t k0 = (uint32_t)c->cfg.seed, k1 = (uint32_t)(c->cfg.seed >> 32);
    const int V = c->cfg.V;
    Partial* pa = c->ws.partials; Counters* cn = c->ws.counters;
    int P = 0;
    if (betaf == floorf(betaf) && betaf >= 1.f && betaf <= 8.f && betaf != 7.f) P = (int)betaf;
#define PSMC_LAUNCH(PP) hipLaunchKernelGGL((vocab_pass_kernel<DT, PP, DENSE>), grid, block, 0, c->stream, logits, \
                                           row_stride_bytes, V, betaf, k0, k1, (uint32_t)t, n_split, vecs_per_split, pa, cn)
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
    // split a row into n_split contiguous runs of whole "tiles" (one vector per thread)
    int n_split = c->n_split;
    int tiles = (nvec + kVocabThreads - 1) / kVocabThreads;
    if (n_split > tiles) n_split = tiles;
    const int tiles_per_split = (tiles + n_split - 1) / n_split;
    n_split = (tiles + tiles_per_split - 1) / tiles_per_split;
    const int vecs_per_split = tiles_per_split * kVocabThreads;

    hipError_t e;
    const float betaf = (float)beta;
    if (dt == SMC_BF16)
        e = c->dense ? launch_k1<SMC_BF16, true>(c, logits, row_stride_bytes, t, betaf, n_split, vecs_per_split)
                     : launch_k1<SMC_BF16, false>(c, logits, row_stride_bytes, t, betaf, n_split, vecs_per_split);
    else
        e = c->dense ? launch_k1<SMC_F32, true>(c, logits, row_stride_bytes, t, betaf, n_split, vecs_per_split)
                     : launch_k1<SMC_F32, false>(c, logits, row_stride_bytes, t, betaf, n_split, vecs_per_split);
    if (e != hipSuccess) return e;

    const uint32_t k0 = (uint32_t)c->cfg.seed, k1 = (uint32_t)(c->cfg.seed >> 32);
    int32_t* const* hist = c->hist_bound ? (int32_t* const*)c->ws.histAB : nullptr;
    auto& w = c->ws;
    if (dt == SMC_BF16)
        hipLaunchKernelGGL((finalize_rows_kernel<SMC_BF16>), dim3(c->R), dim3(kWave), 0, c->stream, logits,
                           row_stride_bytes, c->cfg.V, c->cfg.N, beta, alpha_t, alpha_prev, k0, k1, (uint32_t)t, n_split,
                           w.partials, w.logW, w.cumlogp, w.parity, hist, c->cfg.T_max, tokens_out, w.d_delta,
                           w.d_logZ1, w.d_logZb, w.d_gap, w.d_second, w.counters);
    else
        hipLaunchKernelGGL((finalize_rows_kernel<SMC_F32>), dim3(c->R), dim3(kWave), 0, c->stream, logits,
                           row_stride_bytes, c->cfg.V, c->cfg.N, beta, alpha_t, alpha_prev, k0, k1, (uint32_t)t, n_split,
                           w.partials, w.logW, w.cumlogp, w.parity, hist, c->cfg.T_max, tokens_out, w.d_delta,
                           w.d_logZ1, w.d_logZb, w.d_gap, w.d_second, w.counters);
    return hipGetLastError();
}

}  // namespace psmc
