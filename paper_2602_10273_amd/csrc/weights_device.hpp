// Device functions of the per-prompt weight step: normalisation, ESS (Eq. "ess") and ESS-triggered resampling
// (Alg. 1; Sec. 7 implementation details; the other schemes App. E names).  One wave works on one prompt; the functions
// synchronise that wave only, so they serve both the one-wave kernels of weights.hip and the tail of the vocabulary
// pass, where the wave that finalizes a prompt's last row goes on to resample the prompt.
//
// The sums that decide discrete outcomes (ESS < kappa*N, cumulative weights against the resampling positions)
// are accumulated in particle order by one lane, so that they round like a plain left-to-right loop.
#pragma once
#include "device_rng.hpp"
#include "smc_internal.hpp"

namespace psmc {

// Orders the LDS traffic of one wave: what any lane wrote before is visible to every lane after.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
}

// A log-weight as the resampling wave reads it: at agent scope, because inside the vocabulary pass's launch the weight
// may have been written a moment ago by another workgroup.
__device__ __forceinline__ double weight_at(const double* lw, int i)
{
    return __hip_atomic_load(lw + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// log-sum-exp of x_i and of 2 x_i over one prompt, particle order.  Returns on every lane.
// sh_a / sh_b: LDS scratch of N doubles each.
__device__ inline void prompt_lse(const double* lw, int N, double* sh_a, double* sh_b, double& L1, double& L2)
{
    const int lane = lane_id();
    double mx = -INFINITY;
    for (int i = lane; i < N; i += kWave) mx = fmax(mx, weight_at(lw, i));
    mx = wave_max_f64(mx);
    for (int i = lane; i < N; i += kWave) {
        const double w = weight_at(lw, i);
        sh_a[i] = exp(w - mx);
        sh_b[i] = exp(2.0 * w - 2.0 * mx);
    }
    wave_sync();
    double s1 = 0.0, s2 = 0.0;
    if (lane == 0) {
        for (int i = 0; i < N; ++i) { s1 += sh_a[i]; s2 += sh_b[i]; }
    }
    s1 = read_lane(s1, 0); s2 = read_lane(s2, 0);
    L1 = mx + log(s1);
    L2 = 2.0 * mx + log(s2);
    wave_sync();
}

// first j in [0, n) with C_j >= p for a non-decreasing C; n-1 if rounding leaves none
__device__ __forceinline__ int first_reaching(const double* C, int n, double p)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (C[mid] >= p) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// uniform of word i of the prompt's resampling stream (Philox domain 1, row := prompt)
__device__ __forceinline__ double resampling_uniform(uint32_t i, uint32_t b, uint32_t step, uint32_t key0, uint32_t key1)
{
    const U4 blk = philox4x32_10(i >> 2, b, step, 1u, key0, key1);
    return ((double)pick_word(blk, i & 3u) + 0.5) * 0x1p-32;
}

// a3 + a4 for prompt b by one wave: trigger ESS < kappa*N, ancestors, weights of resampled prompts reset.  Running sums
// of the normalised weights are taken in particle order by one lane.  scheme 0 is the paper's systematic resampling
// (A_i = min{ j : C_j >= (u_0 + i)/N }); 1 stratified ((u_i + i)/N), 2 multinomial (u_i), 3 residual
// (floor(N w_j) copies, the rest multinomial on the residual weights) are the alternatives App. E names.
// sh_a, sh_b: N doubles of LDS each; sh_k: one int of LDS.  Returns whether the prompt resampled.
__device__ inline bool resample_prompt(const ResampleArgs& r, double* __restrict__ logW, int b, uint32_t step,
                                       double* sh_a, double* sh_b, int* sh_k)
{
    const int lane = lane_id();
    const int N = r.N;
    double* lw = logW + (int64_t)b * N;
    double L1, L2;
    prompt_lse(lw, N, sh_a, sh_b, L1, L2);
    const double ess = exp(2.0 * L1 - L2);
    if (lane == 0 && r.ess_out) r.ess_out[b] = ess;
    const bool fire = ess < r.kappa * (double)N;         // strict; false for NaN
    if (lane == 0) r.resampled[b] = fire ? 1 : 0;
    // running estimate of the normalising constant: every resampling contributes the mean unnormalised weight
    if (lane == 0 && fire && r.logZhat) r.logZhat[b] += L1 - log((double)N);
    int32_t* A = r.anc + (int64_t)b * N;
    if (!fire) {
        for (int i = lane; i < N; i += kWave) A[i] = b * N + i;
        return false;
    }
    for (int i = lane; i < N; i += kWave) sh_a[i] = exp(weight_at(lw, i) - L1);
    wave_sync();
    if (r.scheme != 3) {
        if (lane == 0) {
            double c = 0.0;
            for (int j = 0; j < N; ++j) { c += sh_a[j]; sh_b[j] = c; }
        }
        wave_sync();
        const double u0 = resampling_uniform(0u, (uint32_t)b, step, r.key0, r.key1);
        for (int i = lane; i < N; i += kWave) {
            double p;
            if (r.scheme == 0) p = (u0 + (double)i) / (double)N;
            else {
                const double u = resampling_uniform((uint32_t)i, (uint32_t)b, step, r.key0, r.key1);
                p = r.scheme == 1 ? (u + (double)i) / (double)N : u;
            }
            A[i] = b * N + first_reaching(sh_b, N, p);
        }
    } else {
        if (lane == 0) {                                  // deterministic copies, then the residual weights' running sum
            int k = 0;
            for (int j = 0; j < N; ++j) {
                const double nw = (double)N * sh_a[j];
                const int copies = (int)floor(nw);
                sh_b[j] = nw - (double)copies;
                for (int c = 0; c < copies && k < N; ++c) A[k++] = b * N + j;
            }
            *sh_k = k;
            const int rest = N - k;
            if (rest > 0) {
                double c = 0.0;
                for (int j = 0; j < N; ++j) { c += sh_b[j] / (double)rest; sh_b[j] = c; }
            }
        }
        wave_sync();
        const int k = *sh_k;
        for (int i = lane; i < N - k; i += kWave) {
            const double u = resampling_uniform((uint32_t)i, (uint32_t)b, step, r.key0, r.key1);
            A[k + i] = b * N + first_reaching(sh_b, N, u);
        }
    }
    wave_sync();
    for (int i = lane; i < N; i += kWave) lw[i] = 0.0;
    if (r.order == 1) {
        // Survivors stay in place: every distinct ancestor keeps its own slot, the other copies fill the free slots
        // in increasing order, in the order in which they were drawn.  One lane, O(N); the weight arrays are free now.
        // (The ancestors written above are read back by other lanes: the wave_sync above ordered those accesses.)
        int32_t* slot = reinterpret_cast<int32_t*>(sh_a);
        int32_t* seen = reinterpret_cast<int32_t*>(sh_b);
        const int base = b * N;
        for (int i = lane; i < N; i += kWave) { slot[i] = -1; seen[i] = 0; }
        wave_sync();
        for (int i = lane; i < N; i += kWave) { const int a = A[i] - base; slot[a] = a; }
        wave_sync();
        if (lane == 0) {
            int free_slot = 0;
            for (int i = 0; i < N; ++i) {
                const int a = A[i] - base;
                if (!seen[a]) { seen[a] = 1; continue; }
                while (slot[free_slot] != -1) ++free_slot;
                slot[free_slot] = a;
            }
        }
        wave_sync();
        for (int i = lane; i < N; i += kWave) A[i] = base + slot[i];
    }
    return true;
}

// host side: the arguments of resample_prompt for a context (defined in weights.hip)
ResampleArgs resample_args(const smc_ctx* c, double* logW, int32_t* anc, int32_t* resampled, double* ess_out);

}  // namespace psmc
