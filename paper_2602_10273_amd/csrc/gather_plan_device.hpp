// Device side of the reorder's plan (Alg. 1 "reorder KV cache by A"; App. C): one wave groups the moved rows of one
// resampled prompt by ancestor for the gather kernel.  In a header because two kernels run it: the plan kernel of
// smc_kv_reindex, and the resampling kernel when the reorder follows in the same call (the wave that resampled a
// prompt goes on to plan it).
#pragma once
#include "device_rng.hpp"
#include "smc_internal.hpp"

namespace psmc {

// Where a plan is written.
struct PlanArgs {
    int N, mask_words, skip_terminated;
    GatherPlan* plan;
    int32_t* grp_src; int32_t* grp_base; int32_t* grp_srcpar; unsigned long long* grp_mask;
    double* cumlogp; int32_t* done; int32_t* parity;
};

// The plan of one resampled prompt (one wave).  phase: which of the plan's two group counters this call uses.
__device__ inline void plan_prompt(const int32_t* __restrict__ anc, int N, int mask_words, int phase, GatherPlan* __restrict__ plan,
                            int32_t* __restrict__ grp_src, int32_t* __restrict__ grp_base, int32_t* __restrict__ grp_srcpar,
                            unsigned long long* __restrict__ grp_mask, double* __restrict__ cumlogp,
                            int32_t* __restrict__ done, int32_t* __restrict__ parity, int skip_terminated)
{
    __shared__ int32_t sh_anc[SMC_MAX_PARTICLES];
    __shared__ double sh_cum[SMC_MAX_PARTICLES];
    __shared__ int32_t sh_done[SMC_MAX_PARTICLES];
    __shared__ int32_t sh_first[SMC_MAX_PARTICLES];                // lowest moved row that continues each ancestor
    __shared__ int32_t sh_group[SMC_MAX_PARTICLES];                // group number of each ancestor that has one
    __shared__ int32_t sh_base;
    const int b = blockIdx.x, lane = threadIdx.x;
    const int row0 = b * N;
    int bad = 0;
    for (int k = lane; k < N; k += kWave) {
        int a = anc[row0 + k] - row0;
        if (a < 0 || a >= N) { a = -1; ++bad; }                    // outside the prompt: row is left untouched
        if (a == k) a = -1;                                        // its own ancestor: nothing to move
        sh_anc[k] = a;
        sh_cum[k] = cumlogp[row0 + k];
        sh_done[k] = done[row0 + k];
    }
    __syncthreads();
    // leaders: first moved row (in particle order) of each distinct ancestor
    for (int k = lane; k < N; k += kWave) sh_first[k] = N;
    __syncthreads();
    for (int k = lane; k < N; k += kWave)
        if (sh_anc[k] >= 0) atomicMin(&sh_first[sh_anc[k]], k);
    __syncthreads();
    int n_lead = 0;
    for (int k0 = 0; k0 < N; k0 += kWave) {
        const int k = k0 + lane;
        const bool lead = k < N && sh_anc[k] >= 0 && sh_first[sh_anc[k]] == k;
        n_lead += __popcll(__ballot(lead));
    }
    if (lane == 0) sh_base = n_lead ? atomicAdd(&plan->n_groups[phase], n_lead) : 0;
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o);
    if (lane == 0 && bad) atomicAdd(&plan->bad_anc, bad);
    __syncthreads();
    int placed = 0;
    for (int k0 = 0; k0 < N; k0 += kWave) {
        const int k = k0 + lane;
        const bool lead = k < N && sh_anc[k] >= 0 && sh_first[sh_anc[k]] == k;
        const unsigned long long mk = __ballot(lead);
        if (lead) {
            const int a = sh_anc[k];
            const int g = sh_base + placed + mask_rank(mk);
            grp_src[g] = row0 + a;
            grp_base[g] = row0;
            // bit 0: the ancestor's live buffer, before any flip; bit 1 (only where the caller opted in and an
            // end-of-sequence token is configured): the ancestor has terminated -- its cache is never read again
            // (App. D: the absorbing state is a no-op), so its KV rows are not copied
            grp_srcpar[g] = parity[row0 + a] | ((skip_terminated && sh_done[a]) ? 2 : 0);
            for (int w = 0; w < mask_words; ++w) grp_mask[(int64_t)g * mask_words + w] = 0ull;
            sh_group[a] = g;
        }
        placed += __popcll(mk);
    }
    __syncthreads();                                               // group numbers known, bit sets cleared
    for (int k = lane; k < N; k += kWave) {
        const int a = sh_anc[k];
        if (a >= 0) atomicOr(&grp_mask[(int64_t)sh_group[a] * mask_words + (k >> 6)], 1ull << (k & 63));
    }
    __syncthreads();                                               // every group has recorded its source parity
    for (int k = lane; k < N; k += kWave) {
        const int a = sh_anc[k];
        if (a >= 0) {
            cumlogp[row0 + k] = sh_cum[a];
            done[row0 + k] = sh_done[a];
            parity[row0 + k] ^= 1;                                 // from now on: the buffer this row is written to
        }
    }
}

// The two group counters alternate between successive plans, and the switch happens on the device: every workgroup
// of a plan reads plan->phase first and calls this last; the one with the last ticket clears the other counter for
// the next plan and flips the phase.  No host-side state is involved, so a captured launch sequence can be replayed.
__device__ inline void plan_finish(GatherPlan* plan, int phase, int n_workgroups)
{
    if (threadIdx.x == 0) {
        __threadfence();                                           // the read of plan->phase precedes the ticket
        if (atomicAdd(&plan->ticket, 1) == n_workgroups - 1) {
            plan->n_groups[phase ^ 1] = 0;
            plan->ticket = 0;
            plan->phase = phase ^ 1;
        }
    }
}

}  // namespace psmc
