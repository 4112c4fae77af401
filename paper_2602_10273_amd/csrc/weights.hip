// Per-prompt weight normalisation, ESS (Eq. "ess") and ESS-triggered systematic resampling
// (Alg. 1; Sec. 7 implementation details) for gfx950.  O(R) work in fp64: one wave per prompt.
//
// The sums that decide discrete outcomes (ESS < kappa*N, cumulative weights against the resampling positions)
// are accumulated in particle order by one lane, so that they round like a plain left-to-right loop.
#include "device_rng.hpp"
#include "smc_internal.hpp"

namespace psmc {

namespace {

// log-sum-exp of x_i and of 2 x_i over one prompt, particle order.  Returns on every lane.
// sh_a / sh_b: LDS scratch of N doubles each.
__device__ void prompt_lse(const double* __restrict__ lw, int N, double* sh_a, double* sh_b, double& L1, double& L2)
{
    const int lane = threadIdx.x;
    double mx = -INFINITY;
    for (int i = lane; i < N; i += kWave) mx = fmax(mx, lw[i]);
    mx = wave_max_f64(mx);
    for (int i = lane; i < N; i += kWave) {
        sh_a[i] = exp(lw[i] - mx);
        sh_b[i] = exp(2.0 * lw[i] - 2.0 * mx);
    }
    __syncthreads();
    double s1 = 0.0, s2 = 0.0;
    if (lane == 0) {
        for (int i = 0; i < N; ++i) { s1 += sh_a[i]; s2 += sh_b[i]; }
    }
    s1 = __shfl(s1, 0); s2 = __shfl(s2, 0);
    L1 = mx + log(s1);
    L2 = 2.0 * mx + log(s2);
    __syncthreads();
}

}  // namespace

// a3: ESS and normalised log-weights.
__global__ __launch_bounds__(kWave) void ess_kernel(const double* __restrict__ logW, int N, double* __restrict__ ess_out,
                                                    double* __restrict__ lognormw_out)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    const int b = blockIdx.x, lane = threadIdx.x;
    const double* lw = logW + (int64_t)b * N;
    double L1, L2;
    prompt_lse(lw, N, sh_a, sh_b, L1, L2);
    if (lane == 0) ess_out[b] = exp(2.0 * L1 - L2);
    if (lognormw_out)
        for (int i = lane; i < N; i += kWave) lognormw_out[(int64_t)b * N + i] = lw[i] - L1;
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

// a3 + a4: trigger ESS < kappa*N, ancestors, weights of resampled prompts reset.  Running sums of the normalised
// weights are taken in particle order by one lane.  scheme 0 is the paper's systematic resampling
// (A_i = min{ j : C_j >= (u_0 + i)/N }); 1 stratified ((u_i + i)/N), 2 multinomial (u_i), 3 residual
// (floor(N w_j) copies, the rest multinomial on the residual weights) are the alternatives App. E names.
__global__ __launch_bounds__(kWave) void resample_kernel(double* __restrict__ logW, int N, double kappa, uint32_t key0,
                                                         uint32_t key1, uint32_t step, int scheme, int order,
                                                         int32_t* __restrict__ anc, int32_t* __restrict__ resampled,
                                                         double* __restrict__ ess_out, double* __restrict__ logZhat)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    __shared__ int sh_k;
    const int b = blockIdx.x, lane = threadIdx.x;
    double* lw = logW + (int64_t)b * N;
    double L1, L2;
    prompt_lse(lw, N, sh_a, sh_b, L1, L2);
    const double ess = exp(2.0 * L1 - L2);
    if (lane == 0 && ess_out) ess_out[b] = ess;
    const bool fire = ess < kappa * (double)N;           // strict; false for NaN
    if (lane == 0) resampled[b] = fire ? 1 : 0;
    // running estimate of the normalising constant: every resampling contributes the mean unnormalised weight
    if (lane == 0 && fire && logZhat) logZhat[b] += L1 - log((double)N);
    if (!fire) {
        for (int i = lane; i < N; i += kWave) anc[(int64_t)b * N + i] = b * N + i;
        return;
    }
    for (int i = lane; i < N; i += kWave) sh_a[i] = exp(lw[i] - L1);
    __syncthreads();
    int32_t* A = anc + (int64_t)b * N;
    if (scheme != 3) {
        if (lane == 0) {
            double c = 0.0;
            for (int j = 0; j < N; ++j) { c += sh_a[j]; sh_b[j] = c; }
        }
        __syncthreads();
        const double u0 = resampling_uniform(0u, (uint32_t)b, step, key0, key1);
        for (int i = lane; i < N; i += kWave) {
            double p;
            if (scheme == 0) p = (u0 + (double)i) / (double)N;
            else {
                const double u = resampling_uniform((uint32_t)i, (uint32_t)b, step, key0, key1);
                p = scheme == 1 ? (u + (double)i) / (double)N : u;
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
            sh_k = k;
            const int rest = N - k;
            if (rest > 0) {
                double c = 0.0;
                for (int j = 0; j < N; ++j) { c += sh_b[j] / (double)rest; sh_b[j] = c; }
            }
        }
        __syncthreads();
        const int k = sh_k;
        for (int i = lane; i < N - k; i += kWave) {
            const double u = resampling_uniform((uint32_t)i, (uint32_t)b, step, key0, key1);
            A[k + i] = b * N + first_reaching(sh_b, N, u);
        }
    }
    __syncthreads();
    for (int i = lane; i < N; i += kWave) lw[i] = 0.0;
    if (order == 1) {
        // Survivors stay in place: every distinct ancestor keeps its own slot, the other copies fill the free slots
        // in increasing order, in the order in which they were drawn.  One lane, O(N); the weight arrays are free now.
        int32_t* slot = reinterpret_cast<int32_t*>(sh_a);
        int32_t* seen = reinterpret_cast<int32_t*>(sh_b);
        const int base = b * N;
        for (int i = lane; i < N; i += kWave) { slot[i] = -1; seen[i] = 0; }
        __syncthreads();
        for (int i = lane; i < N; i += kWave) { const int a = A[i] - base; slot[a] = a; }
        __syncthreads();
        if (lane == 0) {
            int free_slot = 0;
            for (int i = 0; i < N; ++i) {
                const int a = A[i] - base;
                if (!seen[a]) { seen[a] = 1; continue; }
                while (slot[free_slot] != -1) ++free_slot;
                slot[free_slot] = a;
            }
        }
        __syncthreads();
        for (int i = lane; i < N; i += kWave) A[i] = base + slot[i];
    }
}

// log of the SMC estimate of the normalising constant Z_alpha of the power target, per prompt: the factors
// accumulated at the resampling times (mean unnormalised weight each) times the current mean weight.
__global__ __launch_bounds__(kWave) void log_zhat_kernel(const double* __restrict__ logW, int N,
                                                         const double* __restrict__ logZhat, double* __restrict__ out)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    const int b = blockIdx.x;
    double L1, L2;
    prompt_lse(logW + (int64_t)b * N, N, sh_a, sh_b, L1, L2);
    if (threadIdx.x == 0) out[b] = logZhat[b] + L1 - log((double)N);
}

hipError_t launch_log_zhat(smc_ctx* c, double* out)
{
    hipLaunchKernelGGL(log_zhat_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, c->ws.logW, c->cfg.N, c->ws.logZhat, out);
    return hipGetLastError();
}

// Output of Alg. 1: I ~ Categorical(W) by inversion of the running sum of the normalised weights (particle order).
__global__ __launch_bounds__(kWave) void final_draw_kernel(const double* __restrict__ logW, int N, uint32_t key0,
                                                           uint32_t key1, uint32_t step, int32_t* __restrict__ choice)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    const int b = blockIdx.x, lane = threadIdx.x;
    const double* lw = logW + (int64_t)b * N;
    double L1, L2;
    prompt_lse(lw, N, sh_a, sh_b, L1, L2);
    for (int i = lane; i < N; i += kWave) sh_a[i] = exp(lw[i] - L1);
    __syncthreads();
    if (lane == 0) {
        const U4 blk = philox4x32_10(0u, (uint32_t)b, step, 2u, key0, key1);
        const double u = ((double)blk.x + 0.5) * 0x1p-32;
        double c = 0.0;
        int pick = N - 1;
        for (int j = 0; j < N; ++j) { c += sh_a[j]; if (c >= u) { pick = j; break; } }
        choice[b] = b * N + pick;
    }
}

hipError_t launch_final_draw(smc_ctx* c, int t, int32_t* choice)
{
    hipLaunchKernelGGL(final_draw_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, c->ws.logW, c->cfg.N,
                       (uint32_t)c->cfg.seed, (uint32_t)(c->cfg.seed >> 32), (uint32_t)t, choice);
    return hipGetLastError();
}

// Alg. 1 initialisation: W~ = 1, empty prefixes; all rows live in buffer A; diagnostics cleared.
__global__ void init_state_kernel(double* logW, double* cumlogp, int32_t* parity, int32_t* done, int R, int B, int32_t* rowstat,
                                  GatherPlan* plan, double* logZhat)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) logZhat[i] = 0.0;
    if (i < R) { logW[i] = 0.0; cumlogp[i] = 0.0; done[i] = 0; parity[i] = 0; rowstat[3 * i] = 0; rowstat[3 * i + 1] = 0; rowstat[3 * i + 2] = 0; }
    if (i == 0) {
        plan->n_groups[0] = 0; plan->n_groups[1] = 0; plan->bad_anc = 0; plan->phase = 0; plan->ticket = 0;
    }
}

hipError_t launch_init_state(smc_ctx* c)
{
    const int n = c->R > c->cfg.B ? c->R : c->cfg.B;
    hipLaunchKernelGGL(init_state_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, c->ws.logW, c->ws.cumlogp,
                       c->ws.parity, c->ws.done, c->R, c->cfg.B, c->ws.d_rowstat, c->ws.plan, c->ws.logZhat);
    return hipGetLastError();
}

hipError_t launch_ess(smc_ctx* c, const double* logW, double* ess_out, double* lognormw_out)
{
    hipLaunchKernelGGL(ess_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, logW, c->cfg.N, ess_out, lognormw_out);
    return hipGetLastError();
}

hipError_t launch_resample(smc_ctx* c, double* logW, int t, int32_t* anc, int32_t* resampled, double* ess_out)
{
    hipLaunchKernelGGL(resample_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, logW, c->cfg.N, c->cfg.kappa,
                       (uint32_t)c->cfg.seed, (uint32_t)(c->cfg.seed >> 32), (uint32_t)t, c->resampler, c->ancestor_order, anc,
                       resampled, ess_out, logW == c->ws.logW ? c->ws.logZhat : nullptr);
    return hipGetLastError();
}

}  // namespace psmc
