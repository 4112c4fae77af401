// Per-prompt weight normalisation, ESS (Eq. "ess") and ESS-triggered systematic resampling
// (Alg. 1; Sec. 7 implementation details) for gfx950.  O(R) work in fp64: one wave per prompt.
//
// The sums that decide discrete outcomes (ESS < kappa*N, cumulative weights against the resampling positions)
// are accumulated in particle order by one lane, so that they round like a plain left-to-right loop.
#include "gather_plan_device.hpp"
#include "weights_device.hpp"

namespace psmc {

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

// a3 + a4: one wave per prompt (the arithmetic is resample_prompt's).
// d_step: not null -> the step number is read from the device (a replayed capture advances with the counter).
__global__ __launch_bounds__(kWave) void resample_kernel(double* __restrict__ logW, ResampleArgs r, uint32_t step,
                                                         const int32_t* __restrict__ d_step)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    __shared__ int sh_k;
    if (d_step) step = (uint32_t)*d_step;
    resample_prompt(r, logW, blockIdx.x, step, sh_a, sh_b, &sh_k);
}

// a3 + a4 and the first half of a5 in one launch: the wave that resampled a prompt goes on to plan its reorder (the
// grouping of the moved rows by ancestor that plan_kernel would make in a launch of its own).
__global__ __launch_bounds__(kWave) void resample_plan_kernel(double* __restrict__ logW, ResampleArgs r, uint32_t step,
                                                              const int32_t* __restrict__ d_step, PlanArgs pl)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    __shared__ int sh_k;
    if (d_step) step = (uint32_t)*d_step;
    const int phase = pl.plan->phase;
    const bool fire = resample_prompt(r, logW, blockIdx.x, step, sh_a, sh_b, &sh_k);
    if (fire) {
        __threadfence();                                // the ancestors this wave just wrote are read back through memory
        plan_prompt(r.anc, pl.N, pl.mask_words, phase, pl.plan, pl.grp_src, pl.grp_base, pl.grp_srcpar, pl.grp_mask, pl.cumlogp,
                    pl.done, pl.parity, pl.skip_terminated);
    }
    plan_finish(pl.plan, phase, (int)gridDim.x);
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
                                                           uint32_t key1, uint32_t step, const int32_t* __restrict__ d_step,
                                                           int32_t* __restrict__ choice)
{
    __shared__ double sh_a[SMC_MAX_PARTICLES], sh_b[SMC_MAX_PARTICLES];
    const int b = blockIdx.x, lane = threadIdx.x;
    if (d_step) step = (uint32_t)*d_step;
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
                       (uint32_t)c->cfg.seed, (uint32_t)(c->cfg.seed >> 32), (uint32_t)t,
                       c->device_step ? c->ws.d_step : nullptr, choice);
    return hipGetLastError();
}

// Alg. 1 initialisation: W~ = 1, empty prefixes; all rows live in buffer A; diagnostics cleared.
__global__ void init_state_kernel(double* logW, double* cumlogp, int32_t* parity, int32_t* done, int R, int B, int32_t* rowstat,
                                  GatherPlan* plan, double* logZhat, int32_t* row_ticket, int32_t* prompt_ticket, int32_t* d_step)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) { logZhat[i] = 0.0; prompt_ticket[i] = 0; }
    if (i < R) row_ticket[i] = 0;
    if (i == 0) *d_step = 1;
    if (i < R) { logW[i] = 0.0; cumlogp[i] = 0.0; done[i] = 0; parity[i] = 0; rowstat[3 * i] = 0; rowstat[3 * i + 1] = 0; rowstat[3 * i + 2] = 0; }
    if (i == 0) {
        plan->n_groups[0] = 0; plan->n_groups[1] = 0; plan->bad_anc = 0; plan->phase = 0; plan->ticket = 0;
    }
}

hipError_t launch_init_state(smc_ctx* c)
{
    const int n = c->R > c->cfg.B ? c->R : c->cfg.B;
    hipLaunchKernelGGL(init_state_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, c->ws.logW, c->ws.cumlogp,
                       c->ws.parity, c->ws.done, c->R, c->cfg.B, c->ws.d_rowstat, c->ws.plan, c->ws.logZhat, c->ws.row_ticket,
                       c->ws.prompt_ticket, c->ws.d_step);
    return hipGetLastError();
}

hipError_t launch_ess(smc_ctx* c, const double* logW, double* ess_out, double* lognormw_out)
{
    hipLaunchKernelGGL(ess_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, logW, c->cfg.N, ess_out, lognormw_out);
    return hipGetLastError();
}

ResampleArgs resample_args(const smc_ctx* c, double* logW, int32_t* anc, int32_t* resampled, double* ess_out)
{
    ResampleArgs r;
    r.N = c->cfg.N; r.kappa = c->cfg.kappa;
    r.key0 = (uint32_t)c->cfg.seed; r.key1 = (uint32_t)(c->cfg.seed >> 32);
    r.scheme = c->resampler; r.order = c->ancestor_order;
    r.anc = anc; r.resampled = resampled; r.ess_out = ess_out;
    r.logZhat = logW == c->ws.logW ? c->ws.logZhat : nullptr;    // only the context's own weights feed its estimate
    return r;
}

hipError_t launch_resample(smc_ctx* c, double* logW, int t, int32_t* anc, int32_t* resampled, double* ess_out)
{
    hipLaunchKernelGGL(resample_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, logW,
                       resample_args(c, logW, anc, resampled, ess_out), (uint32_t)t,
                       c->device_step ? c->ws.d_step : nullptr);
    return hipGetLastError();
}

PlanArgs plan_args(const smc_ctx* c);                  // kv_gather.hip

hipError_t launch_resample_plan(smc_ctx* c, double* logW, int t, int32_t* anc, int32_t* resampled, double* ess_out)
{
    hipLaunchKernelGGL(resample_plan_kernel, dim3(c->cfg.B), dim3(kWave), 0, c->stream, logW,
                       resample_args(c, logW, anc, resampled, ess_out), (uint32_t)t,
                       c->device_step ? c->ws.d_step : nullptr, plan_args(c));
    return hipGetLastError();
}

}  // namespace psmc
