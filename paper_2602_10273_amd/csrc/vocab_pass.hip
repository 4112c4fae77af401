// Host side of the vocabulary pass: launch shape, step arguments, dispatch to the per-dtype translation units.
#include <math.h>

#include "weights_device.hpp"

namespace psmc {

hipError_t launch_vocab_bf16(smc_ctx* c, const StepArgs& a, int P);    // vocab_pass_bf16.hip
hipError_t launch_vocab_f32(smc_ctx* c, const StepArgs& a, int P);     // vocab_pass_f32.hip

// Advances the context's device-resident step counter (one thread).
__global__ void advance_step_kernel(int32_t* d_step) { if (threadIdx.x == 0 && blockIdx.x == 0) *d_step += 1; }

int integer_power(double beta)
{
    const float b = (float)beta;
    return (b == floorf(b) && b >= 1.f && b <= 8.f && b != 7.f) ? (int)b : 0;
}

hipError_t launch_vocab_pass(smc_ctx* c, const void* logits, int64_t row_stride, int t, double alpha_t,
                             double alpha_prev, double tau_t, int32_t* tokens_out, const FusedResample* fused)
{
    const int dt = c->cfg.logits_dtype;
    const int esz = dt == SMC_BF16 ? 2 : 4;
    const int epv = 16 / esz;
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

    auto& w = c->ws;
    StepArgs a{};
    a.logits = logits; a.row_stride_bytes = row_stride * esz; a.V = c->cfg.V;
    a.key0 = (uint32_t)c->cfg.seed; a.key1 = (uint32_t)(c->cfg.seed >> 32);
    a.step = (uint32_t)t; a.alpha_t = alpha_t; a.alpha_prev = alpha_prev;
    a.tau_by_value = tau_t;
    a.beta = tau_t <= 0.0 ? alpha_t : 1.0 / tau_t;
    a.n_split = n_split; a.vecs_per_split = vecs_per_split;
    a.partials = w.partials; a.row_ticket = w.row_ticket;
    a.logW = w.logW; a.cumlogp = w.cumlogp; a.parity = w.parity;
    a.histAB = c->hist_bound ? (int32_t* const*)w.histAB : nullptr;
    a.T_max = c->cfg.T_max; a.tokens_out = tokens_out;
    a.d_delta = w.d_delta; a.d_logZ1 = w.d_logZ1; a.d_logZb = w.d_logZb; a.d_gap = w.d_gap; a.d_second = w.d_second;
    a.d_rowstat = w.d_rowstat; a.eos_id = c->cfg.eos_id; a.done = w.done;
    int P = integer_power(a.beta);
    if (c->device_step) {
        // step, exponents (and beta = alpha_t unless a proposal temperature is given by value) come from the device; the
        // integer-exponent instantiation is only safe when every exponent the schedule can still yield is that integer
        a.d_step = w.d_step; a.d_sched = w.d_sched; a.n_sched = c->n_sched;
        P = tau_t <= 0.0 ? c->sched_integer_power : integer_power(a.beta);
    }
    a.fuse_resample = 0;
    if (fused) {
        a.fuse_resample = 1;
        a.prompt_ticket = w.prompt_ticket;
        a.rs = resample_args(c, w.logW, fused->anc, fused->resampled, fused->ess_out);
    }

    ScopedKernelTimer timer(c, 0);
    return dt == SMC_BF16 ? launch_vocab_bf16(c, a, P) : launch_vocab_f32(c, a, P);
}

hipError_t launch_advance_step(smc_ctx* c)
{
    hipLaunchKernelGGL(advance_step_kernel, dim3(1), dim3(64), 0, c->stream, c->ws.d_step);
    return hipGetLastError();
}

}  // namespace psmc
