// Host side of libpower_smc: argument validation, workspace layout, kernel launches.  No device allocation.
#include <math.h>
#include <new>
#include <string.h>

#include "smc_internal.hpp"

using namespace psmc;

namespace {

constexpr size_t kAlign = 256;
inline size_t up(size_t x) { return (x + kAlign - 1) & ~(kAlign - 1); }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

smc_status check_config(const smc_config* c)
{
    if (!c) return SMC_E_NULL;
    if (c->B < 1 || c->N < 1 || c->V < 1 || c->T_max < 1) return SMC_E_SHAPE;
    if (c->N > SMC_MAX_PARTICLES) return SMC_E_SHAPE;
    if ((int64_t)c->B * c->N > (int64_t)1 << 24) return SMC_E_SHAPE;
    if (c->T_max % 4 != 0) return SMC_E_ALIGN;
    if (c->logits_dtype != SMC_BF16 && c->logits_dtype != SMC_F32) return SMC_E_DTYPE;
    if (!(c->kappa >= 0.0 && c->kappa <= 1.0)) return SMC_E_RANGE;
    if (c->eos_id < -1 || c->eos_id >= c->V) return SMC_E_RANGE;
    if (c->kv_tensors < 0 || c->kv_tensors > SMC_MAX_KV_TENSORS) return SMC_E_SHAPE;
    if (c->kv_tensors > 0) {
        if (c->kv_H < 1 || c->kv_S < 1 || c->kv_D < 1) return SMC_E_SHAPE;
        if (c->kv_elem_bytes != 1 && c->kv_elem_bytes != 2 && c->kv_elem_bytes != 4) return SMC_E_DTYPE;
        if (((int64_t)c->kv_D * c->kv_elem_bytes) % 16 != 0) return SMC_E_ALIGN;
    }
    return SMC_OK;
}

// Walks the workspace layout; with base == nullptr only the size is computed.
size_t layout(const smc_config* c, char* base, Workspace* w)
{
    const size_t R = (size_t)c->B * c->N;
    const size_t mask_words = ((size_t)c->N + 63) / 64;
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += up(bytes); return p; };
    char* p;
    p = take(R * 8); if (w) w->logW = (double*)p;
    p = take(R * 8); if (w) w->cumlogp = (double*)p;
    p = take(R * 4); if (w) w->parity = (int32_t*)p;
    p = take(R * 4); if (w) w->done = (int32_t*)p;
    p = take((size_t)c->B * 8); if (w) w->logZhat = (double*)p;
    p = take((size_t)c->B * 8); if (w) w->logZest = (double*)p;
    p = take(R * kMaxSplit * sizeof(Partial)); if (w) w->partials = (Partial*)p;
    p = take(R * 4); if (w) w->row_ticket = (int32_t*)p;
    p = take((size_t)c->B * 4); if (w) w->prompt_ticket = (int32_t*)p;
    p = take(4); if (w) w->d_step = (int32_t*)p;
    p = take(((size_t)c->T_max + 2) * 8); if (w) w->d_sched = (double*)p;
    p = take(R * 8); if (w) w->d_delta = (double*)p;
    p = take(R * 8); if (w) w->d_logZ1 = (double*)p;
    p = take(R * 8); if (w) w->d_logZb = (double*)p;
    p = take(R * 8); if (w) w->d_gap = (double*)p;
    p = take(R * 4); if (w) w->d_second = (int32_t*)p;
    p = take(R * 12); if (w) w->d_rowstat = (int32_t*)p;
    p = take(sizeof(GatherPlan)); if (w) w->plan = (GatherPlan*)p;
    p = take(R * 4); if (w) w->grp_src = (int32_t*)p;
    p = take(R * 4); if (w) w->grp_base = (int32_t*)p;
    p = take(R * 4); if (w) w->grp_srcpar = (int32_t*)p;
    p = take(R * mask_words * 8); if (w) w->grp_mask = (unsigned long long*)p;
    p = take((size_t)(c->kv_tensors > 0 ? c->kv_tensors : 1) * sizeof(void*)); if (w) w->kvA = (void**)p;
    p = take((size_t)(c->kv_tensors > 0 ? c->kv_tensors : 1) * sizeof(void*)); if (w) w->kvB = (void**)p;
    p = take(2 * sizeof(void*)); if (w) w->histAB = (void**)p;
    return off;
}

}  // namespace

namespace psmc {

smc_status validate_config(const smc_config* c) { return check_config(c); }

// Launch shape of the vocabulary pass.  Few rows: big workgroups (16 waves share their bound through LDS) and just
// enough slices per row to put about one workgroup on each of the 256 CUs.  Many rows: 4-wave workgroups, one per row.
void auto_shape(int R, int V, int dtype, int* wg_waves, int* n_split)
{
    const int epv = dtype == SMC_BF16 ? 8 : 4;
    const int nvec = (V + epv - 1) / epv;
    if (R >= 1024) { *wg_waves = 4; *n_split = 1; return; }
    *wg_waves = 16;
    const int tiles = (nvec + 1023) / 1024;
    int s = (256 + R - 1) / R;
    if (s > tiles) s = tiles;
    if (s > kMaxSplit) s = kMaxSplit;
    if (s < 1) s = 1;
    *n_split = s;
}

}  // namespace psmc

extern "C" {

const char* smc_status_str(smc_status s)
{
    switch (s) {
        case SMC_OK: return "ok";
        case SMC_E_NULL: return "null pointer";
        case SMC_E_SHAPE: return "bad shape";
        case SMC_E_DTYPE: return "bad dtype";
        case SMC_E_ALIGN: return "bad alignment";
        case SMC_E_RANGE: return "value out of range";
        case SMC_E_STATE: return "bad state";
        case SMC_E_HIP: return "HIP error";
    }
    return "unknown";
}

size_t smc_workspace_bytes(const smc_config* cfg)
{
    if (check_config(cfg) != SMC_OK) return 0;
    return layout(cfg, nullptr, nullptr);
}

smc_status smc_init(const smc_config* cfg, void* d_workspace, size_t workspace_bytes, void* hip_stream, smc_ctx** out_ctx)
{
    if (!out_ctx) return SMC_E_NULL;
    *out_ctx = nullptr;
    smc_status st = check_config(cfg);
    if (st != SMC_OK) return st;
    if (!d_workspace) return SMC_E_NULL;
    if (((uintptr_t)d_workspace & (kAlign - 1)) != 0) return SMC_E_ALIGN;
    if (workspace_bytes < layout(cfg, nullptr, nullptr)) return SMC_E_SHAPE;

    smc_ctx* c = new (std::nothrow) smc_ctx();
    if (!c) return SMC_E_STATE;
    c->cfg = *cfg;
    c->stream = (hipStream_t)hip_stream;
    c->R = cfg->B * cfg->N;
    layout(cfg, (char*)d_workspace, &c->ws);
    auto_shape(c->R, cfg->V, cfg->logits_dtype, &c->wg_waves, &c->n_split);
    c->dense = 0;
    c->mask_words = (cfg->N + 63) / 64;
    c->resampler = 0;
    c->ancestor_order = 0;
    c->kv_skip_terminated = 0;
    c->device_step = 0;
    c->n_sched = 0;
    c->sched_integer_power = 0;
    c->kv_bound = 0;
    c->hist_bound = 0;
    c->profiling = 0;
    c->ev_used[0] = c->ev_used[1] = c->ev_used[2] = c->ev_used[3] = 0;
    c->paged = PagedKV{};
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    } else {
        (void)hipGetLastError();
        delete c;
        return SMC_E_HIP;
    }
    c->gather_grid = cus * 4;             // measured: any of 4..32 persistent workgroups per CU reaches the copy plateau
    c->gather_variant = 4;                // 4 vectors per thread, plain loads, non-temporal stores
    c->n_cus = cus;
    if (launch_init_state(c) != hipSuccess) { delete c; return SMC_E_HIP; }
    *out_ctx = c;
    return SMC_OK;
}

smc_status smc_destroy(smc_ctx* ctx)
{
    if (!ctx) return SMC_E_NULL;
    const hipError_t e = hipStreamSynchronize(ctx->stream);
    for (auto& pool : ctx->ev_pool)
        for (hipEvent_t ev : pool) (void)hipEventDestroy(ev);
    delete ctx;
    return e == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_kv_bind(smc_ctx* ctx, void* const* h_bufA, void* const* h_bufB, int32_t* d_histA, int32_t* d_histB)
{
    if (!ctx) return SMC_E_NULL;
    int n = ctx->cfg.kv_tensors;
    if (!h_bufA && !h_bufB) n = 0;                     // no dense cache: only the histories are registered
    if (n > 0) {
        if (!h_bufA || !h_bufB) return SMC_E_NULL;
        for (int i = 0; i < n; ++i) {
            if (!h_bufA[i] || !h_bufB[i]) return SMC_E_NULL;
            if (!aligned16(h_bufA[i]) || !aligned16(h_bufB[i])) return SMC_E_ALIGN;
        }
    }
    if ((d_histA == nullptr) != (d_histB == nullptr)) return SMC_E_NULL;
    if (d_histA && (!aligned16(d_histA) || !aligned16(d_histB))) return SMC_E_ALIGN;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    if (n > 0) {
        if (hipMemcpy(ctx->ws.kvA, h_bufA, (size_t)n * sizeof(void*), hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
        if (hipMemcpy(ctx->ws.kvB, h_bufB, (size_t)n * sizeof(void*), hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
    }
    void* hh[2] = {d_histA, d_histB};
    if (hipMemcpy(ctx->ws.histAB, hh, sizeof(hh), hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
    try {                                              // no exception may cross the C boundary
        if (n > 0) { ctx->h_kvA.assign(h_bufA, h_bufA + n); ctx->h_kvB.assign(h_bufB, h_bufB + n); }
        else { ctx->h_kvA.clear(); ctx->h_kvB.clear(); }
    } catch (...) {
        ctx->kv_bound = 0;
        return SMC_E_STATE;
    }
    ctx->kv_bound = n > 0;
    ctx->hist_bound = d_histA != nullptr;
    return SMC_OK;
}

smc_status smc_kv_parity(smc_ctx* ctx, const int32_t** d_parity)
{
    if (!ctx || !d_parity) return SMC_E_NULL;
    *d_parity = ctx->ws.parity;
    return SMC_OK;
}

smc_status smc_step(smc_ctx* ctx, const void* d_logits, int64_t row_stride_elems, int32_t t, double alpha_t,
                    double alpha_prev, double tau_t, int32_t* d_tokens_out)
{
    if (!ctx || !d_logits || !d_tokens_out) return SMC_E_NULL;
    const int esz = ctx->cfg.logits_dtype == SMC_BF16 ? 2 : 4;
    if (row_stride_elems < ctx->cfg.V) return SMC_E_SHAPE;
    if (!aligned16(d_logits) || (row_stride_elems * esz) % 16 != 0) return SMC_E_ALIGN;
    if (t < 1 || t > ctx->cfg.T_max) return SMC_E_RANGE;
    if (!(alpha_t > 0.0) || !(alpha_prev >= 0.0) || !isfinite(alpha_t) || !isfinite(alpha_prev)) return SMC_E_RANGE;
    if (!isfinite(tau_t)) return SMC_E_RANGE;
    const double beta = tau_t <= 0.0 ? alpha_t : 1.0 / tau_t;
    if (!(beta > 0.0) || !isfinite(beta) || beta > 1.0e4) return SMC_E_RANGE;
    return launch_vocab_pass(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out, nullptr) == hipSuccess
               ? SMC_OK : SMC_E_HIP;
}

smc_status smc_step_resample(smc_ctx* ctx, const void* d_logits, int64_t row_stride_elems, int32_t t, double alpha_t,
                             double alpha_prev, double tau_t, int32_t* d_tokens_out, int32_t* d_anc_out,
                             int32_t* d_resampled_out, double* d_ess_out)
{
    if (!ctx || !d_logits || !d_tokens_out || !d_anc_out || !d_resampled_out) return SMC_E_NULL;
    const int esz = ctx->cfg.logits_dtype == SMC_BF16 ? 2 : 4;
    if (row_stride_elems < ctx->cfg.V) return SMC_E_SHAPE;
    if (!aligned16(d_logits) || (row_stride_elems * esz) % 16 != 0) return SMC_E_ALIGN;
    if (t < 1 || t > ctx->cfg.T_max) return SMC_E_RANGE;
    if (!(alpha_t > 0.0) || !(alpha_prev >= 0.0) || !isfinite(alpha_t) || !isfinite(alpha_prev)) return SMC_E_RANGE;
    if (!isfinite(tau_t)) return SMC_E_RANGE;
    const double beta = tau_t <= 0.0 ? alpha_t : 1.0 / tau_t;
    if (!(beta > 0.0) || !isfinite(beta) || beta > 1.0e4) return SMC_E_RANGE;
    // Folding the resampling into the launch saves a launch, but the wave that resamples a prompt keeps its workgroup's
    // slot occupied while it does so.  With few rows the slot has nothing else to run and the fold is a gain; with a
    // thousand rows or more it delays the logit stream of the next row by more than the launch costs (measured on 2048
    // fp32 rows: 206 us folded against 197 + 5 us apart), so large batches take the two launches.
    if (ctx->R >= 1024) {
        if (launch_vocab_pass(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out, nullptr) != hipSuccess)
            return SMC_E_HIP;
        return launch_resample(ctx, ctx->ws.logW, t, d_anc_out, d_resampled_out, d_ess_out) == hipSuccess ? SMC_OK : SMC_E_HIP;
    }
    const FusedResample f{d_anc_out, d_resampled_out, d_ess_out};
    return launch_vocab_pass(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out, &f) == hipSuccess
               ? SMC_OK : SMC_E_HIP;
}

smc_status smc_ess_from(smc_ctx* ctx, const double* d_logW, double* d_ess_out, double* d_lognormw_out)
{
    if (!ctx || !d_logW || !d_ess_out) return SMC_E_NULL;
    return launch_ess(ctx, d_logW, d_ess_out, d_lognormw_out) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_ess(smc_ctx* ctx, double* d_ess_out, double* d_lognormw_out)
{
    if (!ctx) return SMC_E_NULL;
    return smc_ess_from(ctx, ctx->ws.logW, d_ess_out, d_lognormw_out);
}

smc_status smc_resample_from(smc_ctx* ctx, double* d_logW_inout, int32_t t, int32_t* d_anc_out, int32_t* d_resampled_out,
                             double* d_ess_out)
{
    if (!ctx || !d_logW_inout || !d_anc_out || !d_resampled_out) return SMC_E_NULL;
    if (t < 1) return SMC_E_RANGE;
    return launch_resample(ctx, d_logW_inout, t, d_anc_out, d_resampled_out, d_ess_out) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_resample(smc_ctx* ctx, int32_t t, int32_t* d_anc_out, int32_t* d_resampled_out, double* d_ess_out)
{
    if (!ctx) return SMC_E_NULL;
    return smc_resample_from(ctx, ctx->ws.logW, t, d_anc_out, d_resampled_out, d_ess_out);
}

smc_status smc_kv_reindex(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t valid_len, int32_t t)
{
    if (!ctx || !d_anc || !d_resampled) return SMC_E_NULL;
    if (t < 0 || t > ctx->cfg.T_max) return SMC_E_RANGE;
    if (valid_len < 0 || (ctx->cfg.kv_tensors > 0 && valid_len > ctx->cfg.kv_S)) return SMC_E_RANGE;
    if (ctx->cfg.kv_tensors > 0 && valid_len > 0 && !ctx->kv_bound) return SMC_E_STATE;
    return launch_reindex(ctx, d_anc, d_resampled, valid_len, t) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_step_resample_reindex(smc_ctx* ctx, const void* d_logits, int64_t row_stride_elems, int32_t t,
                                     double alpha_t, double alpha_prev, double tau_t, int32_t valid_len,
                                     int32_t* d_tokens_out, int32_t* d_anc_out, int32_t* d_resampled_out, double* d_ess_out)
{
    if (!ctx) return SMC_E_NULL;
    if (valid_len < 0 || (ctx->cfg.kv_tensors > 0 && valid_len > ctx->cfg.kv_S)) return SMC_E_RANGE;
    if (ctx->cfg.kv_tensors > 0 && valid_len > 0 && !ctx->kv_bound) return SMC_E_STATE;
    if (ctx->R < 1024) {
        // few rows: the resampling already rides in the vocabulary pass's launch; plan and gather follow
        const smc_status st = smc_step_resample(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out,
                                                d_anc_out, d_resampled_out, d_ess_out);
        if (st != SMC_OK) return st;
        return launch_reindex(ctx, d_anc_out, d_resampled_out, valid_len, t) == hipSuccess ? SMC_OK : SMC_E_HIP;
    }
    // many rows: the vocabulary pass, then one launch that resamples every prompt and plans its reorder, then the gather
    if (!d_anc_out || !d_resampled_out) return SMC_E_NULL;
    const smc_status st = smc_step(ctx, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out);
    if (st != SMC_OK) return st;
    if (launch_resample_plan(ctx, ctx->ws.logW, t, d_anc_out, d_resampled_out, d_ess_out) != hipSuccess) return SMC_E_HIP;
    return launch_reindex(ctx, d_anc_out, d_resampled_out, valid_len, t, true) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_final_draw(smc_ctx* ctx, int32_t t, int32_t* d_choice_out)
{
    if (!ctx || !d_choice_out) return SMC_E_NULL;
    if (t < 1) return SMC_E_RANGE;
    return launch_final_draw(ctx, t, d_choice_out) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_get_done(smc_ctx* ctx, int32_t* h_done)
{
    if (!ctx || !h_done) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    return hipMemcpy(h_done, ctx->ws.done, (size_t)ctx->R * 4, hipMemcpyDeviceToHost) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_set_done(smc_ctx* ctx, const int32_t* h_done)
{
    if (!ctx || !h_done) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    return hipMemcpy(ctx->ws.done, h_done, (size_t)ctx->R * 4, hipMemcpyHostToDevice) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_get_state(smc_ctx* ctx, double* h_logW, double* h_cumlogp, int32_t* h_parity)
{
    if (!ctx) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    const size_t R = ctx->R;
    if (h_logW && hipMemcpy(h_logW, ctx->ws.logW, R * 8, hipMemcpyDeviceToHost) != hipSuccess) return SMC_E_HIP;
    if (h_cumlogp && hipMemcpy(h_cumlogp, ctx->ws.cumlogp, R * 8, hipMemcpyDeviceToHost) != hipSuccess) return SMC_E_HIP;
    if (h_parity && hipMemcpy(h_parity, ctx->ws.parity, R * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return SMC_E_HIP;
    return SMC_OK;
}

smc_status smc_set_state(smc_ctx* ctx, const double* h_logW, const double* h_cumlogp)
{
    if (!ctx) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    const size_t R = ctx->R;
    if (h_logW && hipMemcpy(ctx->ws.logW, h_logW, R * 8, hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
    if (h_cumlogp && hipMemcpy(ctx->ws.cumlogp, h_cumlogp, R * 8, hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
    return SMC_OK;
}

smc_status smc_get_diag(smc_ctx* ctx, double* h_delta, double* h_logZ1, double* h_logZb, int32_t* h_second, double* h_gap,
                        uint64_t* h_counters)
{
    if (!ctx) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    const size_t R = ctx->R;
    auto get = [&](void* h, const void* d, size_t n) { return !h || hipMemcpy(h, d, n, hipMemcpyDeviceToHost) == hipSuccess; };
    if (!get(h_delta, ctx->ws.d_delta, R * 8) || !get(h_logZ1, ctx->ws.d_logZ1, R * 8) ||
        !get(h_logZb, ctx->ws.d_logZb, R * 8) || !get(h_second, ctx->ws.d_second, R * 4) ||
        !get(h_gap, ctx->ws.d_gap, R * 8))
        return SMC_E_HIP;
    if (h_counters) {
        int32_t* st = new (std::nothrow) int32_t[3 * R];
        if (!st) return SMC_E_STATE;
        if (hipMemcpy(st, ctx->ws.d_rowstat, 3 * R * 4, hipMemcpyDeviceToHost) != hipSuccess) { delete[] st; return SMC_E_HIP; }
        h_counters[0] = h_counters[1] = h_counters[2] = 0;
        for (size_t r = 0; r < R; ++r) {
            h_counters[0] += (uint64_t)st[3 * r]; h_counters[1] += (uint64_t)st[3 * r + 1]; h_counters[2] += (uint64_t)st[3 * r + 2];
        }
        delete[] st;
        h_counters[3] = (uint64_t)R * (uint64_t)ctx->cfg.V;
    }
    return SMC_OK;
}

smc_status smc_get_log_zhat(smc_ctx* ctx, double* h_logZhat, double* h_banked)
{
    if (!ctx || (!h_logZhat && !h_banked)) return SMC_E_NULL;
    if (h_logZhat && launch_log_zhat(ctx, ctx->ws.logZest) != hipSuccess) return SMC_E_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    const size_t n = (size_t)ctx->cfg.B * 8;
    if (h_logZhat && hipMemcpy(h_logZhat, ctx->ws.logZest, n, hipMemcpyDeviceToHost) != hipSuccess) return SMC_E_HIP;
    if (h_banked && hipMemcpy(h_banked, ctx->ws.logZhat, n, hipMemcpyDeviceToHost) != hipSuccess) return SMC_E_HIP;
    return SMC_OK;
}

smc_status smc_set_log_zhat(smc_ctx* ctx, const double* h_banked)
{
    if (!ctx || !h_banked) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    return hipMemcpy(ctx->ws.logZhat, h_banked, (size_t)ctx->cfg.B * 8, hipMemcpyHostToDevice) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_set_kv_skip_terminated(smc_ctx* ctx, int32_t enable)
{
    if (!ctx) return SMC_E_NULL;
    if (enable < 0 || enable > 1) return SMC_E_RANGE;
    ctx->kv_skip_terminated = enable;
    return SMC_OK;
}

smc_status smc_set_schedule(smc_ctx* ctx, const double* h_alpha, int32_t n)
{
    if (!ctx || !h_alpha) return SMC_E_NULL;
    if (n < 2 || n > ctx->cfg.T_max + 2) return SMC_E_SHAPE;
    if (!(h_alpha[0] >= 0.0) || !isfinite(h_alpha[0])) return SMC_E_RANGE;
    for (int i = 1; i < n; ++i)
        if (!(h_alpha[i] > 0.0) || !isfinite(h_alpha[i]) || h_alpha[i] > 1.0e4) return SMC_E_RANGE;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    if (hipMemcpy(ctx->ws.d_sched, h_alpha, (size_t)n * 8, hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
    ctx->n_sched = n;
    int P = integer_power(h_alpha[1]);
    for (int i = 2; i < n && P; ++i)
        if (h_alpha[i] != h_alpha[1]) P = 0;
    ctx->sched_integer_power = P;
    return SMC_OK;
}

smc_status smc_set_device_step(smc_ctx* ctx, int32_t enable, int32_t t)
{
    if (!ctx) return SMC_E_NULL;
    if (enable < 0 || enable > 1) return SMC_E_RANGE;
    if (enable && (t < 1 || t > ctx->cfg.T_max)) return SMC_E_RANGE;
    if (enable && ctx->n_sched < 2) return SMC_E_STATE;            // the exponents have to be on the device too
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    if (enable && hipMemcpy(ctx->ws.d_step, &t, 4, hipMemcpyHostToDevice) != hipSuccess) return SMC_E_HIP;
    ctx->device_step = enable;
    return SMC_OK;
}

smc_status smc_get_device_step(smc_ctx* ctx, int32_t* h_t)
{
    if (!ctx || !h_t) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    return hipMemcpy(h_t, ctx->ws.d_step, 4, hipMemcpyDeviceToHost) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_advance_step(smc_ctx* ctx)
{
    if (!ctx) return SMC_E_NULL;
    if (!ctx->device_step) return SMC_E_STATE;
    return launch_advance_step(ctx) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

smc_status smc_set_resampler(smc_ctx* ctx, int32_t scheme)
{
    if (!ctx) return SMC_E_NULL;
    if (scheme < 0 || scheme > 3) return SMC_E_RANGE;
    ctx->resampler = scheme;
    return SMC_OK;
}

smc_status smc_set_ancestor_order(smc_ctx* ctx, int32_t order)
{
    if (!ctx) return SMC_E_NULL;
    if (order < 0 || order > 1) return SMC_E_RANGE;
    ctx->ancestor_order = order;
    return SMC_OK;
}

smc_status smc_set_gather_tuning(smc_ctx* ctx, int32_t wgs_per_cu, int32_t variant)
{
    if (!ctx) return SMC_E_NULL;
    if (wgs_per_cu < 1 || wgs_per_cu > 64 || variant < 0 || variant > 17) return SMC_E_RANGE;
    ctx->gather_grid = ctx->n_cus * wgs_per_cu;
    ctx->gather_variant = variant;
    return SMC_OK;
}

smc_status smc_profile_enable(smc_ctx* ctx, int32_t enable)
{
    if (!ctx) return SMC_E_NULL;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    ctx->profiling = enable != 0;
    ctx->ev_used[0] = ctx->ev_used[1] = ctx->ev_used[2] = ctx->ev_used[3] = 0;
    return SMC_OK;
}

smc_status smc_profile_read(smc_ctx* ctx, int32_t kind, double* h_total_ms, int64_t* h_launches)
{
    if (!ctx || !h_total_ms || !h_launches) return SMC_E_NULL;
    if (kind < 0 || kind > 3) return SMC_E_RANGE;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    double total = 0.0;
    const size_t n = ctx->ev_used[kind] / 2;
    for (size_t i = 0; i < n; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->ev_pool[kind][2 * i], ctx->ev_pool[kind][2 * i + 1]) != hipSuccess) return SMC_E_HIP;
        total += ms;
    }
    *h_total_ms = total;
    *h_launches = (int64_t)n;
    ctx->ev_used[kind] = 0;
    return SMC_OK;
}

smc_status smc_set_tuning(smc_ctx* ctx, int32_t n_split, int32_t dense, int32_t wg_waves)
{
    if (!ctx) return SMC_E_NULL;
    if (n_split < 0 || n_split > kMaxSplit) return SMC_E_RANGE;
    if (wg_waves != 0 && wg_waves != 4 && wg_waves != 8 && wg_waves != 16) return SMC_E_RANGE;
    if (dense < 0 || dense > 1) return SMC_E_RANGE;
    int aw, as;
    auto_shape(ctx->R, ctx->cfg.V, ctx->cfg.logits_dtype, &aw, &as);
    ctx->wg_waves = wg_waves == 0 ? aw : wg_waves;
    ctx->n_split = n_split == 0 ? (wg_waves == 0 || wg_waves == aw ? as : 1) : n_split;
    ctx->dense = dense;
    return SMC_OK;
}

}  // extern "C"
