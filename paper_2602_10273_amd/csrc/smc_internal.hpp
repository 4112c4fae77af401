// Internal declarations shared by the HIP translation units of libpower_smc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "power_smc.h"

namespace psmc {

constexpr int kWave = 64;
constexpr int kMaxSplit = 32;          // workgroups per row in the vocabulary pass (finalize uses 2 lanes per split)

// Bounds of the Gumbel variate g = -log(-log u), u = (x + 1/2)/2^32 over all 32-bit words x:
// g in [-log(33 log 2), ~33 log 2] = [-3.12999.., 22.87385..].  Rounded outwards.
constexpr float kGumbelMin = -3.1300f;
constexpr float kGumbelMax = 22.8740f;
// Slack added to every "cannot win" test: covers fp32 rounding of keys, and keeps every entry whose key is
// within this distance of the winner among the scored candidates.
constexpr float kKeyMargin = 0.01f;

// One workgroup's summary of its slice of a row.
//   sum_v exp(l_v)        = s1 * 2^M1        (M1, Mb integer-valued floats)
//   sum_v exp(beta * l_v) = sb * 2^Mb
//   two best candidates of the Gumbel-max draw by fp32 key, as (logit, gumbel, index); index < 0: none
struct alignas(16) Partial {
    float M1, s1, Mb, sb;
    float l1, g1; int32_t i1; float l2;
    float g2; int32_t i2; int32_t n_scored, n_drains;   // diagnostics: candidates scored / ring drains in this slice
};
static_assert(sizeof(Partial) == 48, "Partial layout");

// Groups of rows that share one ancestor, built by the plan kernel for the gather kernels.
struct GatherPlan {
    int32_t n_groups[2];          // number of (ancestor, descendants) groups; successive calls alternate the counter
    int32_t bad_anc;              // ancestors outside their prompt's row range (ignored rows)
    int32_t phase;                // counter the NEXT plan uses; flipped on the device by the last workgroup of a plan
    int32_t ticket;               // workgroups of the running plan that have finished
    int32_t pad[3];
};

// What one wave needs to normalise and resample one prompt (a3 + a4).
struct ResampleArgs {
    int N;
    double kappa;
    uint32_t key0, key1;
    int scheme, order;
    int32_t* anc;                 // [R] out: ancestors as global row indices
    int32_t* resampled;           // [B] out
    double* ess_out;              // [B] out, nullable
    double* logZhat;              // [B] in/out, nullable: running log of the normalising-constant estimate
};

// Outputs of a resampling folded into the vocabulary-pass launch.
struct FusedResample { int32_t* anc; int32_t* resampled; double* ess_out; };

// Everything the vocabulary-pass kernel and its tail (row finalizer, optional resampling) take.
struct StepArgs {
    const void* logits; int64_t row_stride_bytes; int V;
    uint32_t key0, key1;
    // the step's scalars by value ...
    uint32_t step; double alpha_t, alpha_prev, beta, tau_by_value;
    // ... or, when d_step is not null, from the device: the step counter and the exponent schedule alpha[0..n_sched)
    const int32_t* d_step; const double* d_sched; int n_sched;
    int n_split, vecs_per_split;
    Partial* partials;            // [R * kMaxSplit]
    int32_t* row_ticket;          // [R] slices of a row that have delivered their record (returns to 0)
    // row state and outputs of the finalizer
    double* logW; double* cumlogp; const int32_t* parity; int32_t* const* histAB; int T_max; int32_t* tokens_out;
    double* d_delta; double* d_logZ1; double* d_logZb; double* d_gap; int32_t* d_second; int32_t* d_rowstat;
    int eos_id; int32_t* done;
    // resampling folded into the same launch
    int fuse_resample;
    int32_t* prompt_ticket;       // [B] rows of a prompt that are final (returns to 0)
    ResampleArgs rs;
};

struct Workspace {                // device pointers carved out of the caller's workspace
    double* logW;                 // [R]
    double* cumlogp;              // [R]
    int32_t* parity;              // [R] which of its two buffers holds a row's live KV / history
    int32_t* done;                // [R] termination flags (Alg. 1)
    double* logZhat;              // [B] log of the product of the mean unnormalised weights at the resampling times
    double* logZest;              // [B] read-out scratch of smc_get_log_zhat
    Partial* partials;            // [R * kMaxSplit]
    int32_t* row_ticket;          // [R] ticket counters of the vocabulary pass (zero between launches)
    int32_t* prompt_ticket;       // [B]
    int32_t* d_step;              // [1] device-resident step counter (smc_set_device_step)
    double* d_sched;              // [T_max + 2] device-resident exponent schedule alpha_0 .. (smc_set_schedule)
    double* d_delta;              // [R] diagnostics of the last step
    double* d_logZ1;              // [R]
    double* d_logZb;              // [R]
    double* d_gap;                // [R]
    int32_t* d_second;            // [R]
    int32_t* d_rowstat;           // [3*R] per row: non-finite flag, candidates scored, ring drains
    GatherPlan* plan;
    int32_t* grp_src;             // [R] ancestor row of each group
    int32_t* grp_base;            // [R] first row of the group's prompt
    int32_t* grp_srcpar;          // [R] which buffer held the ancestor's live row when the plan was made
    unsigned long long* grp_mask; // [R * mask_words] descendants of each group as a bit set over the prompt's rows
    void** kvA;                   // [kv_tensors]
    void** kvB;                   // [kv_tensors]
    void** histAB;                // [2]
};

// Paged form of the KV cache: page numbers per (row, column), reference counts, copy-on-write work list.
struct PagedKV {
    int bound;
    int P, M, Q;                  // positions per page, pages per row, pages per prompt (= N*M)
    int len;                      // positions appended so far (the same for every row)
    int32_t* table;               // [R*M] page of row r for positions [j*P, (j+1)*P), -1 while unused
    int32_t* refcnt;              // [B*Q] rows that reference a page; 0 = free
    int32_t* cow_src;             // [R] source page of each pending copy
    int32_t* cow_dst;             // [R] new page of each pending copy
    int32_t* counters;            // [8] pairs of phase 0 / 1, rows that found no free page, phase, ticket, spare
    int32_t* arrive;              // [B] state workgroups of the running reorder that have finished, per prompt
    int32_t* arrive_table;        // [B] table workgroups of the running reorder that have finished, per prompt
    void** pools;                 // [kv_tensors] page pools [B*Q, H, P, D]
};

}  // namespace psmc

struct smc_ctx {
    smc_config cfg;
    hipStream_t stream;
    psmc::Workspace ws;
    psmc::PagedKV paged;
    int R;
    int n_split;                  // current split of a row over workgroups
    int dense;                    // 1: score every vocabulary entry (no candidate filter)
    int wg_waves;                 // waves per workgroup of the vocabulary pass: 4 or 16
    int mask_words;               // 64-bit words per descendant bit set = ceil(N/64)
    int resampler;                // 0 systematic (the paper's), 1 stratified, 2 multinomial, 3 residual
    int ancestor_order;           // 0 as drawn, 1 survivors stay in place
    int kv_skip_terminated;       // 1: the reorder moves no KV bytes for descendants of a terminated ancestor
    int device_step;              // 1: kernels read the step and the exponents from the device (graph replay advances)
    int n_sched;                  // entries of the device-resident schedule
    int sched_integer_power;      // the integer every schedule entry from index 1 on equals (1..8 except 7), else 0
    int kv_bound;
    std::vector<void*> h_kvA, h_kvB, h_pools;   // host copies of the registered device pointers (kernel arguments)
    int hist_bound;
    int gather_grid;              // workgroups of the persistent gather kernel
    int gather_variant;           // vectors per thread / non-temporal choice of the gather kernel
    int n_cus;
    // optional per-kernel timing: event pairs recorded around launches of kind 0 (vocab pass), 1 (KV gather) and
    // 2 (copy-on-write page copy), 3 (decode attention)
    int profiling;
    std::vector<hipEvent_t> ev_pool[4];   // [2*i] start, [2*i+1] stop
    size_t ev_used[4];
};

namespace psmc {

// Records a start/stop event pair around one kernel launch while profiling is on.
struct ScopedKernelTimer {
    smc_ctx* c; int kind; hipEvent_t stop = nullptr;
    ScopedKernelTimer(smc_ctx* ctx, int k) : c(ctx), kind(k)
    {
        if (!c->profiling) return;
        auto& pool = c->ev_pool[kind];
        if (c->ev_used[kind] + 2 > pool.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
            try { pool.reserve(pool.size() + 2); } catch (...) { (void)hipEventDestroy(a); (void)hipEventDestroy(b); return; }
            pool.push_back(a); pool.push_back(b);
        }
        (void)hipEventRecord(pool[c->ev_used[kind]], c->stream);
        stop = pool[c->ev_used[kind] + 1];
        c->ev_used[kind] += 2;
    }
    ~ScopedKernelTimer() { if (stop) (void)hipEventRecord(stop, c->stream); }
};

// the checks smc_init applies to a configuration
smc_status validate_config(const smc_config* c);

// default launch shape of the vocabulary pass for R rows of V entries: waves per workgroup and workgroups per row
void auto_shape(int R, int V, int dtype, int* wg_waves, int* n_split);

// launchers (each enqueues on ctx->stream; returns hipGetLastError())
hipError_t launch_init_state(smc_ctx* c);
// fused: not null -> the wave that completes a prompt also resamples it (a3 + a4 in the same launch)
hipError_t launch_vocab_pass(smc_ctx* c, const void* logits, int64_t row_stride, int t, double alpha_t,
                             double alpha_prev, double tau_t, int32_t* tokens_out, const FusedResample* fused);
hipError_t launch_advance_step(smc_ctx* c);
int integer_power(double beta);   // the integer-exponent kernel instantiation for beta, or 0 for the generic one
hipError_t launch_ess(smc_ctx* c, const double* logW, double* ess_out, double* lognormw_out);
hipError_t launch_resample(smc_ctx* c, double* logW, int t, int32_t* anc, int32_t* resampled, double* ess_out);
hipError_t launch_reindex(smc_ctx* c, const int32_t* anc, const int32_t* resampled, int valid_len, int t, bool planned = false);
// a3 + a4 and, for the prompts that resample, the plan of the reorder that follows (one launch)
hipError_t launch_resample_plan(smc_ctx* c, double* logW, int t, int32_t* anc, int32_t* resampled, double* ess_out);
hipError_t launch_final_draw(smc_ctx* c, int t, int32_t* choice);
hipError_t launch_log_zhat(smc_ctx* c, double* out);

}  // namespace psmc
