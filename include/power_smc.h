/*
 * power_smc.h -- C ABI of the MI355X (gfx950) Power-SMC per-token step.
 *
 * The library implements what Algorithm 1 of the Power-SMC paper adds on top of one batched decode
 * step, for B independent prompts with N particles each (R = B*N rows, row r = b*N + i):
 *
 *   a0  stage-boundary reweight of exponent bridging (Sec. 5.3, App. B)
 *   a1  draw y ~ q_t = softmax(l / tau_t)                     (Alg. 1 "sample"; Cor. 1)
 *       (a terminated particle emits EOS and keeps its weight: Alg. 1 "if done", App. D)
 *   a2  log W~ += alpha_t log p(y) - log q_t(y)               (Eq. "inc"; Alg. 1 "update")
 *   a3  W = W~ / sum W~ ,  ESS = 1 / sum W^2   per prompt      (Eq. "ess")
 *   a4  if ESS < kappa N: systematic resampling -> ancestors  (Alg. 1; Sec. 7 implementation details)
 *   a5  prefixes, cumulative log p and KV cache gathered by ancestor (Alg. 1 "reorder"; App. C)
 *
 * Conventions shared by every call
 *   - "d_" arguments are DEVICE pointers, "h_" arguments are HOST pointers.  All are caller-owned; the
 *     library allocates no device memory (the caller passes a workspace of smc_workspace_bytes()).
 *   - Calls enqueue kernels on the HIP stream given to smc_init and return without synchronising,
 *     except smc_get_state / smc_set_state / smc_get_diag / smc_kv_bind, which are synchronous.
 *   - Every call returns an smc_status.  Argument errors are detected on the host before anything is
 *     enqueued and leave all state untouched.  Nothing throws or aborts.
 *   - One context per stream; a context is not thread-safe.
 *
 * Random numbers: Philox4x32-10 (Salmon et al., SC'11), key = (seed low word, seed high word), counter =
 * (v div 4, row, step t, domain); the word for vocabulary entry v is word (v mod 4) of that block.
 * domain 0 = token draw, domain 1 = resampling offset (row := prompt index, v := 0).
 * A word x maps to u = (x + 1/2) / 2^32 in (0,1).  (The paper does not fix the sampler; this is the
 * library's definition.)
 */
#ifndef POWER_SMC_H
#define POWER_SMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct smc_ctx smc_ctx; /* opaque, lives in host memory */

typedef enum {
    SMC_OK = 0,
    SMC_E_NULL = 1,   /* a required pointer is null */
    SMC_E_SHAPE = 2,  /* a size is non-positive or exceeds a documented limit */
    SMC_E_DTYPE = 3,  /* unknown logits dtype / unsupported element size */
    SMC_E_ALIGN = 4,  /* a pointer or stride is not 16-byte aligned */
    SMC_E_RANGE = 5,  /* a scalar is outside its domain (t, valid_len, alpha, kappa) */
    SMC_E_STATE = 6,  /* call not valid in the context's state (e.g. KV not bound) */
    SMC_E_HIP = 7     /* the HIP runtime reported an error */
} smc_status;

typedef enum { SMC_BF16 = 0, SMC_F32 = 1 } smc_dtype;

enum { SMC_MAX_PARTICLES = 1024, SMC_MAX_KV_TENSORS = 512, SMC_NOALLOC_MAX_ROWS = 4096 };

typedef struct {
    int32_t B;             /* prompts                                  >= 1 */
    int32_t N;             /* particles per prompt (Alg. 1 input N)    1..SMC_MAX_PARTICLES */
    int32_t V;             /* vocabulary size                          >= 1 */
    int32_t T_max;         /* capacity of the token history (Alg. 1 input T_max); multiple of 4 */
    int32_t logits_dtype;  /* smc_dtype */
    int32_t eos_id;        /* end-of-sequence token (absorbing state, App. D); -1: no token terminates a particle */
    double  kappa;         /* resample iff ESS < kappa*N (strict), 0 <= kappa <= 1 (kappa = 0: never) */
    uint64_t seed;         /* Philox key */
    /* KV cache geometry: kv_tensors tensors (2 per layer), each [R, kv_H, kv_S, kv_D] of kv_elem_bytes;
     * kv_D*kv_elem_bytes must be a multiple of 16.  kv_tensors = 0: no cache is managed. */
    int32_t kv_tensors, kv_H, kv_S, kv_D, kv_elem_bytes;
    int32_t reserved1;
} smc_config;

/* Bytes of device scratch + state the caller must provide to smc_init (0 on an invalid config). */
size_t smc_workspace_bytes(const smc_config* cfg);

/* Creates a context.  d_workspace: device memory, 256-byte aligned, >= smc_workspace_bytes(cfg), owned
 * by the caller and left alone by it until smc_destroy.  hip_stream: a hipStream_t (NULL = default stream).
 * Enqueues the initialisation of Alg. 1: log W~ = 0, cumulative log p = 0, every row live in buffer A. */
smc_status smc_init(const smc_config* cfg, void* d_workspace, size_t workspace_bytes, void* hip_stream,
                    smc_ctx** out_ctx);

/* Frees the host-side context (device memory stays with the caller).  Synchronises the stream. */
smc_status smc_destroy(smc_ctx* ctx);

/* Registers the double-buffered caches (App. C).  h_bufA / h_bufB: host arrays of kv_tensors device pointers
 * (16-byte aligned, each tensor [R, kv_H, kv_S, kv_D]); d_histA / d_histB: device int32 [R, T_max] token
 * histories (may both be NULL: no history is kept).  h_bufA and h_bufB may both be NULL: no dense cache is
 * registered (the cache is paged, see smc_paged_bind, or absent) and only the histories are.  Row k's live data is in buffer A while parity[k] = 0 and in
 * buffer B while parity[k] = 1; smc_kv_reindex reads live buffers, writes the inactive buffer of every row that
 * receives another row's data, and flips the parity of exactly those rows (smc_get_state returns the parities).
 * Synchronous (copies the pointer tables into the workspace). */
smc_status smc_kv_bind(smc_ctx* ctx, void* const* h_bufA, void* const* h_bufB, int32_t* d_histA, int32_t* d_histB);

/* Device pointer to the parity words (int32 [R]; 0: the row lives in buffer A, 1: in buffer B): what a decoder needs
 * to append to, or read, the live buffer of each row.  No synchronisation: order reads after the context's stream. */
smc_status smc_kv_parity(smc_ctx* ctx, const int32_t** d_parity);

/* a0 + a1 + a2 for step t (1-based, <= T_max).
 *   d_logits: [R, row_stride_elems] of cfg.logits_dtype, first V entries of each row used; base address and
 *             row stride in bytes must be multiples of 16.
 *   alpha_t, alpha_prev: exponents of this and the previous token (equal when not bridging; >= 0).
 *   tau_t: proposal temperature; tau_t <= 0 selects the locally optimal tau = 1/alpha_t of Thm 1 exactly.
 *   d_tokens_out: int32 [R], the sampled tokens y_t.
 * Updates log W~, cumulative log p and column t-1 of the live history in the workspace.  With eos_id >= 0 a
 * terminated particle's row is not read at all: it emits eos_id, its increment is 1, and only the stage-boundary
 * reweight touches its weight; a particle that draws eos_id becomes terminated. */
smc_status smc_step(smc_ctx* ctx, const void* d_logits, int64_t row_stride_elems, int32_t t, double alpha_t,
                    double alpha_prev, double tau_t, int32_t* d_tokens_out);

/* a0 .. a4 in one call: smc_step followed by smc_resample, with the same arguments, outputs and results as the two
 * calls.  With fewer than 1024 rows it is ONE launch: the workgroup that completes a row finalizes it, and the wave
 * that finalizes the last row of a prompt goes on to normalise and resample that prompt, so no second launch (and no
 * launch gap) is needed.  Larger batches, where a launch is cheap beside the logit stream, take the two launches.
 * Follow it with smc_kv_reindex / smc_paged_reindex on d_anc_out / d_resampled_out as after smc_resample. */
smc_status smc_step_resample(smc_ctx* ctx, const void* d_logits, int64_t row_stride_elems, int32_t t, double alpha_t,
                             double alpha_prev, double tau_t, int32_t* d_tokens_out, int32_t* d_anc_out,
                             int32_t* d_resampled_out, double* d_ess_out);

/* a0 .. a5 in one call: smc_step_resample followed by smc_kv_reindex(d_anc_out, d_resampled_out, valid_len, t), with
 * the same arguments, outputs, results and errors as the two calls -- the whole per-token step of Alg. 1 ("sample",
 * "update", "resample", "reorder KV cache by A") in three launches at every size: with 1024 rows or more, where
 * smc_step_resample takes a launch of its own for the resampling, the wave that resamples a prompt goes on to plan
 * the prompt's reorder, so the plan needs no launch. */
smc_status smc_step_resample_reindex(smc_ctx* ctx, const void* d_logits, int64_t row_stride_elems, int32_t t,
                                     double alpha_t, double alpha_prev, double tau_t, int32_t valid_len,
                                     int32_t* d_tokens_out, int32_t* d_anc_out, int32_t* d_resampled_out,
                                     double* d_ess_out);

/* ---- Step kept on the device: for launch sequences captured once (HIP graph) and replayed every token -----------
 * The step number t and the exponents alpha_t, alpha_{t-1} are launch arguments, so a captured step would redraw the
 * same random numbers on every replay.  With the step kept on the device, the kernels of smc_step, smc_step_resample,
 * smc_resample(_from) and smc_final_draw read t from a counter in the workspace and the exponents from a schedule
 * uploaded beforehand; their t / alpha_t / alpha_prev arguments are then ignored (still validated), and tau_t <= 0
 * means tau = 1/alpha_t of the schedule (tau_t > 0 stays a fixed temperature).  smc_kv_reindex and smc_paged_reindex
 * move whole history rows in this mode (the host does not know t); valid_len stays a launch argument.
 *   smc_set_schedule: h_alpha[0..n) = alpha_0, alpha_1, ... (2 <= n <= T_max + 2; steps beyond n-1 use the last entry;
 *     alpha_0 >= 0, the others > 0).  Synchronous copy.
 *   smc_set_device_step(enable = 1, t): the counter is set to t (the next step to run, 1-based) and the mode switched
 *     on (SMC_E_STATE without a schedule); enable = 0 returns to by-value arguments.  Synchronous.
 *   smc_advance_step: enqueues counter += 1 (one tiny launch, capturable): call it once per token, after the last call
 *     of the token's sequence.
 *   smc_get_device_step: synchronous read of the counter. */
smc_status smc_set_schedule(smc_ctx* ctx, const double* h_alpha, int32_t n);
smc_status smc_set_device_step(smc_ctx* ctx, int32_t enable, int32_t t);
smc_status smc_advance_step(smc_ctx* ctx);
smc_status smc_get_device_step(smc_ctx* ctx, int32_t* h_t);

/* smc_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The same a0 + a1 + a2, the same kernels, but no context and no workspace: the
 * scratch of the vocabulary pass (one 48-byte record per row and slice, per-row diagnostics) lives in a device array
 * inside the library (about 6.6 MB, held by every GPU the library runs on until the process ends), and the state is
 * the caller's:
 *   cfg: as for smc_init (B, N, V, logits_dtype, eos_id, seed are used); B*N <= SMC_NOALLOC_MAX_ROWS, else SMC_E_SHAPE.
 *   hip_stream: the stream to enqueue on (NULL = default stream).
 *   d_logits, row_stride_elems, t (>= 1), alpha_t, alpha_prev, tau_t, d_tokens_out: as for smc_step.
 *   d_logW_inout, d_cumlogp_inout: device double [R], log W~ and cumulative log p, read and updated in place.
 *   d_done_inout: device int32 [R] termination flags, read and updated; required when eos_id >= 0, else ignored.
 * No token history is written.  Calls nothing that allocates (no hipMalloc / hipFree, no workspace); argument errors
 * are detected on the host before anything is enqueued.  Every call on one GPU uses that GPU's one scratch array,
 * which keeps the previous call's contents (only the per-row ticket counters have to start at zero; each call clears
 * them with a small fill kernel first, everything else it reads it has written itself): calls that overlap in time
 * on one GPU -- other streams, other threads -- race on it and must be serialised by the caller. */
smc_status smc_step_noalloc(const smc_config* cfg, void* hip_stream, const void* d_logits, int64_t row_stride_elems,
                            int32_t t, double alpha_t, double alpha_prev, double tau_t, double* d_logW_inout,
                            double* d_cumlogp_inout, int32_t* d_done_inout, int32_t* d_tokens_out);

/* a3 on the context's weights: d_ess_out double [B]; d_lognormw_out double [R] = log W (nullable). */
smc_status smc_ess(smc_ctx* ctx, double* d_ess_out, double* d_lognormw_out);

/* a3 + a4 on the context's weights at step t: d_anc_out int32 [R], ancestor of each row as a global row index
 * (identity for prompts that do not resample); d_resampled_out int32 [B], 1 where ESS < kappa*N;
 * d_ess_out double [B] nullable.  Resets log W~ to 0 for resampled prompts (Alg. 1 "reset"). */
smc_status smc_resample(smc_ctx* ctx, int32_t t, int32_t* d_anc_out, int32_t* d_resampled_out, double* d_ess_out);

/* Resampling scheme used by smc_resample / smc_resample_from: 0 = systematic (the paper's, Sec. 7; default),
 * 1 = stratified, 2 = multinomial, 3 = residual -- the other unbiased schemes App. E names, in their textbook form.
 * Uniform u_i is word i of the prompt's Philox stream of domain 1; positions are (u_0+i)/N, (u_i+i)/N, u_i; residual
 * resampling places floor(N w_j) copies of each j in index order and draws the rest multinomially from the
 * residual weights. */
smc_status smc_set_resampler(smc_ctx* ctx, int32_t scheme);

/* Order of the ancestor vector that smc_resample / smc_resample_from return: 0 = as drawn (default), 1 = survivors
 * stay in place.  After resampling every weight is 1 and nothing in Alg. 1 depends on a particle's index, so any
 * permutation of a prompt's ancestor vector describes the same particle system (the App. C reorder only has to
 * realise the multiset).  Order 1 returns the permutation in which every distinct ancestor j keeps slot j; the
 * remaining copies, in the order in which they were drawn (the first occurrence of each ancestor is the one that
 * stayed), fill the free slots in increasing order.  Then exactly N - #distinct rows change owner and
 * smc_kv_reindex copies only those.  Tokens drawn afterwards differ from order 0 (the random stream is keyed by row
 * slot) but have the same law. */
smc_status smc_set_ancestor_order(smc_ctx* ctx, int32_t order);

/* a5: for every prompt b with d_resampled[b] != 0 and every row k of it with d_anc[k] != k, copies the live row
 * d_anc[k] into the inactive buffer of row k -- the first valid_len (0..kv_S) positions of every head of every KV
 * tensor, the first t columns of the history -- gathers cumulative log p and the termination flags the same way,
 * then flips parity[k].  Rows that are their own ancestor move no bytes.  d_anc entries of a resampled prompt must
 * lie inside that prompt's row range (others are ignored and the row left as it is).  Each distinct ancestor row is
 * read once and written to all of its moved descendants: afterwards the live KV rows equal the gather by ancestor
 * byte for byte.  See smc_set_kv_skip_terminated for the opt-in shortcut for terminated ancestors. */
smc_status smc_kv_reindex(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t valid_len,
                          int32_t t);

/* Opt-in shortcut of smc_kv_reindex (enable = 1; default 0; only acts with eos_id >= 0): the KV rows of a terminated
 * ancestor are not copied (App. D: the absorbing state is a no-op, a terminated particle's cache is never read
 * again).  Its descendants still receive its history, sum and flag and their parity flips like any moved row's, but
 * from then on the content of the KV rows of terminated particles is unspecified.  Late in a run, when most
 * particles have terminated, the reorder then moves almost nothing. */
smc_status smc_set_kv_skip_terminated(smc_ctx* ctx, int32_t enable);

/* Explicit-input forms of a3 / a4 for component checks: same arithmetic on caller-provided weights.
 * smc_resample_from writes the reset weights to d_logW_inout. */
smc_status smc_ess_from(smc_ctx* ctx, const double* d_logW, double* d_ess_out, double* d_lognormw_out);
smc_status smc_resample_from(smc_ctx* ctx, double* d_logW_inout, int32_t t, int32_t* d_anc_out,
                             int32_t* d_resampled_out, double* d_ess_out);

/* Output of Alg. 1: one particle per prompt, I ~ Categorical(W_t), by inversion of the cumulative normalised
 * weights (particle order) with one uniform of the Philox stream (domain 2, row := prompt, v := 0):
 * I = min{ j : sum_{k<=j} W_k >= u }.  d_choice_out int32 [B] receives the global row index b*N + I. */
smc_status smc_final_draw(smc_ctx* ctx, int32_t t, int32_t* d_choice_out);

/* log of the SMC estimate of the normalising constant Z_alpha = sum_y p(y)^alpha of the power target, per prompt
 * (host double [B]; synchronous): smc_resample adds log(mean unnormalised weight) = LSE_i(log W~_i) - log N to a
 * running sum whenever a prompt resamples (Alg. 1 resets the weights there), and this call returns that sum plus the
 * same term of the current weights.  E[exp(.)] = Z_alpha for any N (the estimate is unbiased).  h_banked (host double
 * [B]) receives the running sum alone, which is what smc_set_log_zhat restores when a run is resumed from a saved
 * state.  Either output may be NULL, not both. */
smc_status smc_get_log_zhat(smc_ctx* ctx, double* h_logZhat, double* h_banked);
smc_status smc_set_log_zhat(smc_ctx* ctx, const double* h_banked);

/* Synchronous access to the termination flags (host int32 [R]; only meaningful with eos_id >= 0). */
smc_status smc_get_done(smc_ctx* ctx, int32_t* h_done);
smc_status smc_set_done(smc_ctx* ctx, const int32_t* h_done);

/* Synchronous inspection / teacher forcing (host arrays; any may be NULL to skip):
 * h_logW, h_cumlogp double [R]; h_parity int32 [R]. */
smc_status smc_get_state(smc_ctx* ctx, double* h_logW, double* h_cumlogp, int32_t* h_parity);
smc_status smc_set_state(smc_ctx* ctx, const double* h_logW, const double* h_cumlogp);

/* Synchronous per-row diagnostics of the last smc_step (host arrays of R entries, any may be NULL):
 * increment a2, log Z_1 = LSE(l), log Z_beta = LSE(l/tau), runner-up token, key gap between winner and
 * runner-up (from fp64 keys where the call is closer than 1e-3, else the fp32 estimate that decided it), and h_counters[4] = {rows with non-finite sums, candidates scored, candidate-queue
 * drains, vocabulary entries seen}, all of that one step. */
smc_status smc_get_diag(smc_ctx* ctx, double* h_delta, double* h_logZ1, double* h_logZb, int32_t* h_second,
                        double* h_gap, uint64_t* h_counters);

/* Tuning knobs of the vocabulary pass (defaults chosen at smc_init): n_split = workgroups a row is split over
 * (1..32; 0 = automatic); dense = 1 scores every entry instead of only those that can win (dense = 0, the default,
 * which itself scores whole 16-byte vectors in place where most of their entries can still win);
 * wg_waves = waves per workgroup, 4, 8 or 16 (0 = automatic).  Every setting returns the same tokens. */
smc_status smc_set_tuning(smc_ctx* ctx, int32_t n_split, int32_t dense, int32_t wg_waves);

/* Tuning knobs of the KV gather: persistent workgroups per compute unit (1..64) and the kernel variant
 * (0..10: 16-byte vectors in flight per thread in {8,4,16,2} crossed with non-temporal loads/stores on or off;
 * the default is 4 workgroups per compute unit and variant 4).  Every setting moves the same bytes. */
smc_status smc_set_gather_tuning(smc_ctx* ctx, int32_t wgs_per_cu, int32_t variant);

/* ---- Paged form of the reorder (Alg. 1 "reorder KV cache by A"; App. C) --------------------------------------
 * An alternative to smc_kv_bind / smc_kv_reindex for callers whose attention kernels read the cache through a page
 * table.  Positions are stored in pages of page_len positions; tensor i's pool is an array
 * [B*Q, kv_H, page_len, kv_D] of kv_elem_bytes elements (smc_paged_pool_bytes each), Q = N*M pages per prompt,
 * M = ceil(kv_S / page_len) pages per row; prompt b owns pages [b*Q, (b+1)*Q).  The table (int32 [R, M], device)
 * names the page of row r for positions [j*page_len, (j+1)*page_len), -1 while unused.  The reorder copies page
 * numbers; descendants of one ancestor share pages until one of them is appended to (copy-on-write).  The logical
 * content of every row equals what the dense reorder gives.  Rules: a page is free iff no row references it; rows
 * that need a page take their prompt's free pages in increasing page order, the rows in increasing row order; of
 * the rows that share the page about to be appended to, the lowest keeps it. */

/* Bytes of device workspace smc_paged_bind needs / bytes of one tensor's pool; 0 if the geometry is invalid
 * (kv_tensors < 1, page_len outside 1..kv_S, kv_D*kv_elem_bytes not a multiple of 16). */
size_t smc_paged_workspace_bytes(const smc_config* cfg, int32_t page_len);
size_t smc_paged_pool_bytes(const smc_config* cfg, int32_t page_len);

/* h_pools: host array of kv_tensors device pointers (16-byte aligned, caller-owned, contents never cleared);
 * d_workspace: 256-byte aligned device memory of at least smc_paged_workspace_bytes, owned by the caller and used
 * until smc_destroy.  The table starts in the state that len0 (0..kv_S) appends with no resampling would leave:
 * table[b*N+k, j] = b*Q + j*N + k for j < ceil(len0/page_len).  Synchronises the stream. */
smc_status smc_paged_bind(smc_ctx* ctx, void* const* h_pools, int32_t page_len, void* d_workspace,
                          size_t workspace_bytes, int32_t len0);

/* To be called before the decoder writes position pos (0-based; must equal the number of positions appended so far,
 * else SMC_E_STATE) of every row: gives every row a page of its own for that position -- a fresh page at a page
 * start, otherwise a fresh page plus a copy of the pos % page_len positions already filled for every sharer of a
 * page but the lowest -- and writes d_slot_out int32 [R]: the page of each row; the decoder stores K/V of the new
 * position at pool[page, h, pos % page_len, :].  The number of appended positions is host-side state of the context:
 * the call returns SMC_E_STATE while its stream is being captured into a HIP graph (a replay would repeat `pos`). */
smc_status smc_paged_prepare_append(smc_ctx* ctx, int32_t pos, int32_t* d_slot_out);

/* a5 in paged form: for prompts with d_resampled[b] != 0, table[k, :] = old table[d_anc[k], :] over the columns in
 * use and reference counts recounted; token history (first t columns), cumulative log p and termination flags are
 * gathered as in smc_kv_reindex.  Ancestors outside the prompt's rows leave the row as it is.  Under stream capture
 * all columns of the table are permuted (unused ones hold -1 everywhere), so a captured reorder stays valid on
 * replays that follow later appends; `t` is baked into the capture like any launch argument. */
smc_status smc_paged_reindex(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t t);

/* smc_paged_reindex followed by smc_paged_prepare_append(next_pos, d_slot_out), with the same arguments, results and
 * errors as the two calls, in one launch less: the table workgroup that finishes a prompt's reorder last goes on to
 * prepare that prompt for next_pos (for a prompt that did not resample, its first table workgroup does).  In a
 * decode loop the reorder after token t and the preparation for the next position are adjacent, and with a paged
 * cache the step is a chain of short dependent launches, so each launch saved is several microseconds.  Returns
 * SMC_E_STATE under stream capture, like smc_paged_prepare_append.  A convenience beside the paper's reorder
 * (Alg. 1 "reorder KV cache by A"; App. C), not an operation of its own. */
smc_status smc_paged_reindex_prepare(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t t,
                                     int32_t next_pos, int32_t* d_slot_out);

/* Device pointers to the table [R, M] and the reference counts [B*Q], M, Q and the number of appended positions
 * (each nullable).  No synchronisation: reads of the device arrays must be ordered after the context's stream. */
smc_status smc_paged_view(smc_ctx* ctx, const int32_t** d_table, const int32_t** d_refcnt, int32_t* pages_per_row,
                          int32_t* pages_per_prompt, int32_t* len);

/* Synchronises and returns how many rows ever found no free page (always 0 unless the table was overwritten). */
smc_status smc_paged_check(smc_ctx* ctx, int32_t* h_alloc_failures);

/* ---- Decode attention over the caches the reorder maintains -------------------------------------------------
 * Not part of the paper's method: the reader a decoder needs so that neither cache layout has to be repacked.
 * For every row r, KV head h and query head g of its group (G = n_q_heads / kv_H <= 16):
 *   out[r, h*G+g, :] = sum_j softmax_j(scale * <q[r, h*G+g, :], K[r, h, j, :]>) V[r, h, j, :],  j < len,
 * with K = KV tensor k_tensor and V = KV tensor v_tensor of the context (bf16, kv_D = 64 or 128), read from the
 * paged pools through the page table if smc_paged_bind was called (then len <= positions appended), else from the
 * live buffer of each row of the tensors given to smc_kv_bind.  d_q: bf16 [R, n_q_heads, kv_D]; d_out: float
 * [R, n_q_heads, kv_D]; both 16-byte aligned.  d_workspace: at least smc_attn_workspace_bytes (0 = invalid
 * geometry), 16-byte aligned, scratch for this call only.  Enqueues on the context's stream.  With eos_id >= 0 the
 * rows of terminated particles are not read and their output is 0 (App. D: the absorbing state is a no-op). */
size_t smc_attn_workspace_bytes(const smc_config* cfg, int32_t n_q_heads);
smc_status smc_attn_decode(smc_ctx* ctx, int32_t k_tensor, int32_t v_tensor, const void* d_q, int32_t n_q_heads,
                           int32_t len, float scale, void* d_workspace, size_t workspace_bytes, float* d_out);

/* The store a decoder makes before it attends: writes position pos of every row of KV tensor k_tensor (and of
 * v_tensor unless it is -1) where that row's data lives -- the row's live buffer (dense) or the page that
 * smc_paged_prepare_append gave it (paged: pos must be below the number of appended positions, else SMC_E_STATE).
 * d_k_new / d_v_new: device, bf16 [R, kv_H, kv_D], rows k_row_stride / v_row_stride elements apart (>= kv_H*kv_D,
 * multiples of 8; pointers 16-byte aligned, else SMC_E_ALIGN), read only.  0 <= pos < kv_S.  Terminated rows are
 * written like any other.  Enqueues one launch on the context's stream.  Not part of the paper's method. */
smc_status smc_kv_append(smc_ctx* ctx, int32_t k_tensor, int32_t v_tensor, const void* d_k_new, int64_t k_row_stride,
                         const void* d_v_new, int64_t v_row_stride, int32_t pos);

/* Optional timing of the dominant kernels.  While enabled, a pair of HIP events is recorded on the context's
 * stream around every launch of kind 0 (the vocabulary-pass kernel of smc_step), kind 1 (the KV gather kernel of
 * smc_kv_reindex), kind 2 (the page copy of smc_paged_prepare_append) and kind 3 (the attention kernel of
 * smc_attn_decode).  smc_profile_read synchronises the stream, returns the summed elapsed milliseconds and the number
 * of launches of that kind since the last read, and clears them.  Events are host objects; no device memory is used. */
smc_status smc_profile_enable(smc_ctx* ctx, int32_t enable);
smc_status smc_profile_read(smc_ctx* ctx, int32_t kind, double* h_total_ms, int64_t* h_launches);

/* Measurement helper, not part of the method: the bandwidth a plain streaming kernel reaches on this device over
 * d_buf (16-byte aligned device memory, bytes >= 1 MiB and a multiple of 64; contents are overwritten), with the
 * read : write mix of kind 0 = read only, 1 = write only, 2 = copy 1:1 (first half to second half), 3 = one read
 * fanned out to three writes.  Runs one warm-up and three timed launches on the given stream, synchronises, and
 * returns bytes moved per second in GB/s.  A second, measured denominator beside the published HBM peak. */
smc_status smc_hbm_probe(int32_t kind, void* d_buf, size_t bytes, void* hip_stream, double* h_gbps);

const char* smc_status_str(smc_status s);

#ifdef __cplusplus
}
#endif
#endif /* POWER_SMC_H */
