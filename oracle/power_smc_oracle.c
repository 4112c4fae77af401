/*
 * Power-SMC per-token step: CPU oracle (TEST INFRASTRUCTURE, not the product).
 *
 * A plain, slow, dense fp64 implementation of what the hot path computes, written
 * from the paper's definitions so that a reader can check it by eye:
 *   - Algorithm 1 (sample / reweight / ESS / resample / reorder),
 *   - the incremental-weight equation (Eq. "inc"):  omega_t = p(y_t)^alpha / q_t(y_t),
 *   - the ESS formula (Eq. "ess"):                  ESS = 1 / sum_i W_i^2,
 *   - the systematic-resampling rule (Sec. 7, implementation details),
 *   - the exponent-bridging boundary update (Sec. 5.3 / App. B),
 *   - "reindex along the particle dimension" (App. C).
 * Where the paper is silent (how q_t is sampled, which random stream) the reading is:
 * Gumbel-max over the whole vocabulary, one Philox4x32-10 word per vocabulary entry.
 *
 * There is no blocking, fusion, skipping or reordering here: every vocabulary entry
 * draws its random word and evaluates its key, sums run left to right.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may call this file.
 * It shares no code with the HIP library.  OpenMP (if enabled) parallelises over rows only.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* threads the row loops run on (1 without OpenMP) */
int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ Philox4x32-10
 * Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11):
 * 10 rounds; each round multiplies counter words 0 and 2 by two fixed odd constants,
 * permutes hi/lo halves and xors in the key; the key is bumped by Weyl constants
 * between rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random word of vocabulary entry v of row r at step t: word (v mod 4) of the block with
 * counter (v div 4, r, t, domain) and key (seed low, seed high).  domain 0 = token draw,
 * 1 = resampling offset, 2 = final output draw (for both v = 0 and r is the prompt index). */
uint32_t orc_random_word(uint64_t seed, uint32_t t, uint32_t r, uint32_t v, uint32_t domain)
{
    uint32_t ctr[4] = { v >> 2, r, t, domain };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[v & 3u];
}

/* u = (x + 1/2) / 2^32, strictly inside (0,1); exact in fp64. */
double orc_uniform(uint32_t x) { return ((double)x + 0.5) * 0x1p-32; }

/* Standard Gumbel variate g = -log(-log u) for u = orc_uniform(x).
 * For u > 1/2 the inner logarithm is taken as log1p(-(1-u)), with 1-u formed exactly
 * from the complemented word, so no precision is lost near u = 1. */
double orc_gumbel(uint32_t x)
{
    double e;
    if (x < 0x80000000u) {
        e = -log(orc_uniform(x));
    } else {
        double one_minus_u = ((double)(~x) + 0.5) * 0x1p-32;
        e = -log1p(-one_minus_u);
    }
    return -log(e);
}

/* Exact widening of a stored logit.  dtype 0: bf16 (upper half of an fp32), 1: fp32, 2: fp64. */
static double load_logit(const void* base, int dtype, int64_t i)
{
    if (dtype == 0) {
        uint32_t bits = (uint32_t)((const uint16_t*)base)[i] << 16;
        float f; memcpy(&f, &bits, 4); return (double)f;
    } else if (dtype == 1) {
        return (double)((const float*)base)[i];
    }
    return ((const double*)base)[i];
}

/* log sum_v exp(scale * x_v), max-shifted, summed left to right. */
static double lse_scaled(const void* x, int dtype, int64_t n, double scale)
{
    double m = -INFINITY;
    for (int64_t v = 0; v < n; ++v) { double z = scale * load_logit(x, dtype, v); if (z > m) m = z; }
    double s = 0.0;
    for (int64_t v = 0; v < n; ++v) s += exp(scale * load_logit(x, dtype, v) - m);
    return m + log(s);
}
double orc_logsumexp(const double* x, int64_t n, double scale) { return lse_scaled(x, 2, n, scale); }

/* One particle's vocabulary pass (Alg. 1, the "sample" and "update" lines; Eq. "inc").
 *   logits : V entries of the given dtype;  beta = 1/tau_t;  alpha = alpha_t.
 *   forced : >= 0 replaces the sampled token (used only by tests of the weight identity).
 * out[0]=token  out[1]=runner-up token (or -1)
 * res[0]=log Z_1 = LSE(l)   res[1]=log Z_beta = LSE(beta*l)   res[2]=log p(y)  res[3]=log q(y)
 * res[4]=increment alpha*log p(y) - log q(y)   res[5]=gap between best and runner-up key */
void orc_vocab_row(const void* logits, int dtype, int32_t V, double beta, double alpha,
                   uint64_t seed, int32_t t, int32_t r, int32_t forced,
                   int32_t out[2], double res[6])
{
    double logZ1 = lse_scaled(logits, dtype, V, 1.0);
    double logZb = lse_scaled(logits, dtype, V, beta);
    double best = -INFINITY, second = -INFINITY;
    int32_t ibest = -1, isecond = -1;
    for (int32_t v = 0; v < V; ++v) {
        double g = orc_gumbel(orc_random_word(seed, (uint32_t)t, (uint32_t)r, (uint32_t)v, 0));
        double key = beta * load_logit(logits, dtype, v) + g;
        if (key > best) { second = best; isecond = ibest; best = key; ibest = v; }  /* strict: lowest v wins ties */
        else if (key > second) { second = key; isecond = v; }
    }
    int32_t y = forced >= 0 ? forced : ibest;
    double ly = load_logit(logits, dtype, y);
    double logp = ly - logZ1;
    double logq = beta * ly - logZb;
    out[0] = y; out[1] = isecond;
    res[0] = logZ1; res[1] = logZb; res[2] = logp; res[3] = logq;
    res[4] = alpha * logp - logq;
    res[5] = best - second;
}

/* Steps a0..a2 for all R rows: boundary reweight (Sec. 5.3), sample, increment, bookkeeping, and the absorbing
 * terminated state (Alg. 1 "if done ... else ..."; App. D).
 *   logits [R, row_stride] of dtype; logW, cumlogp [R] in/out; hist [R, T_max] (column t-1 written);
 *   tokens, second [R], gap [R], delta [R] out (second/gap/delta may be NULL).
 *   eos_id >= 0 with done != NULL: a particle with done[r] != 0 emits eos_id and keeps its weight (increment 1);
 *   a particle that samples eos_id becomes done.  The stage-boundary reweight acts on every particle, terminated
 *   or not: it re-targets the whole prefix distribution from exponent alpha_{t-1} to alpha_t (App. B). */
void orc_step(const void* logits, int dtype, int64_t row_stride, int32_t R, int32_t V,
              double alpha_t, double alpha_prev, double beta, uint64_t seed, int32_t t,
              double* logW, double* cumlogp, int32_t* hist, int32_t T_max,
              int32_t* tokens, int32_t* second, double* gap, double* delta,
              int32_t eos_id, int32_t* done)
{
    int esz = dtype == 0 ? 2 : (dtype == 1 ? 4 : 8);
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t r = 0; r < R; ++r) {
        const void* row = (const char*)logits + (int64_t)r * row_stride * esz;
        int32_t o[2]; double res[6];
        logW[r] += (alpha_t - alpha_prev) * cumlogp[r];           /* stage boundary, prefix y_{1:t-1} */
        if (done && eos_id >= 0 && done[r]) {                      /* absorbing: y_t = EOS, weight kept */
            tokens[r] = eos_id;
            if (hist) hist[(int64_t)r * T_max + (t - 1)] = eos_id;
            if (second) second[r] = -1;
            if (gap) gap[r] = INFINITY;
            if (delta) delta[r] = 0.0;
            continue;
        }
        orc_vocab_row(row, dtype, V, beta, alpha_t, seed, t, r, -1, o, res);
        logW[r] += res[4];
        cumlogp[r] += res[2];
        if (hist) hist[(int64_t)r * T_max + (t - 1)] = o[0];
        tokens[r] = o[0];
        if (second) second[r] = o[1];
        if (gap) gap[r] = res[5];
        if (delta) delta[r] = res[4];
        if (done && eos_id >= 0 && o[0] == eos_id) done[r] = 1;
    }
}

/* Step a3 (Alg. 1 "normalize ... compute ESS"; Eq. "ess") for B independent prompts of N particles:
 * W_i = exp(logW_i - L1), L1 = LSE_i(logW);  ESS = 1/sum W_i^2 evaluated as exp(2 L1 - L2), L2 = LSE_i(2 logW). */
void orc_ess(const double* logW, int32_t B, int32_t N, double* ess, double* lognormw)
{
    for (int32_t b = 0; b < B; ++b) {
        const double* lw = logW + (int64_t)b * N;
        double L1 = orc_logsumexp(lw, N, 1.0);
        double L2 = orc_logsumexp(lw, N, 2.0);
        ess[b] = exp(2.0 * L1 - L2);
        if (lognormw) for (int32_t i = 0; i < N; ++i) lognormw[(int64_t)b * N + i] = lw[i] - L1;
    }
}

/* Systematic resampling of one prompt (Sec. 7): positions p_i = (u0 + i)/N for i = 0..N-1 (the paper's
 * (u0 + i - 1)/N with 1-based i), A_i = min{ j : sum_{k<=j} w_k >= p_i }; N-1 if rounding leaves none. */
void orc_systematic(const double* w, int32_t N, double u0, int32_t* A)
{
    for (int32_t i = 0; i < N; ++i) {
        double p = (u0 + (double)i) / (double)N;
        double c = 0.0; int32_t a = N - 1;
        for (int32_t j = 0; j < N; ++j) { c += w[j]; if (c >= p) { a = j; break; } }
        A[i] = a;
    }
}

/* First index whose running sum reaches p (sums taken left to right); n-1 if rounding leaves none. */
static int32_t invert_cumulative(const double* w, int32_t n, double p)
{
    double c = 0.0;
    for (int32_t j = 0; j < n; ++j) { c += w[j]; if (c >= p) return j; }
    return n - 1;
}

/* The resampling schemes App. E names as equally valid (all unbiased: E[#copies of j] = N w_j), in their textbook
 * form (Doucet & Johansen's tutorial, the reference App. E cites).  u_i is the uniform of word i of the prompt's
 * resampling stream (Philox domain 1, row := prompt b).
 *   0 systematic : p_i = (u_0 + i)/N                      (Sec. 7; one uniform)
 *   1 stratified : p_i = (u_i + i)/N                      (one uniform per stratum)
 *   2 multinomial: p_i = u_i                               (N independent draws, ancestors in draw order)
 *   3 residual   : floor(N w_j) copies of each j in index order, then the remaining N - sum floor(.) ancestors are
 *                  multinomial draws p_i = u_i from the residual weights (N w_j - floor(N w_j)) / remaining
 * A_i = first index whose running sum of the weights used reaches p_i. */
void orc_resample_scheme(const double* w, int32_t N, int32_t scheme, uint64_t seed, int32_t t, int32_t b,
                         int32_t* A, double* scratch)
{
    if (scheme == 0) {
        orc_systematic(w, N, orc_uniform(orc_random_word(seed, (uint32_t)t, (uint32_t)b, 0, 1)), A);
    } else if (scheme == 1 || scheme == 2) {
        for (int32_t i = 0; i < N; ++i) {
            double u = orc_uniform(orc_random_word(seed, (uint32_t)t, (uint32_t)b, (uint32_t)i, 1));
            double p = scheme == 1 ? (u + (double)i) / (double)N : u;
            A[i] = invert_cumulative(w, N, p);
        }
    } else {
        int32_t k = 0;
        for (int32_t j = 0; j < N; ++j) {
            double nw = (double)N * w[j];
            int32_t copies = (int32_t)floor(nw);
            scratch[j] = nw - (double)copies;
            for (int32_t c = 0; c < copies && k < N; ++c) A[k++] = j;
        }
        int32_t rest = N - k;
        if (rest > 0) {
            for (int32_t j = 0; j < N; ++j) scratch[j] /= (double)rest;
            for (int32_t i = 0; i < rest; ++i) {
                double u = orc_uniform(orc_random_word(seed, (uint32_t)t, (uint32_t)b, (uint32_t)i, 1));
                A[k++] = invert_cumulative(scratch, N, u);
            }
        }
    }
}

/* Survivors stay in place: a permutation of the ancestor vector A (same multiset of ancestors) in which every
 * distinct ancestor j keeps slot j.  After resampling all weights are equal and nothing in Alg. 1 depends on a
 * particle's index, so the particle system is the same; only the slots that really change owner have to be copied.
 * Rule: each distinct ancestor takes its own slot; the remaining copies, in the order they occur in A (the first
 * occurrence of each ancestor is the one that stayed), fill the free slots in increasing order. */
void orc_survivors_in_place(const int32_t* A, int32_t N, int32_t* out)
{
    int32_t seen[N];
    for (int32_t k = 0; k < N; ++k) { out[k] = -1; seen[k] = 0; }
    for (int32_t i = 0; i < N; ++i) out[A[i]] = A[i];
    int32_t free_slot = 0;
    for (int32_t i = 0; i < N; ++i) {
        int32_t a = A[i];
        if (!seen[a]) { seen[a] = 1; continue; }
        while (out[free_slot] != -1) ++free_slot;
        out[free_slot] = a;
    }
}

/* Step a4 for B prompts: trigger ESS < kappa*N (strict), ancestors by the chosen scheme (0 = the paper's
 * systematic resampling) as global row indices, weights of resampled prompts reset to 1 (logW = 0).
 * Prompts that do not resample get the identity.  scratch_w: 2N doubles.  in_place != 0 reorders each ancestor
 * vector with orc_survivors_in_place. */
void orc_resample(double* logW, int32_t B, int32_t N, double kappa, uint64_t seed, int32_t t,
                  int32_t* anc, int32_t* resampled, double* ess_out, double* scratch_w, int32_t scheme,
                  int32_t in_place)
{
    for (int32_t b = 0; b < B; ++b) {
        double* lw = logW + (int64_t)b * N;
        double L1 = orc_logsumexp(lw, N, 1.0);
        double L2 = orc_logsumexp(lw, N, 2.0);
        double ess = exp(2.0 * L1 - L2);
        if (ess_out) ess_out[b] = ess;
        if (ess < kappa * (double)N) {
            int32_t A[N], P[N];
            for (int32_t i = 0; i < N; ++i) scratch_w[i] = exp(lw[i] - L1);
            orc_resample_scheme(scratch_w, N, scheme, seed, t, b, A, scratch_w + N);
            if (in_place) { orc_survivors_in_place(A, N, P); for (int32_t i = 0; i < N; ++i) A[i] = P[i]; }
            for (int32_t i = 0; i < N; ++i) { anc[(int64_t)b * N + i] = b * N + A[i]; lw[i] = 0.0; }
            resampled[b] = 1;
        } else {
            for (int32_t i = 0; i < N; ++i) anc[(int64_t)b * N + i] = b * N + i;
            resampled[b] = 0;
        }
    }
}

/* Step a5 (Alg. 1 "reorder ... by A"; App. C): dst[k] = src[anc[k]] along the particle dimension for one
 * tensor laid out [R, H, S, D] with elem_bytes per entry; only the first valid_len of the S positions of
 * every head are copied, and only for rows k whose prompt (k div N) has resampled != 0. */
void orc_gather_kv(const void* src, void* dst, const int32_t* anc, const int32_t* resampled,
                   int32_t R, int32_t N, int32_t H, int32_t S, int32_t D, int32_t elem_bytes, int32_t valid_len)
{
    int64_t head_stride = (int64_t)S * D * elem_bytes, row_stride = head_stride * H;
    int64_t n = (int64_t)valid_len * D * elem_bytes;
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < R; ++k) {
        if (!resampled[k / N]) continue;
        for (int32_t h = 0; h < H; ++h)
            memcpy((char*)dst + k * row_stride + h * head_stride,
                   (const char*)src + (int64_t)anc[k] * row_stride + h * head_stride, (size_t)n);
    }
}

/* Same gather for the small per-particle state: token history (first t columns), cumulative log p, and the
 * termination flags (Alg. 1: done^(k) <- done^(A_k); done_src / done_dst may be NULL). */
void orc_gather_state(const int32_t* hist_src, int32_t* hist_dst, int32_t T_max, int32_t t,
                      const double* cum_src, double* cum_dst,
                      const int32_t* anc, const int32_t* resampled, int32_t R, int32_t N,
                      const int32_t* done_src, int32_t* done_dst)
{
    for (int32_t k = 0; k < R; ++k) {
        if (!resampled[k / N]) { cum_dst[k] = cum_src[k]; if (done_src) done_dst[k] = done_src[k]; continue; }
        memcpy(hist_dst + (int64_t)k * T_max, hist_src + (int64_t)anc[k] * T_max, (size_t)t * 4);
        cum_dst[k] = cum_src[anc[k]];
        if (done_src) done_dst[k] = done_src[anc[k]];
    }
}

/* Output of Alg. 1: I ~ Categorical(W_T) per prompt, by inversion of the cumulative normalised weights with one
 * uniform from the Philox stream (domain 2): I = min{ j : sum_{k<=j} W_k >= u }, N-1 if rounding leaves none.
 * choice[b] is the global row index b*N + I. */
void orc_final_draw(const double* logW, int32_t B, int32_t N, uint64_t seed, int32_t t, int32_t* choice)
{
    for (int32_t b = 0; b < B; ++b) {
        const double* lw = logW + (int64_t)b * N;
        double L1 = orc_logsumexp(lw, N, 1.0);
        double u = orc_uniform(orc_random_word(seed, (uint32_t)t, (uint32_t)b, 0, 2));
        double c = 0.0; int32_t pick = N - 1;
        for (int32_t j = 0; j < N; ++j) { c += exp(lw[j] - L1); if (c >= u) { pick = j; break; } }
        choice[b] = b * N + pick;
    }
}
