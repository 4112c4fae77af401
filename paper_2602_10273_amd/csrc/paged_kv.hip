// Paged (block-table) form of the cache reorder after resampling (Alg. 1 "reorder KV cache by A"; App. C: reindex
// along the batch/particle dimension) for gfx950.
//
// The dense reorder copies whole cache rows.  Here a row's cache is a list of pages of P positions, table[r, j] being
// the page that holds positions [j*P, (j+1)*P) of row r, and the reorder copies page NUMBERS: descendants of one
// ancestor share its pages.  Before position pos is written every row must own its page for that position alone:
// at a page start every row takes a fresh page; otherwise, of the rows that share a page the lowest keeps it and each
// of the others takes a fresh page and receives a copy of the pos % P positions already filled (copy-on-write).
// A reorder therefore moves kilobytes of page numbers, and an append at most (N-1)*(P-1) positions per prompt,
// instead of the whole cache.
//
// Prompt b owns the page numbers [b*Q, (b+1)*Q), Q = N*M, M = ceil(S/P): at most N*M distinct pages can be referenced
// by a prompt, so its pool never runs out.  A page is free iff its reference count is 0; needy rows, in increasing
// row order, take the free pages of their prompt in increasing page order.  These rules are deterministic, so the
// tables can be compared bit for bit with a CPU model that follows them.
//
//   paged_init_kernel     : the state after len0 appends with no resampling (table[b*N+k, j] = b*Q + j*N + k)
//   paged_reorder_kernel  : table[k, :] = old table[anc[k], :]; old row a's pages gain copies(a) - 1 references;
//                           token histories, cumulative log p and termination flags follow in the same launch
//   paged_prepare_kernel  : one workgroup per prompt; finds the needy rows, the lowest free pages, writes the slot of
//                           every row and the list of (source page, new page) pairs.  The reorder can do the same for
//                           the next position in its own launch: the table workgroup that finishes a prompt last
//                           goes on to prepare it
//   paged_copy_kernel     : grid-stride over (pair, tensor): 16-byte vector copy of the filled part of a page
#include "smc_internal.hpp"

namespace psmc {

namespace {
constexpr int kPagedThreads = 256;
constexpr int kEntriesPerBlock = 2048;               // table entries one workgroup of the reorder handles (>= SMC_MAX_PARTICLES)
static_assert(kEntriesPerBlock >= SMC_MAX_PARTICLES, "one column of a prompt must fit in a workgroup's LDS tile");
constexpr int kScanPerThread = 32;                  // reference counts one thread examines per sweep of the free-page search
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));

// Exclusive prefix sum of one int per thread over the 256-thread workgroup; `total` is the sum over all threads.
__device__ inline int block_exclusive_scan(int v, int32_t* sh_wave, int& total)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    int inc = v;
    for (int o = 1; o < kWave; o <<= 1) {
        const int x = __shfl_up(inc, o);
        if (lane >= o) inc += x;
    }
    __syncthreads();                                   // previous use of sh_wave is over
    if (lane == kWave - 1) sh_wave[wave] = inc;
    __syncthreads();
    int before = 0;
    total = 0;
    for (int w = 0; w < kPagedThreads / kWave; ++w) {
        const int s = sh_wave[w];
        if (w < wave) before += s;
        total += s;
    }
    return before + inc - v;
}
}  // namespace

__global__ void paged_init_kernel(int R, int N, int M, int Q, int P, int len0, int32_t* __restrict__ table,
                                  int32_t* __restrict__ refcnt, int32_t* __restrict__ counters,
                                  int32_t* __restrict__ arrive, int32_t* __restrict__ arrive_table)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int ncol = (len0 + P - 1) / P;
    if (i < (int64_t)R * M) {
        const int r = (int)(i / M), j = (int)(i % M);
        const int b = r / N, k = r % N;
        table[i] = j < ncol ? b * Q + j * N + k : -1;
    }
    if (i < (int64_t)(R / N) * Q) refcnt[i] = (int)(i % Q) < ncol * N ? 1 : 0;
    if (i < 8) counters[i] = 0;                        // pair counters of the two phases, failures, phase, ticket
    if (i < R / N) { arrive[i] = 0; arrive_table[i] = 0; }
}

// What the preparation of one position needs besides the table itself.
struct PrepareArgs {
    int j, o;                     // page column and offset of the position
    int32_t* counters; int32_t* cow_src; int32_t* cow_dst; int32_t* slot;
};

__device__ void prepare_prompt(int b, int n_prompts, int N, int M, int Q, const PrepareArgs& pa,
                               int32_t* __restrict__ table, int32_t* __restrict__ refcnt);

// The reorder in one launch.  Two kinds of workgroup, told apart by blockIdx:
//
// state workgroups (hb per prompt): token history (first hist_vecs 16-byte vectors of a row), cumulative log p and
//   termination flags follow their ancestors exactly as in the dense reorder -- a moved row receives its ancestor's
//   live history in its own inactive buffer, then its parity flips.  Every workgroup of a prompt first reads the
//   prompt's ancestors, parities, sums and flags, copies its share of the history vectors and takes a ticket; the one
//   with the last ticket writes sums, flags and parities (nobody reads them any more) and clears the ticket counter.
//
// table workgroups: table[k, j] = old table[anc[k], j].  Old row a's page for column j gains copies(a) - 1
//   references, copies(a) being the number of rows that continue a; a page whose count reaches 0 is free from then on.
//   The permutation acts along the rows and every column is permuted on its own, so one workgroup takes all N rows of
//   `cols` columns of one prompt: it reads them into LDS, then writes them back permuted -- no other workgroup touches
//   these entries, so no copy of the old table is needed.  N * cols <= kEntriesPerBlock.
//   With `prepare` set, the table workgroup of a prompt that finishes last (a ticket per prompt; for a prompt that did
//   not resample, its first table workgroup) goes on to prepare the prompt for the next position, as
//   paged_prepare_kernel would in a launch of its own.
__global__ __launch_bounds__(kPagedThreads) void paged_reorder_kernel(
    const int32_t* __restrict__ anc, const int32_t* __restrict__ resampled, int B, int N,
    int hb, int hist_vecs, long long hist_row_bytes, int32_t* const* __restrict__ histAB, double* __restrict__ cumlogp,
    int32_t* __restrict__ done, int32_t* __restrict__ parity, int32_t* __restrict__ bad_anc, int32_t* __restrict__ arrive,
    int M, int Q, int ncol, int cols, int chunks, int32_t* __restrict__ table, int32_t* __restrict__ refcnt,
    int prepare, PrepareArgs pa, int32_t* __restrict__ arrive_table)
{
    __shared__ int32_t sh_anc[SMC_MAX_PARTICLES];
    __shared__ int32_t sh_aux[SMC_MAX_PARTICLES];      // table: copies of each ancestor; state: parity of each row
    __shared__ int32_t sh_old[kEntriesPerBlock];       // table: the old entries; state: termination flags
    __shared__ double sh_cum[SMC_MAX_PARTICLES];
    __shared__ int sh_last;
    const int tid = threadIdx.x;
    const int n_state = B * hb;
    if ((int)blockIdx.x < n_state) {
        const int b = blockIdx.x / hb, part = blockIdx.x % hb;
        if (!resampled[b]) return;
        const int row0 = b * N;
        int bad = 0;
        for (int k = tid; k < N; k += kPagedThreads) {
            int a = anc[row0 + k] - row0;
            if (a < 0 || a >= N) { a = -1; ++bad; }        // outside the prompt: the row is left untouched
            if (a == k) a = -1;                            // its own ancestor: nothing to move
            sh_anc[k] = a;
            sh_aux[k] = parity[row0 + k];
            sh_cum[k] = cumlogp[row0 + k];
            sh_old[k] = done[row0 + k];
        }
        if (part == 0 && bad) atomicAdd(bad_anc, bad);
        __syncthreads();
        if (hist_vecs > 0) {
            const char* hA = (const char*)histAB[0];
            const char* hB = (const char*)histAB[1];
            const int per = (hist_vecs + hb - 1) / hb;
            const int lo = part * per, hi = min(hist_vecs, lo + per);
            for (int k = 0; k < N; ++k) {
                const int a = sh_anc[k];
                if (a < 0) continue;
                const char* src = (sh_aux[a] ? hB : hA) + (long long)(row0 + a) * hist_row_bytes;      // live
                char* dst = (char*)(sh_aux[k] ? hA : hB) + (long long)(row0 + k) * hist_row_bytes;     // inactive
                for (int v = lo + tid; v < hi; v += kPagedThreads) *(vec16*)(dst + (long long)v * 16) = *(const vec16*)(src + (long long)v * 16);
            }
        }
        __syncthreads();
        if (tid == 0) {
            __threadfence();                                   // this workgroup's reads precede its ticket
            sh_last = atomicAdd(&arrive[b], 1) == hb - 1;
        }
        __syncthreads();
        if (sh_last) {
            for (int k = tid; k < N; k += kPagedThreads) {
                const int a = sh_anc[k];
                if (a >= 0) {
                    cumlogp[row0 + k] = sh_cum[a];
                    done[row0 + k] = sh_old[a];
                    parity[row0 + k] = sh_aux[k] ^ 1;
                }
            }
            if (tid == 0) arrive[b] = 0;
        }
        return;
    }
    const int bid = blockIdx.x - n_state;
    const int b = bid / chunks;
    if (!resampled[b]) {
        if (prepare && bid % chunks == 0) prepare_prompt(b, B, N, M, Q, pa, table, refcnt);
        return;
    }
    const int row0 = b * N, page0 = b * Q;
    for (int k = tid; k < N; k += kPagedThreads) sh_aux[k] = 0;
    __syncthreads();
    for (int k = tid; k < N; k += kPagedThreads) {
        int a = anc[row0 + k] - row0;
        if (a < 0 || a >= N) a = k;                    // outside the prompt: the row keeps its own pages
        sh_anc[k] = a;
        atomicAdd(&sh_aux[a], 1);
    }
    const int j0 = (bid % chunks) * cols;
    const int nc = min(cols, ncol - j0);               // columns of this workgroup
    const int n = N * nc;
    for (int e = tid; e < n; e += kPagedThreads) {
        const int k = e / nc, j = j0 + e % nc;
        sh_old[e] = table[(int64_t)(row0 + k) * M + j];
    }
    __syncthreads();
    for (int e = tid; e < n; e += kPagedThreads) {
        const int k = e / nc, c = e % nc;
        const int a = sh_anc[k];
        if (a != k) table[(int64_t)(row0 + k) * M + j0 + c] = sh_old[a * nc + c];
        const int gained = sh_aux[k] - 1;
        if (gained != 0) {
            const int p = sh_old[e];
            if (p >= page0 && p < page0 + Q) atomicAdd(&refcnt[p], gained);
        }
    }
    if (prepare) {
        // every thread's table entries and counts are out before the workgroup's ticket; the workgroup with the
        // prompt's last ticket sees what the others wrote
        __threadfence();
        __syncthreads();
        if (tid == 0) sh_last = atomicAdd(&arrive_table[b], 1) == chunks - 1;
        __syncthreads();
        if (sh_last) {
            if (tid == 0) arrive_table[b] = 0;
            __threadfence();
            prepare_prompt(b, B, N, M, Q, pa, table, refcnt);
        }
    }
}

// counters: [0], [1] number of (source, new page) pairs, alternating between successive calls; [2] rows that found no
// free page; [3] the pair counter the next call uses; [4] workgroups of the running call that have finished.  Every
// workgroup reads counters[3] first and takes a ticket last; the one with the last ticket clears the other pair
// counter and flips counters[3] on the device (no memset between calls).  The page column j and offset o are launch
// arguments derived from the host-side count of appended positions, so smc_paged_prepare_append refuses to be
// captured into a graph.
// One 256-thread workgroup prepares prompt b; n_prompts workgroups do so per call (the last of them flips the phase).
__device__ void prepare_prompt(int b, int n_prompts, int N, int M, int Q, const PrepareArgs& pa,
                               int32_t* __restrict__ table, int32_t* __restrict__ refcnt)
{
    const int j = pa.j, o = pa.o;
    int32_t* const counters = pa.counters;
    int32_t* const cow_src = pa.cow_src;
    int32_t* const cow_dst = pa.cow_dst;
    int32_t* const slot = pa.slot;
    __shared__ int32_t sh_page[SMC_MAX_PARTICLES];     // page of each row for this position (-1 at a page start)
    __shared__ int32_t sh_rank[SMC_MAX_PARTICLES];     // rank of a needy row among the prompt's needy rows, else -1
    __shared__ int32_t sh_free[SMC_MAX_PARTICLES];     // the prompt's lowest free pages, increasing
    __shared__ int32_t sh_wave[kPagedThreads / kWave];
    __shared__ int32_t sh_base;
    const int tid = threadIdx.x;
    const int row0 = b * N, page0 = b * Q;
    const int phase = counters[3];
    for (int k = tid; k < N; k += kPagedThreads) sh_page[k] = o == 0 ? -1 : table[(int64_t)(row0 + k) * M + j];
    __syncthreads();
    // needy rows: all of them at a page start; otherwise every sharer of a page but the lowest
    int n_needy = 0;
    for (int k0 = 0; k0 < N; k0 += kPagedThreads) {
        const int k = k0 + tid;
        int needy = 0;
        if (k < N) {
            if (o == 0) needy = 1;
            else {
                const int p = sh_page[k];
                for (int q = 0; q < k; ++q) if (sh_page[q] == p) { needy = 1; break; }
            }
        }
        int total;
        const int before = block_exclusive_scan(needy, sh_wave, total);
        if (k < N) sh_rank[k] = needy ? n_needy + before : -1;
        n_needy += total;
    }
    // the n_needy lowest free pages of the prompt.  Sweeps of 256*32 pages: every thread loads the counts of 32
    // consecutive pages (independent 16-byte loads), one prefix sum over the workgroup orders the free ones.
    int n_free = 0;
    for (int base = 0; base < Q && n_free < n_needy; base += kPagedThreads * kScanPerThread) {
        const int lo = base + tid * kScanPerThread;
        int cnt[kScanPerThread];
        if (lo + kScanPerThread <= Q && ((page0 + lo) & 3) == 0) {
            const int4* src = reinterpret_cast<const int4*>(refcnt + page0 + lo);
#pragma unroll
            for (int v = 0; v < kScanPerThread / 4; ++v) {
                const int4 x = src[v];
                cnt[4 * v] = x.x; cnt[4 * v + 1] = x.y; cnt[4 * v + 2] = x.z; cnt[4 * v + 3] = x.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < kScanPerThread; ++i) cnt[i] = lo + i < Q ? refcnt[page0 + lo + i] : 1;
        }
        unsigned free_bits = 0;
#pragma unroll
        for (int i = 0; i < kScanPerThread; ++i) free_bits |= (cnt[i] == 0 ? 1u : 0u) << i;
        int total;
        int z = n_free + block_exclusive_scan(__popc(free_bits), sh_wave, total);
        while (free_bits && z < n_needy) {
            const int i = __ffs(free_bits) - 1;
            free_bits &= free_bits - 1;
            sh_free[z++] = lo + i;
        }
        n_free += total;
    }
    const int n_served = min(n_needy, n_free);         // n_free >= n_needy unless the table was corrupted
    if (tid == 0) {
        sh_base = (o > 0 && n_served > 0) ? atomicAdd(&counters[phase], n_served) : 0;
        if (n_served < n_needy) atomicAdd(&counters[2], n_needy - n_served);
    }
    __syncthreads();
    for (int k = tid; k < N; k += kPagedThreads) {
        const int rank = sh_rank[k];
        int page = sh_page[k];
        if (rank >= 0 && rank < n_served) {
            const int fresh = page0 + sh_free[rank];
            if (o > 0) { cow_src[sh_base + rank] = page; cow_dst[sh_base + rank] = fresh; }
            table[(int64_t)(row0 + k) * M + j] = fresh;
            refcnt[fresh] = 1;
            page = fresh;
        } else if (rank < 0 && page >= page0 && page < page0 + Q) {
            refcnt[page] = 1;                          // the lowest sharer keeps the page for itself
        }
        slot[row0 + k] = page;
    }
    if (tid == 0) {
        __threadfence();                               // the read of counters[3] precedes the ticket
        if (atomicAdd(&counters[4], 1) == n_prompts - 1) {
            counters[phase ^ 1] = 0;
            counters[4] = 0;
            counters[3] = phase ^ 1;
        }
    }
}

__global__ __launch_bounds__(kPagedThreads) void paged_prepare_kernel(
    int N, int M, int Q, PrepareArgs pa, int32_t* __restrict__ table, int32_t* __restrict__ refcnt)
{
    prepare_prompt((int)blockIdx.x, (int)gridDim.x, N, M, Q, pa, table, refcnt);
}

// Copies the first copy_bytes bytes (a multiple of 16) of each of the n_heads head chunks of a page, for every tensor
// and every (source page, new page) pair.  One work item is a (pair, tensor): its n_heads * copy_bytes / 16 vectors
// are spread over the workgroup's threads as one flat range, so short prefixes of a page still keep every lane busy.
__global__ __launch_bounds__(kPagedThreads) void paged_copy_kernel(
    void* const* __restrict__ pools, int n_tensors, int n_heads, long long page_stride, long long head_stride,
    int vecs_per_head, int n_pages, const int32_t* __restrict__ counters,
    const int32_t* __restrict__ cow_src, const int32_t* __restrict__ cow_dst)
{
    const int n_pairs = counters[counters[3] ^ 1];     // the prepare kernel flipped the phase after using it
    const int64_t total = (int64_t)n_tensors * n_pairs;
    const int n_vec = n_heads * vecs_per_head;
    for (int64_t w = blockIdx.x; w < total; w += gridDim.x) {
        const int pair = (int)(w / n_tensors);
        const int tensor = (int)(w - (int64_t)pair * n_tensors);
        const int from = cow_src[pair], to = cow_dst[pair];
        if (from < 0 || from >= n_pages || to < 0 || to >= n_pages) continue;      // only after a corrupted table
        const char* s = (const char*)pools[tensor] + (int64_t)from * page_stride;
        char* d = (char*)pools[tensor] + (int64_t)to * page_stride;
        for (int v = threadIdx.x; v < n_vec; v += kPagedThreads) {
            const int head = v / vecs_per_head;
            const int64_t off = (int64_t)head * head_stride + (int64_t)(v - head * vecs_per_head) * 16;
            __builtin_nontemporal_store(*(const vec16*)(s + off), (vec16*)(d + off));
        }
    }
}

}  // namespace psmc

using namespace psmc;

namespace {
constexpr size_t kAlign = 256;
inline size_t up(size_t x) { return (x + kAlign - 1) & ~(kAlign - 1); }

struct PagedDims { int P, M, Q; size_t n_table, n_pages; };

void launch_paged_copy(smc_ctx* ctx, int o);       // below, with the reorder launch

bool stream_is_capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
    return st != hipStreamCaptureStatusNone;
}

bool paged_dims(const smc_config* c, int page_len, PagedDims* d)
{
    if (!c || c->kv_tensors < 1 || c->kv_S < 1 || c->N < 1 || c->B < 1 || page_len < 1 || page_len > c->kv_S) return false;
    if (((int64_t)c->kv_D * c->kv_elem_bytes) % 16 != 0) return false;
    d->P = page_len;
    d->M = (c->kv_S + page_len - 1) / page_len;
    const int64_t Q = (int64_t)c->N * d->M;
    const int64_t pages = Q * c->B;
    if (pages > ((int64_t)1 << 30)) return false;
    d->Q = (int)Q;
    d->n_pages = (size_t)pages;
    d->n_table = (size_t)c->B * c->N * d->M;
    return true;
}

size_t paged_layout(const smc_config* c, const PagedDims& d, char* base, PagedKV* p)
{
    const size_t R = (size_t)c->B * c->N;
    size_t off = 0;
    auto take = [&](size_t bytes) { char* q = base ? base + off : nullptr; off += up(bytes); return q; };
    char* q;
    q = take(d.n_table * 4); if (p) p->table = (int32_t*)q;
    q = take(d.n_pages * 4); if (p) p->refcnt = (int32_t*)q;
    q = take(R * 4); if (p) p->cow_src = (int32_t*)q;
    q = take(R * 4); if (p) p->cow_dst = (int32_t*)q;
    q = take(8 * 4); if (p) p->counters = (int32_t*)q;
    q = take((size_t)c->B * 4); if (p) p->arrive = (int32_t*)q;
    q = take((size_t)c->B * 4); if (p) p->arrive_table = (int32_t*)q;
    q = take((size_t)c->kv_tensors * sizeof(void*)); if (p) p->pools = (void**)q;
    return off;
}
}  // namespace

extern "C" {

size_t smc_paged_workspace_bytes(const smc_config* cfg, int32_t page_len)
{
    PagedDims d;
    if (!paged_dims(cfg, page_len, &d)) return 0;
    return paged_layout(cfg, d, nullptr, nullptr);
}

size_t smc_paged_pool_bytes(const smc_config* cfg, int32_t page_len)
{
    PagedDims d;
    if (!paged_dims(cfg, page_len, &d)) return 0;
    return d.n_pages * (size_t)cfg->kv_H * (size_t)d.P * (size_t)cfg->kv_D * (size_t)cfg->kv_elem_bytes;
}

smc_status smc_paged_bind(smc_ctx* ctx, void* const* h_pools, int32_t page_len, void* d_workspace, size_t workspace_bytes,
                          int32_t len0)
{
    if (!ctx || !h_pools || !d_workspace) return SMC_E_NULL;
    PagedDims d;
    if (!paged_dims(&ctx->cfg, page_len, &d)) return SMC_E_SHAPE;
    if (len0 < 0 || len0 > ctx->cfg.kv_S) return SMC_E_RANGE;
    if (((uintptr_t)d_workspace & (kAlign - 1)) != 0) return SMC_E_ALIGN;
    if (workspace_bytes < paged_layout(&ctx->cfg, d, nullptr, nullptr)) return SMC_E_SHAPE;
    for (int i = 0; i < ctx->cfg.kv_tensors; ++i) {
        if (!h_pools[i]) return SMC_E_NULL;
        if (((uintptr_t)h_pools[i] & 15u) != 0) return SMC_E_ALIGN;
    }
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    PagedKV& p = ctx->paged;
    p.bound = 0;                                       // a failed (re)bind leaves the context unbound
    paged_layout(&ctx->cfg, d, (char*)d_workspace, &p);
    p.P = d.P; p.M = d.M; p.Q = d.Q; p.len = len0;
    if (hipMemcpy(p.pools, h_pools, (size_t)ctx->cfg.kv_tensors * sizeof(void*), hipMemcpyHostToDevice) != hipSuccess)
        return SMC_E_HIP;
    try { ctx->h_pools.assign(h_pools, h_pools + ctx->cfg.kv_tensors); } catch (...) { return SMC_E_STATE; }
    const size_t n = d.n_table > d.n_pages ? d.n_table : d.n_pages;
    hipLaunchKernelGGL(paged_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, ctx->R, ctx->cfg.N,
                       d.M, d.Q, d.P, len0, p.table, p.refcnt, p.counters, p.arrive, p.arrive_table);
    if (hipGetLastError() != hipSuccess) return SMC_E_HIP;
    p.bound = 1;
    return SMC_OK;
}

smc_status smc_paged_prepare_append(smc_ctx* ctx, int32_t pos, int32_t* d_slot_out)
{
    if (!ctx || !d_slot_out) return SMC_E_NULL;
    PagedKV& p = ctx->paged;
    if (!p.bound) return SMC_E_STATE;
    if (pos < 0 || pos >= ctx->cfg.kv_S) return SMC_E_RANGE;
    if (pos != p.len) return SMC_E_STATE;              // positions are appended one by one, the same for every row
    // The appended length is host-side state and the page column / offset of `pos` are launch arguments: a captured
    // call would replay the same position for ever.  Refuse rather than corrupt the table silently.
    if (stream_is_capturing(ctx->stream)) return SMC_E_STATE;
    const auto& cfg = ctx->cfg;
    const int j = pos / p.P, o = pos % p.P;
    const PrepareArgs pa{j, o, p.counters, p.cow_src, p.cow_dst, d_slot_out};
    hipLaunchKernelGGL(paged_prepare_kernel, dim3(cfg.B), dim3(kPagedThreads), 0, ctx->stream, cfg.N, p.M, p.Q, pa,
                       p.table, p.refcnt);
    if (o > 0) launch_paged_copy(ctx, o);
    if (hipGetLastError() != hipSuccess) return SMC_E_HIP;
    p.len = pos + 1;
    return SMC_OK;
}

}  // extern "C"

namespace {

// The reorder launch; with `pa`, the same launch also prepares every prompt for the position pa describes.
// *fused tells whether it did (a cache without a page in use has no table workgroup to do it).
smc_status launch_paged_reorder(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t t,
                                const PrepareArgs* pa, bool* fused)
{
    PagedKV& p = ctx->paged;
    const auto& cfg = ctx->cfg;
    const int N = cfg.N;
    // token history: whole 16-byte vectors of the first t columns, as in the dense reorder
    int hist_vecs = 0;
    if (ctx->hist_bound && (t > 0 || ctx->device_step)) {
        int64_t bytes = (((int64_t)t * 4) + 15) & ~15ll;
        // with the step kept on the device the host does not know how long the prefixes are: whole rows move
        if (bytes > (int64_t)cfg.T_max * 4 || ctx->device_step) bytes = (int64_t)cfg.T_max * 4;
        hist_vecs = (int)(bytes / 16);
    }
    int hb = (int)(((int64_t)N * hist_vecs * 16 + 65535) / 65536);          // ~64 KiB of history per state workgroup
    if (hb > 64) hb = 64;
    if (hb > hist_vecs) hb = hist_vecs;
    if (hb < 1) hb = 1;
    // Columns in use.  The count is a launch argument, so under stream capture (where later replays may follow
    // appends that this call cannot see) every column is permuted: unused columns hold -1 in every row, and
    // permuting them changes nothing.
    const int ncol = stream_is_capturing(ctx->stream) ? p.M : (p.len + p.P - 1) / p.P;
    int cols = 1, chunks = 0;
    if (ncol > 0) {
        cols = kEntriesPerBlock / N < ncol ? kEntriesPerBlock / N : ncol;   // >= 1: N <= SMC_MAX_PARTICLES
        chunks = (ncol + cols - 1) / cols;
    }
    const int64_t blocks = (int64_t)cfg.B * hb + (int64_t)cfg.B * chunks;
    if (blocks > 0x7FFFFFFFll) return SMC_E_SHAPE;
    const bool prepare = pa && chunks > 0;
    if (fused) *fused = prepare;
    hipLaunchKernelGGL(paged_reorder_kernel, dim3((unsigned)blocks), dim3(kPagedThreads), 0, ctx->stream, d_anc, d_resampled,
                       cfg.B, N, hb, hist_vecs, (long long)cfg.T_max * 4, (int32_t* const*)ctx->ws.histAB, ctx->ws.cumlogp,
                       ctx->ws.done, ctx->ws.parity, &ctx->ws.plan->bad_anc, p.arrive, p.M, p.Q, ncol, cols, chunks, p.table,
                       p.refcnt, prepare ? 1 : 0, prepare ? *pa : PrepareArgs{}, p.arrive_table);
    return hipGetLastError() == hipSuccess ? SMC_OK : SMC_E_HIP;
}

// The copy of the filled part of every shared page that the preparation of position `pos` (offset o > 0) listed.
void launch_paged_copy(smc_ctx* ctx, int o)
{
    const auto& cfg = ctx->cfg;
    PagedKV& p = ctx->paged;
    const long long pos_bytes = (long long)cfg.kv_D * cfg.kv_elem_bytes;
    const long long head_stride = pos_bytes * p.P;
    ScopedKernelTimer timer(ctx, 2);
    hipLaunchKernelGGL(paged_copy_kernel, dim3(ctx->n_cus * 8), dim3(kPagedThreads), 0, ctx->stream,
                       (void* const*)p.pools, cfg.kv_tensors, cfg.kv_H, head_stride * cfg.kv_H, head_stride,
                       (int)(pos_bytes * o / 16), cfg.B * p.Q, p.counters, p.cow_src, p.cow_dst);
}

}  // namespace

extern "C" {

smc_status smc_paged_reindex(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t t)
{
    if (!ctx || !d_anc || !d_resampled) return SMC_E_NULL;
    if (!ctx->paged.bound) return SMC_E_STATE;
    if (t < 0 || t > ctx->cfg.T_max) return SMC_E_RANGE;
    return launch_paged_reorder(ctx, d_anc, d_resampled, t, nullptr, nullptr);
}

smc_status smc_paged_reindex_prepare(smc_ctx* ctx, const int32_t* d_anc, const int32_t* d_resampled, int32_t t,
                                     int32_t next_pos, int32_t* d_slot_out)
{
    if (!ctx || !d_anc || !d_resampled || !d_slot_out) return SMC_E_NULL;
    PagedKV& p = ctx->paged;
    if (!p.bound) return SMC_E_STATE;
    if (t < 0 || t > ctx->cfg.T_max) return SMC_E_RANGE;
    if (next_pos < 0 || next_pos >= ctx->cfg.kv_S) return SMC_E_RANGE;
    if (next_pos != p.len) return SMC_E_STATE;
    if (stream_is_capturing(ctx->stream)) return SMC_E_STATE;     // as smc_paged_prepare_append: the position is host-side state
    const int j = next_pos / p.P, o = next_pos % p.P;
    const PrepareArgs pa{j, o, p.counters, p.cow_src, p.cow_dst, d_slot_out};
    bool fused = false;
    const smc_status st = launch_paged_reorder(ctx, d_anc, d_resampled, t, &pa, &fused);
    if (st != SMC_OK) return st;
    if (!fused) return smc_paged_prepare_append(ctx, next_pos, d_slot_out);
    if (o > 0) launch_paged_copy(ctx, o);
    if (hipGetLastError() != hipSuccess) return SMC_E_HIP;
    p.len = next_pos + 1;
    return SMC_OK;
}

smc_status smc_paged_view(smc_ctx* ctx, const int32_t** d_table, const int32_t** d_refcnt, int32_t* pages_per_row,
                          int32_t* pages_per_prompt, int32_t* len)
{
    if (!ctx) return SMC_E_NULL;
    const PagedKV& p = ctx->paged;
    if (!p.bound) return SMC_E_STATE;
    if (d_table) *d_table = p.table;
    if (d_refcnt) *d_refcnt = p.refcnt;
    if (pages_per_row) *pages_per_row = p.M;
    if (pages_per_prompt) *pages_per_prompt = p.Q;
    if (len) *len = p.len;
    return SMC_OK;
}

smc_status smc_paged_check(smc_ctx* ctx, int32_t* h_alloc_failures)
{
    if (!ctx || !h_alloc_failures) return SMC_E_NULL;
    if (!ctx->paged.bound) return SMC_E_STATE;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SMC_E_HIP;
    return hipMemcpy(h_alloc_failures, ctx->paged.counters + 2, 4, hipMemcpyDeviceToHost) == hipSuccess ? SMC_OK : SMC_E_HIP;
}

}  // extern "C"
