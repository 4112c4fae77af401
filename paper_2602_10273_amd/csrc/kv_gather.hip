// Cache-safe reindex after resampling (Alg. 1 "reorder KV cache by A"; App. C: reindex along the
// batch/particle dimension) for gfx950: an out-of-place, double-buffered row gather.
//
// Every row (particle slot) k has two buffers and a parity bit: its live data is in buffer A while parity[k] = 0,
// in buffer B while parity[k] = 1.  For a resampled prompt, a row whose ancestor is another row (anc[k] != k)
// receives the ancestor's LIVE row in its own INACTIVE buffer, for every KV tensor and the token history, and then
// its parity flips.  Readers only touch live buffers and writers only inactive ones, so any ancestor vector is safe,
// and a row that is its own ancestor moves no bytes at all.  Pure HBM traffic, 16-byte vector loads and stores.
// Moved rows that share an ancestor form a group: the ancestor's bytes are read ONCE into registers and stored to
// every member, so a reindex moves (distinct ancestors of moved rows + moved rows) rows, the least the method allows.
//
//   plan_kernel    : one wave per prompt, builds the groups (ancestor row, bit set of moved descendants).
//   gather_kernel  : persistent grid-stride loop over (group, tensor, head chunk, slab of 8..64 KiB).
//   commit_kernel  : cumulative log p and termination flags gathered the same way, parities flipped, plan cleared.
#include "device_rng.hpp"
#include "smc_internal.hpp"

namespace psmc {

namespace {
constexpr int kGatherThreads = 256;
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));    // one 16-byte global load / store
}  // namespace

__global__ __launch_bounds__(kWave) void plan_kernel(const int32_t* __restrict__ anc, const int32_t* __restrict__ resampled,
                                                     int N, int mask_words, GatherPlan* __restrict__ plan,
                                                     int32_t* __restrict__ grp_src, int32_t* __restrict__ grp_base,
                                                     unsigned long long* __restrict__ grp_mask)
{
    __shared__ int32_t sh_anc[SMC_MAX_PARTICLES];
    __shared__ int32_t sh_base;
    const int b = blockIdx.x, lane = threadIdx.x;
    if (!resampled[b]) return;
    const int row0 = b * N;
    int bad = 0;
    for (int k = lane; k < N; k += kWave) {
        int a = anc[row0 + k] - row0;
        if (a < 0 || a >= N) { a = -1; ++bad; }                    // outside the prompt: row is left untouched
        if (a == k) a = -1;                                        // its own ancestor: nothing to move
        sh_anc[k] = a;
    }
    __syncthreads();
    // leaders: first moved row (in particle order) of each distinct ancestor
    int n_lead = 0;
    for (int k0 = 0; k0 < N; k0 += kWave) {
        const int k = k0 + lane;
        bool lead = false;
        if (k < N && sh_anc[k] >= 0) {
            lead = true;
            const int a = sh_anc[k];
            for (int j = 0; j < k; ++j) if (sh_anc[j] == a) { lead = false; break; }
        }
        n_lead += __popcll(__ballot(lead));
    }
    if (lane == 0) {
        sh_base = n_lead ? atomicAdd(&plan->n_groups, n_lead) : 0;
    }
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o);
    if (lane == 0 && bad) atomicAdd(&plan->bad_anc, bad);
    __syncthreads();
    int done = 0;
    for (int k0 = 0; k0 < N; k0 += kWave) {
        const int k = k0 + lane;
        bool lead = false;
        int a = -1;
        if (k < N && sh_anc[k] >= 0) {
            lead = true;
            a = sh_anc[k];
            for (int j = 0; j < k; ++j) if (sh_anc[j] == a) { lead = false; break; }
        }
        const unsigned long long mk = __ballot(lead);
        if (lead) {
            const int g = sh_base + done + mask_rank(mk);
            grp_src[g] = row0 + a;
            grp_base[g] = row0;
            for (int w = 0; w < mask_words; ++w) {
                unsigned long long bits = 0;
                const int hi = min(N - w * 64, 64);
                for (int j = 0; j < hi; ++j) if (sh_anc[w * 64 + j] == a) bits |= 1ull << j;
                grp_mask[(int64_t)g * mask_words + w] = bits;
            }
        }
        done += __popcll(mk);
    }
}

// One launch copies `n_tensors` tensors of identical geometry.  Row r of a tensor starts at r*row_stride bytes;
// of each of its `n_chunks` chunks (chunk_stride bytes apart) the first `copy_bytes` bytes are copied.
// copy_bytes is a multiple of 16; the last vector of a chunk may be cut at `chunk_limit` bytes (history rows).
// VPT: 16-byte vectors in flight per thread (a workgroup iteration moves a slab of 256*VPT*16 bytes);
// NT_LD / NT_ST: non-temporal loads / stores.
template <int VPT, bool NT_LD, bool NT_ST>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(
    void* const* __restrict__ bufA, void* const* __restrict__ bufB, const int32_t* __restrict__ parity, int N,
    int n_tensors, int n_chunks, int64_t row_stride, int64_t chunk_stride, int64_t copy_bytes, int slabs_per_chunk,
    int mask_words, const GatherPlan* __restrict__ plan, const int32_t* __restrict__ grp_src,
    const int32_t* __restrict__ grp_base, const unsigned long long* __restrict__ grp_mask)
{
    constexpr int kVecPerThread = VPT;
    constexpr int kSlabBytes = kGatherThreads * VPT * 16;
    const int n_groups = plan->n_groups;
    const int64_t per_group = (int64_t)n_tensors * n_chunks * slabs_per_chunk;
    const int64_t total = per_group * n_groups;
    const int tid = threadIdx.x;
    for (int64_t w = blockIdx.x; w < total; w += gridDim.x) {
        const int g = (int)(w / per_group);
        int64_t rem = w - (int64_t)g * per_group;
        const int tensor = (int)(rem / ((int64_t)n_chunks * slabs_per_chunk));
        rem -= (int64_t)tensor * n_chunks * slabs_per_chunk;
        const int chunk = (int)(rem / slabs_per_chunk);
        const int slab = (int)(rem - (int64_t)chunk * slabs_per_chunk);

        const int src_row = grp_src[g];
        const int row0 = grp_base[g];
        char* const baseA = (char*)bufA[tensor];
        char* const baseB = (char*)bufB[tensor];
        const char* src = parity[src_row] ? baseB : baseA;          // the ancestor's live buffer
        const int64_t off0 = (int64_t)chunk * chunk_stride + (int64_t)slab * kSlabBytes;
        const int64_t left = copy_bytes - (int64_t)slab * kSlabBytes;       // bytes of this chunk from the slab start

        vec16 v[kVecPerThread];
        const char* s = src + (int64_t)src_row * row_stride + off0;
#pragma unroll
        for (int u = 0; u < kVecPerThread; ++u) {
            const int64_t o = ((int64_t)u * kGatherThreads + tid) * 16;
            if (o < left) {
                if constexpr (NT_LD) v[u] = __builtin_nontemporal_load((const vec16*)(s + o));
                else v[u] = *(const vec16*)(s + o);
            }
        }
        for (int mw = 0; mw < mask_words; ++mw) {
            unsigned long long bits = grp_mask[(int64_t)g * mask_words + mw];
            while (bits) {
                const int j = __ffsll((long long)bits) - 1;
                bits &= bits - 1;
                const int drow = row0 + mw * 64 + j;
                char* d = (parity[drow] ? baseA : baseB) + (int64_t)drow * row_stride + off0;   // its inactive buffer
#pragma unroll
                for (int u = 0; u < kVecPerThread; ++u) {
                    const int64_t o = ((int64_t)u * kGatherThreads + tid) * 16;
                    if (o < left) {
                        if constexpr (NT_ST) __builtin_nontemporal_store(v[u], (vec16*)(d + o));
                        else *(vec16*)(d + o) = v[u];
                    }
                }
            }
        }
    }
}

// After the gathers: cumulative log p follows its particle, parity flips, the plan is cleared.
__global__ __launch_bounds__(kWave) void commit_kernel(const int32_t* __restrict__ anc, const int32_t* __restrict__ resampled,
                                                       int N, double* __restrict__ cumlogp, int32_t* __restrict__ done,
                                                       int32_t* __restrict__ parity, GatherPlan* __restrict__ plan)
{
    __shared__ double sh[SMC_MAX_PARTICLES];
    __shared__ int32_t sh_done[SMC_MAX_PARTICLES];
    const int b = blockIdx.x, lane = threadIdx.x;
    if (b == 0 && lane == 0) plan->n_groups = 0;
    if (!resampled[b]) return;
    const int row0 = b * N;
    for (int k = lane; k < N; k += kWave) { sh[k] = cumlogp[row0 + k]; sh_done[k] = done[row0 + k]; }
    __syncthreads();
    for (int k = lane; k < N; k += kWave) {
        const int a = anc[row0 + k] - row0;
        if (a >= 0 && a < N && a != k) {
            cumlogp[row0 + k] = sh[a]; done[row0 + k] = sh_done[a];
            parity[row0 + k] ^= 1;                                 // the row now lives in the buffer just written
        }
    }
}

template <int VPT, bool NT_LD, bool NT_ST>
static void launch_gather(smc_ctx* c, void* const* bufA, void* const* bufB, int n_tensors, int n_chunks, int64_t row_stride,
                          int64_t chunk_stride, int64_t copy_bytes)
{
    constexpr int64_t slab = (int64_t)kGatherThreads * VPT * 16;
    const int slabs = (int)((copy_bytes + slab - 1) / slab);
    auto& w = c->ws;
    hipLaunchKernelGGL((gather_kernel<VPT, NT_LD, NT_ST>), dim3(c->gather_grid), dim3(kGatherThreads), 0, c->stream, bufA, bufB,
                       w.parity, c->cfg.N, n_tensors, n_chunks, row_stride, chunk_stride, copy_bytes, slabs, c->mask_words,
                       w.plan, w.grp_src, w.grp_base, w.grp_mask);
}

static void launch_gather_variant(smc_ctx* c, int variant, void* const* bufA, void* const* bufB, int n_tensors, int n_chunks,
                                  int64_t row_stride, int64_t chunk_stride, int64_t copy_bytes)
{
#define PSMC_G(V, L, S) launch_gather<V, L, S>(c, bufA, bufB, n_tensors, n_chunks, row_stride, chunk_stride, copy_bytes)
    switch (variant) {
        case 0: PSMC_G(8, true, true); break;
        case 1: PSMC_G(8, false, true); break;
        case 2: PSMC_G(8, false, false); break;
        case 3: PSMC_G(4, true, true); break;
        case 4: PSMC_G(4, false, true); break;
        case 5: PSMC_G(4, false, false); break;
        case 6: PSMC_G(16, true, true); break;
        case 7: PSMC_G(16, false, true); break;
        case 8: PSMC_G(16, false, false); break;
        case 9: PSMC_G(2, true, true); break;
        case 10: PSMC_G(2, false, false); break;
        default: PSMC_G(8, true, true); break;
    }
#undef PSMC_G
}

hipError_t launch_reindex(smc_ctx* c, const int32_t* anc, const int32_t* resampled, int valid_len, int t)
{
    const auto& cfg = c->cfg;
    auto& w = c->ws;
    const bool have_kv = c->kv_bound && cfg.kv_tensors > 0 && valid_len > 0;
    const bool have_hist = c->hist_bound && t > 0;
    if (have_kv || have_hist) {
        hipLaunchKernelGGL(plan_kernel, dim3(cfg.B), dim3(kWave), 0, c->stream, anc, resampled, cfg.N, c->mask_words,
                           w.plan, w.grp_src, w.grp_base, w.grp_mask);
    }
    if (have_kv) {
        const int64_t pos_bytes = (int64_t)cfg.kv_D * cfg.kv_elem_bytes;
        const int64_t head_stride = (int64_t)cfg.kv_S * pos_bytes;
        const int64_t row_stride = head_stride * cfg.kv_H;
        int n_chunks = cfg.kv_H;
        int64_t copy_bytes = (int64_t)valid_len * pos_bytes;
        if (valid_len == cfg.kv_S) { n_chunks = 1; copy_bytes = row_stride; }       // whole row is contiguous
        ScopedKernelTimer timer(c, 1);
        launch_gather_variant(c, c->gather_variant, (void* const*)w.kvA, (void* const*)w.kvB, cfg.kv_tensors, n_chunks,
                              row_stride, head_stride, copy_bytes);
    }
    if (have_hist) {
        const int64_t row_stride = (int64_t)cfg.T_max * 4;
        int64_t copy_bytes = (((int64_t)t * 4) + 15) & ~15ll;                       // whole 16-byte vectors
        if (copy_bytes > row_stride) copy_bytes = row_stride;
        launch_gather<4, false, false>(c, (void* const*)w.histAB, (void* const*)(w.histAB + 1), 1, 1, row_stride, row_stride,
                                       copy_bytes);
    }
    hipLaunchKernelGGL(commit_kernel, dim3(cfg.B), dim3(kWave), 0, c->stream, anc, resampled, cfg.N, w.cumlogp, w.done, w.parity,
                       w.plan);
    return hipGetLastError();
}

}  // namespace psmc
