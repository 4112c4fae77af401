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
//   plan_kernel    : one wave per prompt.  Builds the groups (ancestor row, which of its buffers is live and whether
//                    it has terminated, bit set of moved descendants), gathers cumulative log p and termination flags the same way, and flips
//                    the parity of the moved rows -- so after it, a moved row's parity names the buffer to WRITE.
//   gather_kernel  : persistent grid-stride loop over (group, tensor, head chunk, slab of 8..64 KiB) for the KV
//                    tensors, followed in the same launch by the token-history rows.
#include "gather_plan_device.hpp"

namespace psmc {

namespace {
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));    // one 16-byte global load / store
}  // namespace

// One wave per prompt.
__global__ __launch_bounds__(kWave) void plan_kernel(const int32_t* __restrict__ anc, const int32_t* __restrict__ resampled,
                                                     PlanArgs pl)
{
    const int phase = pl.plan->phase;
    if (resampled[blockIdx.x])
        plan_prompt(anc, pl.N, pl.mask_words, phase, pl.plan, pl.grp_src, pl.grp_base, pl.grp_srcpar, pl.grp_mask, pl.cumlogp,
                    pl.done, pl.parity, pl.skip_terminated);
    plan_finish(pl.plan, phase, (int)gridDim.x);
}

struct GatherGeom {               // one family of tensors with identical geometry
    void* const* bufA; void* const* bufB;
    int n_tensors, n_chunks, slabs_per_chunk;
    long long row_stride, chunk_stride, copy_bytes;
};

// Row r of a tensor starts at r*row_stride bytes; of each of its n_chunks chunks (chunk_stride bytes apart) the first
// copy_bytes bytes (a multiple of 16) are copied.  `kv` and `hist` are the two families handled by one launch.
// THREADS: workgroup size; VPT: 16-byte vectors in flight per thread (a workgroup iteration moves a slab of
// THREADS*VPT*16 bytes); NT_LD / NT_ST: non-temporal loads / stores.
template <int THREADS, int VPT, bool NT_LD, bool NT_ST>
__global__ __launch_bounds__(THREADS) void gather_kernel(
    GatherGeom kv, GatherGeom hist, const int32_t* __restrict__ parity, int mask_words,
    const GatherPlan* __restrict__ plan, const int32_t* __restrict__ grp_src, const int32_t* __restrict__ grp_base,
    const int32_t* __restrict__ grp_srcpar, const unsigned long long* __restrict__ grp_mask)
{
    constexpr int kGatherThreads = THREADS;
    constexpr int kVecPerThread = VPT;
    constexpr int kSlabBytes = kGatherThreads * VPT * 16;
    const int n_groups = plan->n_groups[plan->phase ^ 1];          // the plan flipped the phase after using it
    const int64_t per_group_kv = (int64_t)kv.n_tensors * kv.n_chunks * kv.slabs_per_chunk;
    const int64_t per_group_h = (int64_t)hist.n_tensors * hist.n_chunks * hist.slabs_per_chunk;
    const int64_t total_kv = per_group_kv * n_groups;
    const int64_t total = total_kv + per_group_h * n_groups;
    const int tid = threadIdx.x;
    for (int64_t w = blockIdx.x; w < total; w += gridDim.x) {
        const bool is_kv = w < total_kv;
        const GatherGeom& ge = is_kv ? kv : hist;
        const int64_t per_group = is_kv ? per_group_kv : per_group_h;
        int64_t rem = is_kv ? w : w - total_kv;
        const int g = (int)(rem / per_group);
        rem -= (int64_t)g * per_group;
        const int tensor = (int)(rem / ((int64_t)ge.n_chunks * ge.slabs_per_chunk));
        rem -= (int64_t)tensor * ge.n_chunks * ge.slabs_per_chunk;
        const int chunk = (int)(rem / ge.slabs_per_chunk);
        const int slab = (int)(rem - (int64_t)chunk * ge.slabs_per_chunk);

        const int src_state = grp_srcpar[g];
        if (is_kv && (src_state & 2)) continue;                     // terminated ancestor: only its history moves
        const int src_row = grp_src[g];
        const int row0 = grp_base[g];
        char* const baseA = (char*)ge.bufA[tensor];
        char* const baseB = (char*)ge.bufB[tensor];
        const char* src = (src_state & 1) ? baseB : baseA;          // the ancestor's live buffer
        const int64_t off0 = (int64_t)chunk * ge.chunk_stride + (int64_t)slab * kSlabBytes;
        const int64_t left = ge.copy_bytes - (int64_t)slab * kSlabBytes;    // bytes of this chunk from the slab start

        vec16 v[kVecPerThread];
        const char* s = src + (int64_t)src_row * ge.row_stride + off0;
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
                // the plan has already flipped the parity of moved rows: it names the buffer to write
                char* d = (parity[drow] ? baseB : baseA) + (int64_t)drow * ge.row_stride + off0;
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

template <int THREADS, int VPT, bool NT_LD, bool NT_ST>
static void launch_gather(smc_ctx* c, GatherGeom kv, GatherGeom hist)
{
    constexpr int64_t slab = (int64_t)THREADS * VPT * 16;
    kv.slabs_per_chunk = (int)((kv.copy_bytes + slab - 1) / slab);
    hist.slabs_per_chunk = (int)((hist.copy_bytes + slab - 1) / slab);
    auto& w = c->ws;
    // the same number of resident waves whatever the workgroup size
    const int grid = c->gather_grid * 256 / THREADS > 0 ? c->gather_grid * 256 / THREADS : 1;
    hipLaunchKernelGGL((gather_kernel<THREADS, VPT, NT_LD, NT_ST>), dim3(grid), dim3(THREADS), 0, c->stream, kv, hist,
                       w.parity, c->mask_words, w.plan, w.grp_src, w.grp_base, w.grp_srcpar, w.grp_mask);
}

static void launch_gather_variant(smc_ctx* c, int variant, const GatherGeom& kv, const GatherGeom& hist)
{
#define PSMC_G(T, V, L, S) launch_gather<T, V, L, S>(c, kv, hist)
    switch (variant) {
        case 0: PSMC_G(256, 8, true, true); break;
        case 1: PSMC_G(256, 8, false, true); break;
        case 2: PSMC_G(256, 8, false, false); break;
        case 3: PSMC_G(256, 4, true, true); break;
        case 4: PSMC_G(256, 4, false, true); break;
        case 5: PSMC_G(256, 4, false, false); break;
        case 6: PSMC_G(256, 16, true, true); break;
        case 7: PSMC_G(256, 16, false, true); break;
        case 8: PSMC_G(256, 16, false, false); break;
        case 9: PSMC_G(256, 2, true, true); break;
        case 10: PSMC_G(256, 2, false, false); break;
        case 11: PSMC_G(1024, 4, false, true); break;
        case 12: PSMC_G(1024, 4, false, false); break;
        case 13: PSMC_G(1024, 4, true, true); break;
        case 14: PSMC_G(1024, 2, false, true); break;
        case 15: PSMC_G(1024, 8, false, true); break;
        case 16: PSMC_G(512, 4, false, true); break;
        case 17: PSMC_G(512, 8, false, true); break;
        default: PSMC_G(256, 4, false, true); break;
    }
#undef PSMC_G
}

PlanArgs plan_args(const smc_ctx* c)
{
    const auto& w = c->ws;
    return PlanArgs{c->cfg.N, c->mask_words, (c->kv_skip_terminated && c->cfg.eos_id >= 0) ? 1 : 0, w.plan, w.grp_src,
                    w.grp_base, w.grp_srcpar, w.grp_mask, w.cumlogp, w.done, w.parity};
}

// planned: the plan of this reorder has already been made (by the resampling kernel of the same call).
hipError_t launch_reindex(smc_ctx* c, const int32_t* anc, const int32_t* resampled, int valid_len, int t, bool planned)
{
    const auto& cfg = c->cfg;
    auto& w = c->ws;
    const bool have_kv = c->kv_bound && cfg.kv_tensors > 0 && valid_len > 0;
    const bool have_hist = c->hist_bound && (t > 0 || c->device_step);
    if (!planned)
        hipLaunchKernelGGL(plan_kernel, dim3(cfg.B), dim3(kWave), 0, c->stream, anc, resampled, plan_args(c));
    if (have_kv || have_hist) {
        GatherGeom kv{}, hist{};
        if (have_kv) {
            const int64_t pos_bytes = (int64_t)cfg.kv_D * cfg.kv_elem_bytes;
            const int64_t head_stride = (int64_t)cfg.kv_S * pos_bytes;
            kv.bufA = (void* const*)w.kvA; kv.bufB = (void* const*)w.kvB;
            kv.n_tensors = cfg.kv_tensors;
            kv.row_stride = head_stride * cfg.kv_H;
            kv.chunk_stride = head_stride;
            kv.n_chunks = cfg.kv_H;
            kv.copy_bytes = (int64_t)valid_len * pos_bytes;
            if (valid_len == cfg.kv_S) { kv.n_chunks = 1; kv.copy_bytes = kv.row_stride; }   // whole row is contiguous
        }
        if (have_hist) {
            hist.bufA = (void* const*)w.histAB; hist.bufB = (void* const*)(w.histAB + 1);
            hist.n_tensors = 1; hist.n_chunks = 1;
            hist.row_stride = (int64_t)cfg.T_max * 4;
            hist.chunk_stride = hist.row_stride;
            hist.copy_bytes = (((int64_t)t * 4) + 15) & ~15ll;                              // whole 16-byte vectors
            // with the step kept on the device the host does not know how long the prefixes are: whole rows move
            if (hist.copy_bytes > hist.row_stride || c->device_step) hist.copy_bytes = hist.row_stride;
        }
        ScopedKernelTimer timer(c, 1);
        launch_gather_variant(c, c->gather_variant, kv, hist);
    }
    return hipGetLastError();
}

}  // namespace psmc
