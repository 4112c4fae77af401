// Writes the new position of every row into the cache the reorder maintains: the store a decoder makes before it
// attends.  A row's data lives in buffer A or B (dense, by the row's parity) or in the page the table names (paged),
// so the caller would otherwise have to read that state back; this is the one store that follows it on the device.
// Not part of the paper's method (App. C only moves what is already cached).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "smc_internal.hpp"

namespace psmc {

namespace {
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));

struct AppendDst {
    char* a[2];                 // dense: the tensors in buffer A; paged: their pools
    char* b[2];                 // dense: the same tensors in buffer B
    const char* src[2];         // new entries, [R, H, D] with a row stride
    int64_t src_row_bytes[2];
    const int32_t* parity;
    const int32_t* table;       // paged: [R, M]; nullptr = dense
    int n;                      // 1 or 2 tensors
    int P, M, H, S;
    int n_pages;                // paged: pages in a pool
    int row_vecs;               // H * D * 2 / 16
    int head_vecs;              // D * 2 / 16
};
}  // namespace

__global__ __launch_bounds__(256) void kv_append_kernel(AppendDst d, int R, int pos)
{
    const int which = blockIdx.y;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)R * d.row_vecs) return;
    const int r = (int)(i / d.row_vecs), v = (int)(i % d.row_vecs);
    const int h = v / d.head_vecs, c = v % d.head_vecs;
    const vec16 x = *(const vec16*)(d.src[which] + (int64_t)r * d.src_row_bytes[which] + (int64_t)v * 16);
    char* base;
    int64_t unit, offset;            // (row or page) index, position inside it
    int span;                        // positions per unit
    if (d.table) {
        base = d.a[which]; unit = d.table[(int64_t)r * d.M + pos / d.P]; offset = pos % d.P; span = d.P;
        if (unit < 0 || unit >= d.n_pages) return;    // never the case for a table the library maintains
    } else {
        base = d.parity[r] ? d.b[which] : d.a[which]; unit = r; offset = pos; span = d.S;
    }
    *(vec16*)(base + (((unit * d.H + h) * span + offset) * d.head_vecs + c) * 16) = x;
}

}  // namespace psmc

extern "C" smc_status smc_kv_append(smc_ctx* ctx, int32_t k_tensor, int32_t v_tensor, const void* d_k_new, int64_t k_row_stride,
                                    const void* d_v_new, int64_t v_row_stride, int32_t pos)
{
    using namespace psmc;
    if (!ctx || !d_k_new) return SMC_E_NULL;
    const auto& cfg = ctx->cfg;
    if (cfg.kv_tensors < 1 || k_tensor < 0 || k_tensor >= cfg.kv_tensors || v_tensor < -1 || v_tensor >= cfg.kv_tensors)
        return SMC_E_RANGE;
    if (v_tensor >= 0 && !d_v_new) return SMC_E_NULL;
    if (v_tensor >= 0 && v_tensor == k_tensor) return SMC_E_RANGE;
    if (cfg.kv_elem_bytes != 2) return SMC_E_DTYPE;
    if (cfg.kv_D % 8 != 0) return SMC_E_ALIGN;
    const bool paged = ctx->paged.bound != 0;
    if (!paged && !ctx->kv_bound) return SMC_E_STATE;
    if (pos < 0 || pos >= cfg.kv_S) return SMC_E_RANGE;
    if (paged && pos >= ctx->paged.len) return SMC_E_STATE;      // the position has no page of its own yet
    const int64_t row_elems = (int64_t)cfg.kv_H * cfg.kv_D;
    const int n = v_tensor >= 0 ? 2 : 1;
    const void* src[2] = {d_k_new, d_v_new};
    const int64_t stride[2] = {k_row_stride, v_row_stride};
    for (int i = 0; i < n; ++i) {
        if (stride[i] < row_elems || stride[i] % 8 != 0 || ((uintptr_t)src[i] & 15u) != 0) return SMC_E_ALIGN;
    }
    AppendDst d{};
    const int32_t tensors[2] = {k_tensor, v_tensor};
    for (int i = 0; i < n; ++i) {
        if (paged) {
            d.a[i] = (char*)ctx->h_pools[tensors[i]];
        } else {
            d.a[i] = (char*)ctx->h_kvA[tensors[i]]; d.b[i] = (char*)ctx->h_kvB[tensors[i]];
            if (!d.a[i] || !d.b[i]) return SMC_E_STATE;
        }
        d.src[i] = (const char*)src[i];
        d.src_row_bytes[i] = stride[i] * 2;
    }
    d.parity = ctx->ws.parity;
    d.table = paged ? ctx->paged.table : nullptr;
    d.n = n;
    d.P = paged ? ctx->paged.P : 1; d.M = paged ? ctx->paged.M : 0;
    d.n_pages = paged ? cfg.B * ctx->paged.Q : 0;
    d.H = cfg.kv_H; d.S = cfg.kv_S;
    d.head_vecs = cfg.kv_D / 8;
    d.row_vecs = cfg.kv_H * d.head_vecs;
    const int64_t total = (int64_t)ctx->R * d.row_vecs;
    const dim3 grid((unsigned)((total + 255) / 256), (unsigned)n), block(256);
    hipLaunchKernelGGL(kv_append_kernel, grid, block, 0, ctx->stream, d, ctx->R, pos);
    return hipGetLastError() == hipSuccess ? SMC_OK : SMC_E_HIP;
}
