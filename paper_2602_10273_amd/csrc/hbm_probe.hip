// Measured HBM ceilings of the device this library runs on, as a second denominator beside the published peak:
// plain streaming kernels (16-byte vectors, persistent grid-stride, 4 vectors in flight per thread) with the
// read : write mixes of the library's two dominant kernels.  Not part of the method.
//   kind 0  read only (non-temporal loads)            -- the mix of the vocabulary pass
//   kind 1  write only
//   kind 2  copy, 1 read : 1 write (first half of the buffer to the second half)
//   kind 3  fan-out, 1 read : 3 writes (first quarter to the other three) -- the mix of a reorder in which each
//           surviving ancestor has three moved descendants
#include <hip/hip_runtime.h>

#include "power_smc.h"

namespace psmc {
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256, kInFlight = 4;

__global__ __launch_bounds__(kThreads) void hbm_probe_read(const vec16* __restrict__ p, size_t n_vec, unsigned* sink)
{
    unsigned acc = 0;
    const size_t stride = (size_t)gridDim.x * kThreads * kInFlight;
    for (size_t base = (size_t)blockIdx.x * kThreads * kInFlight + threadIdx.x; base < n_vec; base += stride) {
        vec16 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const size_t i = base + (size_t)u * kThreads;
            v[u] = i < n_vec ? __builtin_nontemporal_load(p + i) : vec16{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;               // keeps the loads alive; practically never true
}

// Reads n_vec vectors from src once and writes them to `copies` destinations dst, dst + n_vec, ...; copies = 0 with
// src == nullptr is the write-only case (one destination, a constant pattern).
__global__ __launch_bounds__(kThreads) void hbm_probe_fanout(const vec16* __restrict__ src, vec16* __restrict__ dst, size_t n_vec,
                                                         int copies)
{
    const size_t stride = (size_t)gridDim.x * kThreads * kInFlight;
    for (size_t base = (size_t)blockIdx.x * kThreads * kInFlight + threadIdx.x; base < n_vec; base += stride) {
        vec16 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const size_t i = base + (size_t)u * kThreads;
            v[u] = (src && i < n_vec) ? src[i] : vec16{1u, 2u, 3u, (unsigned)blockIdx.x};
        }
        for (int w = 0; w < (src ? copies : 1); ++w)
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const size_t i = base + (size_t)u * kThreads;
                if (i < n_vec) __builtin_nontemporal_store(v[u], dst + (size_t)w * n_vec + i);
            }
    }
}
}  // namespace psmc

using namespace psmc;

extern "C" smc_status smc_hbm_probe(int32_t kind, void* d_buf, size_t bytes, void* hip_stream, double* h_gbps)
{
    if (!d_buf || !h_gbps) return SMC_E_NULL;
    if (kind < 0 || kind > 3) return SMC_E_RANGE;
    if (((uintptr_t)d_buf & 15u) != 0) return SMC_E_ALIGN;
    if (bytes < (size_t)1 << 20 || bytes % 64 != 0) return SMC_E_SHAPE;
    hipStream_t st = (hipStream_t)hip_stream;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess) return SMC_E_HIP;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const dim3 grid((unsigned)(cus * 4)), block(kThreads);
    const size_t n_all = bytes / 16;
    vec16* p = (vec16*)d_buf;
    size_t moved = 0;
    auto launch = [&]() {
        switch (kind) {
            case 0: hipLaunchKernelGGL(hbm_probe_read, grid, block, 0, st, p, n_all, (unsigned*)d_buf); moved = bytes; break;
            case 1: hipLaunchKernelGGL(hbm_probe_fanout, grid, block, 0, st, (const vec16*)nullptr, p, n_all, 0); moved = bytes; break;
            case 2: hipLaunchKernelGGL(hbm_probe_fanout, grid, block, 0, st, p, p + n_all / 2, n_all / 2, 1); moved = (n_all / 2) * 32; break;
            default: hipLaunchKernelGGL(hbm_probe_fanout, grid, block, 0, st, p, p + n_all / 4, n_all / 4, 3); moved = (n_all / 4) * 64; break;
        }
    };
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return SMC_E_HIP;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return SMC_E_HIP; }
    launch();                                           // warm-up
    const int reps = 3;
    bool ok = hipEventRecord(a, st) == hipSuccess;
    for (int i = 0; i < reps; ++i) launch();
    ok = ok && hipEventRecord(b, st) == hipSuccess && hipEventSynchronize(b) == hipSuccess && hipGetLastError() == hipSuccess;
    float ms = 0.f;
    ok = ok && hipEventElapsedTime(&ms, a, b) == hipSuccess && ms > 0.f;
    (void)hipEventDestroy(a); (void)hipEventDestroy(b);
    if (!ok) return SMC_E_HIP;
    *h_gbps = (double)moved * reps / (ms * 1e-3) / 1e9;
    return SMC_OK;
}
