// smc_step_noalloc: a0 + a1 + a2 of smc_step for callers that cannot allocate device memory and hold no context.
//
// The vocabulary pass needs scratch beyond its inputs and outputs: one Partial record per (row, slice) and the
// per-row diagnostics the row finalizer writes.  smc_step takes them from the workspace given to smc_init; this entry
// point takes them from a file-scope device array instead, so that the call itself needs no workspace, no context and
// no allocation: it only enqueues the same two kernels on the caller's stream.
//
// The array exists once per GPU (each device that loads the library holds its own copy until the process ends).
// Its device address is looked up once per device with hipGetSymbolAddress and kept; host code never passes the
// array's name to a kernel.  Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
// (different streams, or different threads) race on it.  Only the per-row ticket counters have to start at zero; each call
// clears them first.  Every record that the finalizer reads is written by the vocabulary pass of the same call.
#include <math.h>

#include <mutex>

#include "smc_internal.hpp"

using namespace psmc;

namespace {

constexpr int kNoAllocMaxRows = SMC_NOALLOC_MAX_ROWS;
constexpr size_t kAlignUp = 256;
constexpr size_t up256(size_t x) { return (x + kAlignUp - 1) & ~(kAlignUp - 1); }

// layout of the scratch array for kNoAllocMaxRows rows (fixed offsets, whatever the call's R)
constexpr size_t kOffPartials = 0;
constexpr size_t kOffDelta = kOffPartials + up256((size_t)kNoAllocMaxRows * kMaxSplit * sizeof(Partial));
constexpr size_t kOffLogZ1 = kOffDelta + up256((size_t)kNoAllocMaxRows * 8);
constexpr size_t kOffLogZb = kOffLogZ1 + up256((size_t)kNoAllocMaxRows * 8);
constexpr size_t kOffGap = kOffLogZb + up256((size_t)kNoAllocMaxRows * 8);
constexpr size_t kOffSecond = kOffGap + up256((size_t)kNoAllocMaxRows * 8);
constexpr size_t kOffRowstat = kOffSecond + up256((size_t)kNoAllocMaxRows * 4);
constexpr size_t kOffTicket = kOffRowstat + up256((size_t)kNoAllocMaxRows * 12);
constexpr size_t kScratchBytes = kOffTicket + up256((size_t)kNoAllocMaxRows * 4);
static_assert(kScratchBytes <= (size_t)8 << 20, "the static scratch array is meant to stay modest");

constexpr int kMaxDevices = 64;
std::mutex g_lock;
char* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, once looked up

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

__global__ void clear_tickets_kernel(int32_t* tickets, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) tickets[i] = 0;
}

namespace {

// Device address of this GPU's scratch array (nullptr + error status on failure).
smc_status scratch_for_current_device(char** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return SMC_E_HIP; }
    if (dev < 0 || dev >= kMaxDevices) return SMC_E_STATE;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        char* p = nullptr;
        if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SMC_E_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SMC_OK;
}

}  // namespace

extern "C" smc_status smc_step_noalloc(const smc_config* cfg, void* hip_stream, const void* d_logits,
                                       int64_t row_stride_elems, int32_t t, double alpha_t, double alpha_prev,
                                       double tau_t, double* d_logW_inout, double* d_cumlogp_inout,
                                       int32_t* d_done_inout, int32_t* d_tokens_out)
{
    const smc_status cs = validate_config(cfg);
    if (cs != SMC_OK) return cs;
    if (!d_logits || !d_logW_inout || !d_cumlogp_inout || !d_tokens_out) return SMC_E_NULL;
    if (cfg->eos_id >= 0 && !d_done_inout) return SMC_E_NULL;
    const int64_t R = (int64_t)cfg->B * cfg->N;
    if (R > kNoAllocMaxRows) return SMC_E_SHAPE;          // the static scratch array holds records for this many rows
    const int esz = cfg->logits_dtype == SMC_BF16 ? 2 : 4;
    if (row_stride_elems < cfg->V) return SMC_E_SHAPE;
    if (((uintptr_t)d_logits & 15u) != 0 || (row_stride_elems * esz) % 16 != 0) return SMC_E_ALIGN;
    if (t < 1) return SMC_E_RANGE;
    if (!(alpha_t > 0.0) || !(alpha_prev >= 0.0) || !isfinite(alpha_t) || !isfinite(alpha_prev)) return SMC_E_RANGE;
    if (!isfinite(tau_t)) return SMC_E_RANGE;
    const double beta = tau_t <= 0.0 ? alpha_t : 1.0 / tau_t;
    if (!(beta > 0.0) || !isfinite(beta) || beta > 1.0e4) return SMC_E_RANGE;

    char* base = nullptr;
    const smc_status ss = scratch_for_current_device(&base);
    if (ss != SMC_OK) return ss;

    // a context on the stack: the caller's arrays are the state, the static array is the scratch; no history is
    // kept and no cache is bound, so the finalizer writes tokens, weights and sums only
    smc_ctx c{};
    c.cfg = *cfg;
    c.stream = (hipStream_t)hip_stream;
    c.R = (int)R;
    c.ws = Workspace{};
    c.ws.logW = d_logW_inout;
    c.ws.cumlogp = d_cumlogp_inout;
    c.ws.done = d_done_inout;
    c.ws.partials = (Partial*)(base + kOffPartials);
    c.ws.d_delta = (double*)(base + kOffDelta);
    c.ws.d_logZ1 = (double*)(base + kOffLogZ1);
    c.ws.d_logZb = (double*)(base + kOffLogZb);
    c.ws.d_gap = (double*)(base + kOffGap);
    c.ws.d_second = (int32_t*)(base + kOffSecond);
    c.ws.d_rowstat = (int32_t*)(base + kOffRowstat);
    c.ws.row_ticket = (int32_t*)(base + kOffTicket);
    c.paged = PagedKV{};
    auto_shape(c.R, cfg->V, cfg->logits_dtype, &c.wg_waves, &c.n_split);
    c.mask_words = (cfg->N + 63) / 64;
    // The per-row ticket counters of the kernel must start at zero.  They return to zero by themselves, but the array is
    // shared by every call on this GPU, so it is cleared here rather than trusted (a fill kernel, not a memset node: the
    // call may be under stream capture).
    hipLaunchKernelGGL(clear_tickets_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, c.stream, c.ws.row_ticket, (int)R);
    if (hipGetLastError() != hipSuccess) return SMC_E_HIP;
    return launch_vocab_pass(&c, d_logits, row_stride_elems, t, alpha_t, alpha_prev, tau_t, d_tokens_out, nullptr) == hipSuccess
               ? SMC_OK : SMC_E_HIP;
}
