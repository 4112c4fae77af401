// The vocabulary-pass kernels for fp32 logits (a translation unit of its own so that the two dtypes compile in parallel).
#include "vocab_pass_kernel.hpp"

namespace psmc {
hipError_t launch_vocab_f32(smc_ctx* c, const StepArgs& a, int P) { return launch_vocab_dt<SMC_F32>(c, a, P); }
}  // namespace psmc
