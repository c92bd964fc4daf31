// Instantiations of the fused ECO step kernel: FP8 codes, bfloat16 optimizer state.
#include "eco_step_kernel.hpp"

namespace eco {
hipError_t launch_step_fp8_bf16(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
  return launch_step_variants<FMT_FP8, true>(kv, args, grid, stream);
}
}  // namespace eco
