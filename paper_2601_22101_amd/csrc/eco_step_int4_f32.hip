// Instantiations of the fused ECO step kernel: INT4 codes, fp32 optimizer state.
#include "eco_step_kernel.hpp"

namespace eco {
hipError_t launch_step_int4_f32(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
  return launch_step_variants<FMT_INT4, false>(kv, args, grid, stream);
}
}  // namespace eco
