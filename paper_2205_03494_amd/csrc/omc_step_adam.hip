// Fused decompress -> adam update -> recompress kernels, one per code width.
#include "omc_step_impl.h"

namespace omc {
int launch_step_group_adam(uint32_t bits, uint32_t variant, const StepArgs &sa, bool keep, hipStream_t st) {
    return launch_step_group_mode<kStepAdam>(bits, variant, sa, keep, st);
}
}  // namespace omc
