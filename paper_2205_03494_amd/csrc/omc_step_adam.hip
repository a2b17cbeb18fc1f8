// Fused decompress -> adam update -> recompress kernels, one per code width.
#include "omc_step_impl.h"

namespace omc {
int launch_step_group_adam(uint32_t bits, bool wide, const StepArgs &sa, hipStream_t st) {
    return launch_step_group_mode<kStepAdam>(bits, wide, sa, st);
}
}  // namespace omc
