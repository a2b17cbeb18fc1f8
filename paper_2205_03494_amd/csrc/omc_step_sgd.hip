// Fused decompress -> sgd update -> recompress kernels, one per code width.
#include "omc_step_impl.h"

namespace omc {
int launch_step_group_sgd(uint32_t bits, uint32_t variant, const StepArgs &sa, bool keep, hipStream_t st) {
    return launch_step_group_mode<kStepSgd>(bits, variant, sa, keep, st);
}
}  // namespace omc
