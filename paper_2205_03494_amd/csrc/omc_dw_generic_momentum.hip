// Update kernels of the fused weight-gradient step for every code width, momentum optimizer.
#include "omc_dw_generic_impl.h"

namespace omc {
int launch_dw_generic_momentum(uint32_t bits, uint32_t variant, uint32_t rows, const DwArgs &a, uint32_t tiles, uint32_t tiles_x,
                          hipStream_t st) {
    return launch_dw_generic_mode<kStepMomentum>(bits, variant, rows, a, tiles, tiles_x, st);
}
}  // namespace omc
