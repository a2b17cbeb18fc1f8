// Shared by the weight-gradient kernels (omc_dw.hip) and their any-code-width update kernels.
#pragma once
#include "omc_stream.h"

namespace omc {

constexpr int kDwCols = 128, kDwStep = 32;

struct DwArgs {
    const uint16_t *X, *dY;
    uint32_t *codes;
    const float *sb;
    float *st0, *st1;
    float *dW_out;
    Partial *ws;
    float *partials;         // split contraction: [tile][split][ROWS * 128] accumulators
    uint32_t nsplit;         // workgroups per tile along the contraction (gridDim.z)
    uint32_t park;           // 1: the matrix-core kernel only parks its accumulators (several splits, or a code
                             // width other than 8, whose update runs in a kernel of its own)
    FmtParams fp;
    OptConst oc;
    uint32_t M, N, K;
};

// Second kernel of omc_dw_update_recompress for code widths other than 8: one launcher per optimizer.
int launch_dw_generic_sgd(uint32_t bits, uint32_t variant, uint32_t rows, const DwArgs &a, uint32_t tiles, uint32_t tiles_x,
                          hipStream_t st);
int launch_dw_generic_momentum(uint32_t bits, uint32_t variant, uint32_t rows, const DwArgs &a, uint32_t tiles, uint32_t tiles_x,
                               hipStream_t st);
int launch_dw_generic_adam(uint32_t bits, uint32_t variant, uint32_t rows, const DwArgs &a, uint32_t tiles, uint32_t tiles_x,
                           hipStream_t st);

}  // namespace omc
