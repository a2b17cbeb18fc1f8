// Step kernel over the quantized variables of one code width; included once per optimizer.
#pragma once
#include "omc_stream.h"

namespace omc {

struct StepArgs {
    uint8_t *arena;
    const uint8_t *plan;      // device copy of the plan blob
    uint64_t var_off, item_off;
    uint32_t first_item, nitems;
    float *sb_table;
    const float *grads;
    float *st0, *st1;
    Partial *ws;
    OptConst oc;
};

template <int B, int MODE, bool WIDE>
__global__ __launch_bounds__(64, (Tuning<MODE, B>::waves)) void step_kernel(StepArgs sa) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    const PlanItem *items = reinterpret_cast<const PlanItem *>(sa.plan + sa.item_off);
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(sa.plan + sa.var_off);
    const uint32_t item = sa.first_item + blockIdx.x;
    const PlanItem it = to_scalar_regs(items[item]);
    const PlanVar pv = to_scalar_regs(vars[it.var]);
    TileArgs a{};
    a.codes = reinterpret_cast<uint32_t *>(sa.arena + pv.data_offset);
    a.total_dwords = pv.total_dwords;
    a.grad = sa.grads + pv.aux_offset;
    a.st0 = sa.st0 ? sa.st0 + pv.aux_offset : nullptr;
    a.st1 = sa.st1 ? sa.st1 + pv.aux_offset : nullptr;
    a.n = pv.n;
    a.s = to_scalar_regs(sa.sb_table[2 * static_cast<uint64_t>(it.var)]);
    a.b = to_scalar_regs(sa.sb_table[2 * static_cast<uint64_t>(it.var) + 1]);
    const FmtParams fp = pv.fp;
    do_chunk<B, MODE, WIDE>(a, fp, sa.oc, it.chunk, lds, sa.ws + item);
}

template <int MODE>
inline int launch_step_group_mode(uint32_t bits, bool wide, const StepArgs &sa, hipStream_t st) {
    switch (bits) {
#define X(BITS)                                                              \
    case BITS:                                                               \
        if (wide) step_kernel<BITS, MODE, true><<<dim3(sa.nitems), dim3(64), 0, st>>>(sa);   \
        else step_kernel<BITS, MODE, false><<<dim3(sa.nitems), dim3(64), 0, st>>>(sa);       \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

int launch_step_group_sgd(uint32_t bits, bool wide, const StepArgs &sa, hipStream_t st);
int launch_step_group_momentum(uint32_t bits, bool wide, const StepArgs &sa, hipStream_t st);
int launch_step_group_adam(uint32_t bits, bool wide, const StepArgs &sa, hipStream_t st);

}  // namespace omc
