// Step kernel over the quantized variables of one code width; included once per optimizer.
#pragma once
#include "omc_stream.h"

namespace omc {

#ifndef OMC_TUNE_WAVES_FP6
#define OMC_TUNE_WAVES_FP6 2
#endif
#ifndef OMC_TUNE_OCP_MAXMODE
#define OMC_TUNE_OCP_MAXMODE 2      // kStepSgd: the hardware FP8 variant serves plain SGD only
#endif
#ifndef OMC_TUNE_FP6_MAXMODE
#define OMC_TUNE_FP6_MAXMODE 2      // kStepSgd: the hardware 6-bit variant serves plain SGD only
#endif

struct StepArgs {
    uint8_t *arena;
    const uint8_t *plan;      // device copy of the plan blob
    uint64_t var_off, item_off;
    uint32_t first_item, nitems;
    uint32_t fp32_first, fp32_nitems;   // work items of fp32 variables appended to this launch's grid
    float *sb_table;
    const float *grads;
    float *st0, *st1;
    Partial *ws;
    OptConst oc;
};

// Variables kept in fp32 (paper Sec. 2.4, 2.5): the update alone, 16-byte pieces, coalesced.
template <int MODE>
__device__ __forceinline__ void do_fp32_item(const StepArgs &sa, uint32_t item) {
    const PlanItem *items = reinterpret_cast<const PlanItem *>(sa.plan + sa.item_off);
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(sa.plan + sa.var_off);
    const PlanItem it = to_scalar_regs(items[item]);
    const PlanVar pv = to_scalar_regs(vars[it.var]);
    const uint32_t lane = threadIdx.x;
    float *__restrict__ w = reinterpret_cast<float *>(sa.arena + pv.data_offset);
    const float *__restrict__ g = sa.grads + pv.aux_offset;
    float *__restrict__ m = sa.st0 ? sa.st0 + pv.aux_offset : nullptr;
    float *__restrict__ v = sa.st1 ? sa.st1 + pv.aux_offset : nullptr;
    const uint64_t n = pv.n;
    const uint64_t begin = static_cast<uint64_t>(it.chunk) * kChunkElems;
    constexpr int kIters = kChunkElems / 256;
#pragma unroll 4
    for (int j = 0; j < kIters; ++j) {
        const uint64_t e = begin + (static_cast<uint64_t>(j) * 64 + lane) * 4;
        if (e >= n) continue;
        float xw[4], xg[4], xm[4] = {0, 0, 0, 0}, xv[4] = {0, 0, 0, 0};
        const bool full = e + 4 <= n;
        if (full) {
            const float4 tw = *reinterpret_cast<const float4 *>(w + e);
            const float4 tg = *reinterpret_cast<const float4 *>(g + e);
            xw[0] = tw.x; xw[1] = tw.y; xw[2] = tw.z; xw[3] = tw.w;
            xg[0] = tg.x; xg[1] = tg.y; xg[2] = tg.z; xg[3] = tg.w;
            if (MODE >= kStepMomentum) {
                const float4 tm = *reinterpret_cast<const float4 *>(m + e);
                xm[0] = tm.x; xm[1] = tm.y; xm[2] = tm.z; xm[3] = tm.w;
            }
            if (MODE == kStepAdam) {
                const float4 tv = *reinterpret_cast<const float4 *>(v + e);
                xv[0] = tv.x; xv[1] = tv.y; xv[2] = tv.z; xv[3] = tv.w;
            }
        } else {
            for (int c = 0; c < 4; ++c) {
                const bool ok = e + c < n;
                xw[c] = ok ? w[e + c] : 0.0f;
                xg[c] = ok ? g[e + c] : 0.0f;
                if (MODE >= kStepMomentum) xm[c] = ok ? m[e + c] : 0.0f;
                if (MODE == kStepAdam) xv[c] = ok ? v[e + c] : 0.0f;
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) xw[c] = apply_update<MODE>(xw[c], xg[c], xm[c], xv[c], sa.oc);
        if (full) {
            *reinterpret_cast<float4 *>(w + e) = make_float4(xw[0], xw[1], xw[2], xw[3]);
            if (MODE >= kStepMomentum) *reinterpret_cast<float4 *>(m + e) = make_float4(xm[0], xm[1], xm[2], xm[3]);
            if (MODE == kStepAdam) *reinterpret_cast<float4 *>(v + e) = make_float4(xv[0], xv[1], xv[2], xv[3]);
        } else {
            for (int c = 0; c < 4; ++c) {
                if (e + c < n) {
                    w[e + c] = xw[c];
                    if (MODE >= kStepMomentum) m[e + c] = xm[c];
                    if (MODE == kStepAdam) v[e + c] = xv[c];
                }
            }
        }
    }
}

template <int B, int MODE, int VARIANT>
__global__ __launch_bounds__(64, (VARIANT == 3 ? OMC_TUNE_WAVES_FP6 : Tuning<MODE, B>::waves)) void step_kernel(StepArgs sa) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    if (blockIdx.x >= sa.nitems) {                       // the workgroups past the end serve fp32 variables
        do_fp32_item<MODE>(sa, sa.fp32_first + (blockIdx.x - sa.nitems));
        return;
    }
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
    do_chunk<B, MODE, VARIANT>(a, fp, sa.oc, it.chunk, lds, sa.ws + item);
}

template <int MODE>
inline int launch_step_group_mode(uint32_t bits, uint32_t variant, const StepArgs &sa, hipStream_t st) {
    // the hardware-conversion variant pays off where the vector ALU is the limit: plain SGD
    if (bits == 8 && variant == 2 && MODE <= OMC_TUNE_OCP_MAXMODE) {
        step_kernel<8, MODE, 2><<<dim3(sa.nitems + sa.fp32_nitems), dim3(64), 0, st>>>(sa);
        return static_cast<int>(hipGetLastError());
    }
    if (bits == 6 && variant == 3 && MODE <= OMC_TUNE_FP6_MAXMODE) {
        step_kernel<6, MODE, 3><<<dim3(sa.nitems + sa.fp32_nitems), dim3(64), 0, st>>>(sa);
        return static_cast<int>(hipGetLastError());
    }
    switch (bits) {
#define X(BITS)                                                              \
    case BITS:                                                               \
        if (variant == 1) step_kernel<BITS, MODE, 1><<<dim3(sa.nitems + sa.fp32_nitems), dim3(64), 0, st>>>(sa);   \
        else step_kernel<BITS, MODE, 0><<<dim3(sa.nitems + sa.fp32_nitems), dim3(64), 0, st>>>(sa);       \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

int launch_step_group_sgd(uint32_t bits, uint32_t variant, const StepArgs &sa, hipStream_t st);
int launch_step_group_momentum(uint32_t bits, uint32_t variant, const StepArgs &sa, hipStream_t st);
int launch_step_group_adam(uint32_t bits, uint32_t variant, const StepArgs &sa, hipStream_t st);

}  // namespace omc
