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
#ifndef OMC_TUNE_SGD8_MAX_WAVES
#define OMC_TUNE_SGD8_MAX_WAVES 2      // waves per SIMD of the 8-bit SGD kernel with hardware conversion (0: no cap)
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
    uint32_t fp32_keep_items;           // the first so many fp32 work items keep their values cached from step to step
};

// Variables kept in fp32 (paper Sec. 2.4, 2.5): the update alone, 16-byte pieces, coalesced.
// Every stream is touched once per step, so all loads and stores are non-temporal; a batch of
// kFp32Batch pieces per lane is loaded before any of them is updated (memory-level parallelism is
// all this loop needs).
#ifndef OMC_TUNE_FP32_NT
#define OMC_TUNE_FP32_NT 1
#endif
#ifndef OMC_TUNE_FP32_BATCH
#define OMC_TUNE_FP32_BATCH 4
#endif
template <int MODE, bool KEEPW>
__device__ __forceinline__ void fp32_item_body(const StepArgs &sa, uint32_t item) {
    constexpr bool NT = OMC_TUNE_FP32_NT != 0;
    constexpr bool NTW = NT && !KEEPW;                   // the values themselves: read and rewritten by every step
    constexpr int kFp32Batch = OMC_TUNE_FP32_BATCH;
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
    static_assert(kIters % kFp32Batch == 0, "batches tile the chunk");
    auto ld = [&](const float *p, bool nt = NT) {
        const f32x4 *q = reinterpret_cast<const f32x4 *>(p);
        return nt ? __builtin_nontemporal_load(q) : *q;
    };
    auto st = [&](float *p, const f32x4 &x, bool nt = NT) {
        f32x4 *q = reinterpret_cast<f32x4 *>(p);
        if (nt) __builtin_nontemporal_store(x, q); else *q = x;
    };
    for (int j0 = 0; j0 < kIters; j0 += kFp32Batch) {
        const uint64_t e0 = begin + (static_cast<uint64_t>(j0) * 64 + lane) * 4;
        if (begin + static_cast<uint64_t>(j0 + kFp32Batch) * 256 <= n) {          // the whole batch is inside: wave-uniform
            f32x4 xw[kFp32Batch], xg[kFp32Batch], xm[kFp32Batch], xv[kFp32Batch];
#pragma unroll
            for (int u = 0; u < kFp32Batch; ++u) {
                const uint64_t e = e0 + static_cast<uint64_t>(u) * 256;
                xw[u] = ld(w + e, NTW);
                xg[u] = ld(g + e);
                xm[u] = (MODE >= kStepMomentum) ? ld(m + e) : f32x4{0, 0, 0, 0};
                xv[u] = (MODE == kStepAdam) ? ld(v + e) : f32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < kFp32Batch; ++u) {
                const uint64_t e = e0 + static_cast<uint64_t>(u) * 256;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float tm = xm[u][c], tv = xv[u][c];
                    xw[u][c] = apply_update<MODE>(xw[u][c], xg[u][c], tm, tv, sa.oc);
                    xm[u][c] = tm;
                    xv[u][c] = tv;
                }
                st(w + e, xw[u], NTW);
                if (MODE >= kStepMomentum) st(m + e, xm[u]);
                if (MODE == kStepAdam) st(v + e, xv[u]);
            }
            continue;
        }
        for (int u = 0; u < kFp32Batch; ++u) {                                     // the variable ends in this batch
            const uint64_t e = e0 + static_cast<uint64_t>(u) * 256;
            for (int c = 0; c < 4; ++c) {
                if (e + c >= n) break;
                float tm = (MODE >= kStepMomentum) ? m[e + c] : 0.0f, tv = (MODE == kStepAdam) ? v[e + c] : 0.0f;
                w[e + c] = apply_update<MODE>(w[e + c], g[e + c], tm, tv, sa.oc);
                if (MODE >= kStepMomentum) m[e + c] = tm;
                if (MODE == kStepAdam) v[e + c] = tv;
            }
        }
    }
}

template <int MODE>
__device__ __forceinline__ void do_fp32_item(const StepArgs &sa, uint32_t item) {
    if (item - sa.fp32_first < sa.fp32_keep_items) fp32_item_body<MODE, true>(sa, item);
    else fp32_item_body<MODE, false>(sa, item);
}

// KEEP: the launch's work items keep their packed codes cached from step to step; without it the code
// loads and stores carry the non-temporal hint.
// Occupancy: the register budget follows Tuning<>::waves (waves per SIMD the compiler must make room for).  The
// 8-bit SGD kernel with hardware conversion needs few registers and would run four waves per SIMD; it is held
// at two (8 workgroups per compute unit), because fewer streams open at once suit the memory system better when
// the traffic really comes from HBM (codes streamed, caches flushed between steps: 120 -> 113 us; caps of 10
// workgroups measure like 8, 6 and 4 are slower).  The kernels with more arithmetic per element lose 7-10 %
// under the same cap and are left alone.
template <int B, int MODE, int VARIANT>
struct StepOccupancy {
    static constexpr int min_waves = (VARIANT == 3) ? OMC_TUNE_WAVES_FP6 : Tuning<MODE, B>::waves;
    static constexpr bool capped = (VARIANT == 2 && MODE == kStepSgd && OMC_TUNE_SGD8_MAX_WAVES > 0);
    static constexpr int lo = capped ? (min_waves < OMC_TUNE_SGD8_MAX_WAVES ? min_waves : OMC_TUNE_SGD8_MAX_WAVES) : min_waves;
    static constexpr int hi = capped ? OMC_TUNE_SGD8_MAX_WAVES : 8;
};
template <int B, int MODE, int VARIANT, bool KEEP>
__global__ __attribute__((amdgpu_flat_work_group_size(64, 64)))
__attribute__((amdgpu_waves_per_eu(StepOccupancy<B, MODE, VARIANT>::lo, StepOccupancy<B, MODE, VARIANT>::hi)))
void step_kernel(StepArgs sa) {
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
    a.s = to_scalar_regs(sa.sb_table[2 * static_cast<uint64_t>(pv.sb_index)]);
    a.b = to_scalar_regs(sa.sb_table[2 * static_cast<uint64_t>(pv.sb_index) + 1]);
    const FmtParams fp = pv.fp;
    do_chunk<B, MODE, VARIANT, KEEP>(a, fp, sa.oc, it.chunk, lds, sa.ws + item);
}

// Variants 0 / 1 and, for code widths that can hold 16 mantissa bits, 4 / 5 (error-carrying sums).
template <int BITS, int MODE, bool KEEP>
inline void launch_step_generic_variant(uint32_t variant, dim3 grid, dim3 block, const StepArgs &sa, hipStream_t st) {
    if constexpr (BITS >= 18) {
        if (variant == 4) { step_kernel<BITS, MODE, 4, KEEP><<<grid, block, 0, st>>>(sa); return; }
        if (variant == 5) { step_kernel<BITS, MODE, 5, KEEP><<<grid, block, 0, st>>>(sa); return; }
    }
    if (variant == 1) step_kernel<BITS, MODE, 1, KEEP><<<grid, block, 0, st>>>(sa);
    else step_kernel<BITS, MODE, 0, KEEP><<<grid, block, 0, st>>>(sa);
}

template <int MODE, bool KEEP>
inline int launch_step_group_keep(uint32_t bits, uint32_t variant, const StepArgs &sa, hipStream_t st) {
    const dim3 grid(sa.nitems + sa.fp32_nitems), block(64);
    // the hardware-conversion variant pays off where the vector ALU is the limit: plain SGD
    if (bits == 8 && variant == 2 && MODE <= OMC_TUNE_OCP_MAXMODE) {
        step_kernel<8, MODE, 2, KEEP><<<grid, block, 0, st>>>(sa);
        return static_cast<int>(hipGetLastError());
    }
    if (bits == 6 && variant == 3 && MODE <= OMC_TUNE_FP6_MAXMODE) {
        step_kernel<6, MODE, 3, KEEP><<<grid, block, 0, st>>>(sa);
        return static_cast<int>(hipGetLastError());
    }
    switch (bits) {
#define X(BITS)                                                              \
    case BITS:                                                               \
        launch_step_generic_variant<BITS, MODE, KEEP>(variant, grid, block, sa, st); \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

template <int MODE>
inline int launch_step_group_mode(uint32_t bits, uint32_t variant, const StepArgs &sa, bool keep, hipStream_t st) {
    return keep ? launch_step_group_keep<MODE, true>(bits, variant, sa, st)
                : launch_step_group_keep<MODE, false>(bits, variant, sa, st);
}

int launch_step_group_sgd(uint32_t bits, uint32_t variant, const StepArgs &sa, bool keep, hipStream_t st);
int launch_step_group_momentum(uint32_t bits, uint32_t variant, const StepArgs &sa, bool keep, hipStream_t st);
int launch_step_group_adam(uint32_t bits, uint32_t variant, const StepArgs &sa, bool keep, hipStream_t st);

}  // namespace omc
