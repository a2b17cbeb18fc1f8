// omc_step_update_recompress: orchestration over the plan's groups, the fp32-variable kernels
// and the per-variable finalize.
#include "omc_step_impl.h"

namespace omc {

// Variables kept in fp32 (paper Sec. 2.4, 2.5): the update alone, 16-byte pieces, coalesced.
template <int MODE>
__global__ __launch_bounds__(64) void step_fp32_kernel(StepArgs sa) {
    const PlanItem *items = reinterpret_cast<const PlanItem *>(sa.plan + sa.item_off);
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(sa.plan + sa.var_off);
    const PlanItem it = to_scalar_regs(items[sa.first_item + blockIdx.x]);
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

// Ragged tails of quantized variables, one wave each (code width read from the plan).
template <int MODE, bool WIDE>
__global__ __launch_bounds__(64) void step_tail_kernel(StepArgs sa) {
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
    do_tail<MODE, WIDE>(a, fp, sa.oc, sa.ws + item);
}

template <int MODE>
static int launch_tail(bool wide, const StepArgs &sa, hipStream_t st) {
    if (wide) step_tail_kernel<MODE, true><<<dim3(sa.nitems), dim3(64), 0, st>>>(sa);
    else step_tail_kernel<MODE, false><<<dim3(sa.nitems), dim3(64), 0, st>>>(sa);
    return static_cast<int>(hipGetLastError());
}

// One wave per variable: new (s, b) of every quantized variable from its chunks' partials.
__global__ __launch_bounds__(64) void finalize_plan_kernel(const uint8_t *__restrict__ plan, uint64_t var_off,
                                                           const Partial *__restrict__ ws,
                                                           float *__restrict__ sb_table) {
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(plan + var_off);
    const PlanVar &pv = vars[blockIdx.x];
    if (!(pv.flags & OMC_VAR_QUANTIZED)) return;
    finalize_variable(pv.nitems ? ws + pv.first_item : ws, pv.nitems,
                      pv.tail_item != kNoItem ? ws + pv.tail_item : nullptr, pv.n,
                      !(pv.flags & OMC_VAR_NO_PVT), sb_table + 2 * static_cast<uint64_t>(blockIdx.x));
}

int launch_step(void *arena, const PlanHeader *ph, const void *plan_dev, float *sb_table, const float *grads,
                float *state0, float *state1, const omc_opt &opt, Partial *ws, void *stream,
                void *const *events) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t launch = 0;
    auto mark = [&](uint32_t which) -> int {   // optional caller-owned events around each launch
        if (!events) return 0;
        return static_cast<int>(hipEventRecord(static_cast<hipEvent_t>(events[2 * launch + which]), st));
    };
    const uint8_t *ph_bytes = reinterpret_cast<const uint8_t *>(ph);
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(ph_bytes + ph->group_off);
    StepArgs sa{};
    sa.arena = static_cast<uint8_t *>(arena);
    sa.plan = static_cast<const uint8_t *>(plan_dev);
    sa.var_off = ph->var_off;
    sa.item_off = ph->item_off;
    sa.sb_table = sb_table;
    sa.grads = grads;
    sa.st0 = opt.kind >= OMC_MOMENTUM ? state0 : nullptr;
    sa.st1 = opt.kind == OMC_ADAM ? state1 : nullptr;
    sa.ws = ws;
    sa.oc = OptConst{opt.lr, opt.momentum, opt.beta1, opt.beta2, opt.eps, opt.one_minus_beta1,
                     opt.one_minus_beta2, opt.bias_corr1, opt.bias_corr2};
    for (uint32_t gi = 0; gi < ph->ngroups; ++gi) {
        const PlanGroup &g = groups[gi];
        if (g.nitems == 0) continue;
        sa.first_item = g.first_item;
        sa.nitems = g.nitems;
        int rc = mark(0);
        if (rc != 0) return rc;
        if (g.kind == kGroupTail) {
            if (opt.kind == OMC_SGD) rc = launch_tail<kStepSgd>(g.wide != 0, sa, st);
            else if (opt.kind == OMC_MOMENTUM) rc = launch_tail<kStepMomentum>(g.wide != 0, sa, st);
            else rc = launch_tail<kStepAdam>(g.wide != 0, sa, st);
        } else if (g.kind == kGroupFp32) {
            if (opt.kind == OMC_SGD) step_fp32_kernel<kStepSgd><<<dim3(g.nitems), dim3(64), 0, st>>>(sa);
            else if (opt.kind == OMC_MOMENTUM) step_fp32_kernel<kStepMomentum><<<dim3(g.nitems), dim3(64), 0, st>>>(sa);
            else step_fp32_kernel<kStepAdam><<<dim3(g.nitems), dim3(64), 0, st>>>(sa);
            rc = static_cast<int>(hipGetLastError());
        } else if (opt.kind == OMC_SGD) {
            rc = launch_step_group_sgd(g.bits, g.wide != 0, sa, st);
        } else if (opt.kind == OMC_MOMENTUM) {
            rc = launch_step_group_momentum(g.bits, g.wide != 0, sa, st);
        } else {
            rc = launch_step_group_adam(g.bits, g.wide != 0, sa, st);
        }
        if (rc != 0) return rc;
        rc = mark(1);
        if (rc != 0) return rc;
        ++launch;
    }
    if (ph->nquant > 0) {
        int rc = mark(0);
        if (rc != 0) return rc;
        finalize_plan_kernel<<<dim3(ph->nvars), dim3(64), 0, st>>>(sa.plan, ph->var_off, ws, sb_table);
        rc = static_cast<int>(hipGetLastError());
        if (rc != 0) return rc;
        return mark(1);
    }
    return 0;
}

}  // namespace omc
