// omc_step_update_recompress: orchestration over the plan's groups, the fp32-variable kernels
// and the per-variable finalize.
#include <algorithm>

#include "omc_step_impl.h"

#ifndef OMC_TUNE_KEEP_BUDGET_MIB
#define OMC_TUNE_KEEP_BUDGET_MIB 224     // packed codes that stay cached when the set's codes do not fit as a whole
#endif
#ifndef OMC_TUNE_KEEP_FP32
#define OMC_TUNE_KEEP_FP32 1             // bit k: optimizer kind k keeps fp32 values cached (measured: pays for SGD only)
#endif
#ifndef OMC_TUNE_KEEP_ALL_MIB
#define OMC_TUNE_KEEP_ALL_MIB 264        // up to this size all codes stay cached
#endif

namespace omc {

template <int MODE>
__global__ __launch_bounds__(64) void step_fp32_kernel(StepArgs sa) {
    do_fp32_item<MODE>(sa, sa.first_item + blockIdx.x);
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
    a.s = to_scalar_regs(sa.sb_table[2 * static_cast<uint64_t>(pv.sb_index)]);
    a.b = to_scalar_regs(sa.sb_table[2 * static_cast<uint64_t>(pv.sb_index) + 1]);
    const FmtParams fp = pv.fp;
    do_tail<MODE, WIDE>(a, fp, sa.oc, sa.ws + item);
}

template <int MODE>
static int launch_tail(bool wide, const StepArgs &sa, hipStream_t st) {
    if (wide) step_tail_kernel<MODE, true><<<dim3(sa.nitems), dim3(64), 0, st>>>(sa);
    else step_tail_kernel<MODE, false><<<dim3(sa.nitems), dim3(64), 0, st>>>(sa);
    return static_cast<int>(hipGetLastError());
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
    // the fp32 variables ride along with the first full-tile launch as extra workgroups
    const PlanGroup *fp32_group = nullptr;
    bool fuse = false;
    for (uint32_t gi = 0; gi < ph->ngroups; ++gi) {
        if (groups[gi].kind == kGroupFp32 && groups[gi].nitems > 0) fp32_group = &groups[gi];
        if (groups[gi].kind == kGroupFull && groups[gi].nitems > 0) fuse = true;
    }
    fuse = fuse && fp32_group != nullptr;
    bool fused_done = false;
    // Packed codes are read and rewritten by every step.  In a training loop a forward and a backward pass lie
    // between two steps and nothing survives in the caches, so by default every code access carries the
    // non-temporal hint.  A caller that runs steps back to back asks for OMC_OPT_KEEP_CODES: the codes then
    // come back from the memory-side cache at the next step if they still sit there.  Work items get to keep
    // their codes cached, in launch order, up to a budget below that cache's 256 MB; the codes of all other
    // items carry the non-temporal hint and pass it by.  A group whose items fall on both sides of the limit
    // is launched in two parts.
    uint64_t keep_budget = 0;                              // bytes of packed codes that stay cached
    uint32_t fp32_keep_items = 0;                          // fp32 work items whose values stay cached
    if (opt.flags & OMC_OPT_KEEP_CODES) {                  // (default: other work runs between two steps, nothing would survive)
        const uint64_t cache = static_cast<uint64_t>(OMC_TUNE_KEEP_BUDGET_MIB) << 20;
        uint64_t all_codes = 0;
        for (uint32_t gi = 0; gi < ph->ngroups; ++gi)
            if (groups[gi].kind == kGroupFull) all_codes += static_cast<uint64_t>(groups[gi].nitems) * tiles_per_chunk(groups[gi].bits) * kTileElems * groups[gi].bits / 8;
        // a set that exceeds the cache by little still gets most of its hits and is not worth a second, small launch
        keep_budget = all_codes <= (static_cast<uint64_t>(OMC_TUNE_KEEP_ALL_MIB) << 20) ? all_codes : cache;
        // what the codes leave goes to the values of the fp32 variables, which are read and rewritten in place as well
        // (optimizer state is not worth keeping: measured slower)
        const uint64_t left = cache > all_codes ? cache - all_codes : 0;
        if (fp32_group && ((OMC_TUNE_KEEP_FP32 >> opt.kind) & 1)) fp32_keep_items = static_cast<uint32_t>(std::min<uint64_t>(fp32_group->nitems, left / (4ull * kChunkElems)));
    }
    auto take = [&](uint32_t nitems, uint64_t item_bytes) -> uint32_t {   // how many of nitems the budget still covers
        const uint64_t k = std::min<uint64_t>(nitems, keep_budget / item_bytes);
        keep_budget -= k * item_bytes;
        return static_cast<uint32_t>(k);
    };
    for (uint32_t gi = 0; gi < ph->ngroups; ++gi) {
        const PlanGroup &g = groups[gi];
        if (g.nitems == 0) continue;
        if (fuse && g.kind == kGroupFp32) continue;
        sa.first_item = g.first_item;
        sa.nitems = g.nitems;
        sa.fp32_first = 0;
        sa.fp32_nitems = 0;
        auto ride_along = [&]() {                                          // with the first full-tile launch of the step
            if (!fuse || fused_done) return;
            sa.fp32_first = fp32_group->first_item;
            sa.fp32_nitems = fp32_group->nitems;
            sa.fp32_keep_items = fp32_keep_items;
            fused_done = true;
        };
        int rc = mark(0);
        if (rc != 0) return rc;
        if (g.kind == kGroupTail) {
            if (opt.kind == OMC_SGD) rc = launch_tail<kStepSgd>(g.wide != 0, sa, st);
            else if (opt.kind == OMC_MOMENTUM) rc = launch_tail<kStepMomentum>(g.wide != 0, sa, st);
            else rc = launch_tail<kStepAdam>(g.wide != 0, sa, st);
        } else if (g.kind == kGroupFp32) {
            sa.fp32_first = g.first_item;
            sa.fp32_keep_items = fp32_keep_items;
            if (opt.kind == OMC_SGD) step_fp32_kernel<kStepSgd><<<dim3(g.nitems), dim3(64), 0, st>>>(sa);
            else if (opt.kind == OMC_MOMENTUM) step_fp32_kernel<kStepMomentum><<<dim3(g.nitems), dim3(64), 0, st>>>(sa);
            else step_fp32_kernel<kStepAdam><<<dim3(g.nitems), dim3(64), 0, st>>>(sa);
            rc = static_cast<int>(hipGetLastError());
        } else {
            const uint32_t kept = take(g.nitems, static_cast<uint64_t>(tiles_per_chunk(g.bits)) * kTileElems * g.bits / 8);
            for (int part = 0; part < 2 && rc == 0; ++part) {              // the cached items, then the streaming ones
                sa.first_item = g.first_item + (part == 0 ? 0 : kept);
                sa.nitems = part == 0 ? kept : g.nitems - kept;
                if (sa.nitems == 0) continue;
                sa.fp32_first = 0;
                sa.fp32_nitems = 0;
                ride_along();
                if (opt.kind == OMC_SGD) rc = launch_step_group_sgd(g.bits, g.wide, sa, part == 0, st);
                else if (opt.kind == OMC_MOMENTUM) rc = launch_step_group_momentum(g.bits, g.wide, sa, part == 0, st);
                else rc = launch_step_group_adam(g.bits, g.wide, sa, part == 0, st);
            }
        }
        if (rc != 0) return rc;
        rc = mark(1);
        if (rc != 0) return rc;
        ++launch;
    }
    if (ph->nquant > 0) {
        int rc = mark(0);
        if (rc != 0) return rc;
        finalize_plan_kernel<kFinalizeWaves><<<dim3(ph->nvars), dim3(64 * kFinalizeWaves), 0, st>>>(sa.plan, ph->var_off, ws, sb_table);
        rc = static_cast<int>(hipGetLastError());
        if (rc != 0) return rc;
        return mark(1);
    }
    return 0;
}

}  // namespace omc
