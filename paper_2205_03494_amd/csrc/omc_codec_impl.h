// Kernels shared by the single-variable calls (omc_compress, omc_decompress) and the variable-set
// calls (omc_compress_set, omc_decompress_set): the same full-tile / tail device code, fed either
// from one variable described in the kernel arguments or from a plan's work items.
#pragma once
#include "omc_stream.h"

namespace omc {

struct CodecArgs {
    uint8_t *arena;              // base of the data offsets (single variable: its packed buffer)
    const uint8_t *plan;         // device plan blob, or nullptr: one variable, described by `single`
    uint64_t var_off, item_off;
    uint32_t first_item, nitems;
    uint32_t fp32_first, fp32_nitems;   // set calls: copies of fp32 variables appended to the grid
    PlanVar single;
    uint32_t single_tiles;       // single variable: full tiles per work item
    uint32_t single_tail;        // single variable: 1 = one more workgroup of the full-tile launch serves the ragged tail
    const float *sb_in;          // decompress: (s, b) table / pair, nullptr = (1, 0)
    const float *vin;            // compress: fp32 values, indexed by aux_offset
    float *vout;                 // decompress: fp32 output, indexed by aux_offset
    Partial *ws;
};

// fp32 variable of a set: plain copy between the aux-indexed array and the arena (16-byte pieces)
template <int MODE>
__device__ __forceinline__ void copy_fp32_item(const CodecArgs &ca, uint32_t item) {
    const PlanItem *items = reinterpret_cast<const PlanItem *>(ca.plan + ca.item_off);
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(ca.plan + ca.var_off);
    const PlanItem it = to_scalar_regs(items[item]);
    const PlanVar pv = to_scalar_regs(vars[it.var]);
    const uint32_t lane = threadIdx.x;
    float *in_arena = reinterpret_cast<float *>(ca.arena + pv.data_offset);
    const float *src = (MODE == kCompress) ? ca.vin + pv.aux_offset : in_arena;
    float *dst = (MODE == kCompress) ? in_arena : ca.vout + pv.aux_offset;
    const uint64_t begin = static_cast<uint64_t>(it.chunk) * kChunkElems;
    constexpr int kBatch = 8;                              // pieces per lane in flight; both streams are touched once
    for (int j0 = 0; j0 < kChunkElems / 256; j0 += kBatch) {
        const uint64_t e0 = begin + (static_cast<uint64_t>(j0) * 64 + lane) * 4;
        if (begin + static_cast<uint64_t>(j0 + kBatch) * 256 <= pv.n) {   // the whole batch is inside: wave-uniform
            f32x4 x[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                x[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src + e0 + static_cast<uint64_t>(u) * 256));
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                __builtin_nontemporal_store(x[u], reinterpret_cast<f32x4 *>(dst + e0 + static_cast<uint64_t>(u) * 256));
            continue;
        }
        for (int u = 0; u < kBatch; ++u) {                   // the variable ends in this batch
            const uint64_t e = e0 + static_cast<uint64_t>(u) * 256;
            for (int c = 0; c < 4; ++c)
                if (e + c < pv.n) dst[e + c] = src[e + c];
        }
    }
}

template <int MODE>
__device__ __forceinline__ void codec_tile_args(const CodecArgs &ca, const PlanVar &pv, uint32_t var, TileArgs &a) {
    a.codes = reinterpret_cast<uint32_t *>(ca.arena + pv.data_offset);
    a.total_dwords = pv.total_dwords;
    a.n = pv.n;
    a.s = 1.0f;
    a.b = 0.0f;
    if (MODE == kCompress) {
        a.vin = ca.vin + pv.aux_offset;
    } else {
        a.vout = ca.vout + pv.aux_offset;
        if (ca.sb_in) {
            a.s = to_scalar_regs(ca.sb_in[2 * static_cast<uint64_t>(var)]);
            a.b = to_scalar_regs(ca.sb_in[2 * static_cast<uint64_t>(var) + 1]);
        }
    }
}

template <int B, int MODE, int VARIANT>
__global__ __launch_bounds__(64, (Tuning<MODE, B>::waves)) void codec_kernel(CodecArgs ca) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    if (blockIdx.x >= ca.nitems) {
        copy_fp32_item<MODE>(ca, ca.fp32_first + (blockIdx.x - ca.nitems));
        return;
    }
    uint32_t item = blockIdx.x, var = 0, chunk = blockIdx.x;
    PlanVar pv = ca.single;
    uint32_t tiles = tiles_per_chunk(B);
    if (!ca.plan) {
        tiles = ca.single_tiles;
        if (ca.single_tail && blockIdx.x == ca.nitems - 1) {       // the last workgroup: the variable's ragged tail
            TileArgs a{};
            codec_tile_args<MODE>(ca, pv, 0, a);
            OptConst oc{};
            do_tail<MODE, variant_wide(VARIANT)>(a, pv.fp, oc, ca.ws + item);   // (a format's rounding kind follows its variant)
            return;
        }
    }
    if (ca.plan) {
        const PlanItem *items = reinterpret_cast<const PlanItem *>(ca.plan + ca.item_off);
        const PlanVar *vars = reinterpret_cast<const PlanVar *>(ca.plan + ca.var_off);
        item = ca.first_item + blockIdx.x;
        const PlanItem it = to_scalar_regs(items[item]);
        chunk = it.chunk;
        pv = to_scalar_regs(vars[it.var]);
        var = pv.sb_index;
    }
    TileArgs a{};
    codec_tile_args<MODE>(ca, pv, var, a);
    OptConst oc{};
    do_chunk<B, MODE, VARIANT>(a, pv.fp, oc, chunk, lds, ca.ws + item, tiles);
}

template <int MODE, bool WIDE>
__global__ __launch_bounds__(64) void codec_tail_kernel(CodecArgs ca) {
    uint32_t item = ca.first_item, var = 0;     // single variable: first_item is the tail's partial slot
    PlanVar pv = ca.single;
    if (ca.plan) {
        const PlanItem *items = reinterpret_cast<const PlanItem *>(ca.plan + ca.item_off);
        const PlanVar *vars = reinterpret_cast<const PlanVar *>(ca.plan + ca.var_off);
        item = ca.first_item + blockIdx.x;
        const PlanItem it = to_scalar_regs(items[item]);
        pv = to_scalar_regs(vars[it.var]);
        var = pv.sb_index;
    }
    TileArgs a{};
    codec_tile_args<MODE>(ca, pv, var, a);
    OptConst oc{};
    do_tail<MODE, WIDE>(a, pv.fp, oc, ca.ws + item);
}

}  // namespace omc
