// Update kernel of the fused weight-gradient step for any code width (included once per optimizer).
// The matrix-core kernel has parked its accumulators in the workspace (accumulator layout, one or
// several contraction splits); here one wave takes a slab of 16 weight rows x 128 columns = 2048
// elements, sums the splits in order, and runs the same cycle as the streaming step kernels on it: a
// tile row is 128 consecutive elements of the variable, i.e. 4 B whole dwords of the packed stream
// (16-byte aligned), so with four lanes per row a lane again owns 32 consecutive elements = B dwords.
// Only the addressing differs from a contiguous tile: every 16-byte piece is located through its row.
#pragma once
#include "omc_dw_args.h"

namespace omc {

template <int B, int MODE, bool WIDE, bool EXACT = false>
__global__ __launch_bounds__(64, 2) void dw_reduce_update_generic_kernel(DwArgs a, uint32_t tiles_x, uint32_t rows) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    const uint32_t lane = threadIdx.x;
    const uint32_t f_row = lane & 31u, f_half = lane >> 5;
    // slab = (tile, wave of the first kernel, 32-row MFMA tile mi, half h of it)
    const uint32_t mi_count = rows / 128;
    uint32_t id = blockIdx.x;
    const uint32_t h = id & 1u; id >>= 1;
    const uint32_t mi = id % mi_count; id /= mi_count;
    const uint32_t wave = id & 3u;
    const uint32_t block = id >> 2;
    const uint32_t k0t = (block % tiles_x) * rows, n0 = (block / tiles_x) * kDwCols;
    const uint64_t tile_floats = static_cast<uint64_t>(rows) * kDwCols;
    // weight row of slab row sr: tile row (rows / 4) * wave + q  ->  weight row 4 q + wave
    auto weight_row = [&](uint32_t sr) { return k0t + 4u * (32u * mi + 16u * h + sr) + wave; };

    // ---- gradient: this lane's 8 pieces of the slab from every split, summed in split order ----------
    f32x4 gp[8];
    const float *all = a.partials + static_cast<uint64_t>(block) * a.nsplit * tile_floats;
    for (uint32_t sp = 0; sp < a.nsplit; ++sp) {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(all + sp * tile_floats);
#pragma unroll
        for (int gj = 0; gj < 8; ++gj) {                     // gj = 4 g' + j: slab row 8 g' + 4 f_half + j
            const uint32_t v = 8u * h + gj;
            const f32x4 t = __builtin_nontemporal_load(src + ((mi * 16u + v) * 256u + wave * 64u + lane));
            gp[gj] = (sp == 0) ? t : gp[gj] + t;
        }
    }
    // to the lane-owns-32-elements layout: piece (slab row sr, quarter-row index f_row) is piece q = 32 sr + f_row
    float rg[32], rm[32], rv[32];
    {
        f32x4 *l4 = reinterpret_cast<f32x4 *>(lds);
#pragma unroll
        for (int gj = 0; gj < 8; ++gj) {
            const uint32_t sr = 8u * (gj >> 2) + 4u * f_half + (gj & 3);
            const uint32_t q = 32u * sr + f_row;
            l4[piece_slot_flat(q >> 6, q & 63u)] = gp[gj];
        }
        lds_fence();
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const f32x4 t = l4[piece_slot_own(k, lane)];
            rg[4 * k + 0] = t.x; rg[4 * k + 1] = t.y; rg[4 * k + 2] = t.z; rg[4 * k + 3] = t.w;
        }
        lds_fence();
    }
    // ---- codes and optimizer state of the slab, piece by piece through the rows ------------------------
    const uint32_t row_dwords = 4u * B;                      // 128 elements of B bits
    auto row_codes = [&](uint32_t sr) {
        return a.codes + (static_cast<uint64_t>(weight_row(sr)) * a.N + n0) / 32u * B;
    };
    u32x4 cq[CodePieces<B>::rounds];
#pragma unroll
    for (int j = 0; j < CodePieces<B>::rounds; ++j) {
        const uint32_t q = j * 64u + lane;
        if (CodePieces<B>::in_tile(j, q)) cq[j] = reinterpret_cast<const u32x4 *>(row_codes(q / B))[q % B];
        else cq[j] = u32x4{0u, 0u, 0u, 0u};
    }
    (void)row_dwords;
    auto row_f32 = [&](float *base, uint32_t sr) { return base + static_cast<uint64_t>(weight_row(sr)) * a.N + n0; };
    f32x4 mq[8], vq[8];
    if (MODE >= kStepMomentum) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t q = j * 64u + lane;
            mq[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(row_f32(a.st0, q >> 5)) + (q & 31u));
        }
    }
    if (MODE == kStepAdam) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t q = j * 64u + lane;
            vq[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(row_f32(a.st1, q >> 5)) + (q & 31u));
        }
    }
    uint32_t w[B];
    code_pieces_to_lanes<B>(cq, w, lds, lane);
    if (MODE >= kStepMomentum) pieces_to_lanes(mq, rm, lds, lane);
    if (MODE == kStepAdam) pieces_to_lanes(vq, rv, lds, lane);

    // ---- the cycle: decode, transform, update, round, pack, sums of the fit ----------------------------
    TileArgs ta{};
    ta.s = to_scalar_regs(a.sb[0]);
    ta.b = to_scalar_regs(a.sb[1]);
    FitAcc fit;
    fit.clear();
    uint32_t o[B];
    if (a.dW_out) {                                          // the gradient as consumed, before rg is reused
        f32x4 og[8];
        lanes_to_pieces(rg, og, lds, lane);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t q = j * 64u + lane;
            __builtin_nontemporal_store(og[j], reinterpret_cast<f32x4 *>(row_f32(a.dW_out, q >> 5)) + (q & 31u));
        }
    }
    cycle_generic<B, MODE, WIDE, EXACT>(ta, a.fp, a.oc, w, rg, rm, rv, o, fit);

    // ---- back out -----------------------------------------------------------------------------------------
    if (MODE >= kStepMomentum) {
        f32x4 out[8];
        lanes_to_pieces(rm, out, lds, lane);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t q = j * 64u + lane;
            __builtin_nontemporal_store(out[j], reinterpret_cast<f32x4 *>(row_f32(a.st0, q >> 5)) + (q & 31u));
        }
    }
    if (MODE == kStepAdam) {
        f32x4 out[8];
        lanes_to_pieces(rv, out, lds, lane);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t q = j * 64u + lane;
            __builtin_nontemporal_store(out[j], reinterpret_cast<f32x4 *>(row_f32(a.st1, q >> 5)) + (q & 31u));
        }
    }
    u32x4 cout[CodePieces<B>::rounds];
    lanes_to_code_pieces<B>(o, cout, lds, lane);
#pragma unroll
    for (int j = 0; j < CodePieces<B>::rounds; ++j) {
        const uint32_t q = j * 64u + lane;
        if (CodePieces<B>::in_tile(j, q)) reinterpret_cast<u32x4 *>(row_codes(q / B))[q % B] = cout[j];
    }
    fit.template reduce_and_store<EXACT>(a.ws + blockIdx.x);
}

// variant: FmtParams::variant (0 / 1 rounding by add-subtract / ldexp; 4 / 5 the same with error-carrying sums,
// which only code widths of 18 bits and more can ask for)
template <int BITS, int MODE>
inline void launch_dw_generic_variant(uint32_t variant, dim3 grid, const DwArgs &a, uint32_t tiles_x, uint32_t rows,
                                      hipStream_t st) {
    if constexpr (BITS >= 18) {
        if (variant == 4) { dw_reduce_update_generic_kernel<BITS, MODE, false, true><<<grid, dim3(64), 0, st>>>(a, tiles_x, rows); return; }
        if (variant == 5) { dw_reduce_update_generic_kernel<BITS, MODE, true, true><<<grid, dim3(64), 0, st>>>(a, tiles_x, rows); return; }
    }
    if (variant == 1) dw_reduce_update_generic_kernel<BITS, MODE, (BITS >= 9)><<<grid, dim3(64), 0, st>>>(a, tiles_x, rows);
    else dw_reduce_update_generic_kernel<BITS, MODE, false><<<grid, dim3(64), 0, st>>>(a, tiles_x, rows);
}

template <int MODE>
inline int launch_dw_generic_mode(uint32_t bits, uint32_t variant, uint32_t rows, const DwArgs &a, uint32_t tiles,
                                  uint32_t tiles_x, hipStream_t st) {
    const dim3 grid(tiles * 4u * (rows / 128u) * 2u);        // one wave per slab of 16 rows
    switch (bits) {
#define X(BITS)                                                                  \
    case BITS:                                                                   \
        launch_dw_generic_variant<BITS, MODE>(variant, grid, a, tiles_x, rows, st); \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

}  // namespace omc
