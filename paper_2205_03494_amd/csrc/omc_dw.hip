// omc_dw_update_recompress: the backward pass of a linear layer on a compressed weight matrix
// (paper Sec. 2.1, backward propagation: decompress the layer's parameters, apply the gradients,
// compress, discard).  The weight gradient dW = X^T dY is formed on the matrix cores and consumed in
// the epilogue of the same kernel: the tile's codes are read, decoded and transformed (Sec. 2.2,
// 2.3), updated with the accumulators as gradient, rounded and written back, and the sums of the fit
// are taken on the way.  With an 8-bit format and enough tiles for the chip the fp32 gradient never exists
// in memory (unless the caller asks for a copy); on the other routes -- contraction split between
// workgroups, code widths other than 8, the 16-wave kernel -- the accumulators pass through the workspace
// once and a second kernel consumes them.
//
// Tiling.  Workgroup = 4 waves, tile of W = 256 rows (k) x 128 columns (n), contraction over the M rows of
// X and dY in steps of 32.  Both operands are contraction-strided in memory, so threads load 4 x 4
// patches (four rows of 8 bytes), transpose them in registers and store 8-byte runs of four
// consecutive m to LDS, laid out as in the forward GEMM: [m-chunk of 8][row or column][16 bytes].
// Tile row r = 64 i + q stands for weight row 4 q + i, so that the stores of neighbouring threads are
// neighbours in LDS (the order of the rows of a tile is free); tile column slot 32 i + q stands for
// column 4 q + i, so that a lane ends up with four adjacent columns of a row: one dword of 8-bit codes.
#include "omc_dw_args.h"

namespace omc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kDwBChunk = kDwCols * 16;

__device__ __forceinline__ uint32_t dw_a_slot(uint32_t row, uint32_t chunk) { return row ^ (2u * chunk); }

// column i of a 4 x 4 patch of bf16 (rows = consecutive m): the four values as 8 bytes
__device__ __forceinline__ u32x2 patch_column(const u32x2 (&rows)[4], int i) {
    const int d = i >> 1;
    const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
    u32x2 out;
    out[0] = __builtin_amdgcn_perm(rows[1][d], rows[0][d], sel);
    out[1] = __builtin_amdgcn_perm(rows[3][d], rows[2][d], sel);
    return out;
}

// ROWS = weight rows per tile (256 or 128); a wave owns ROWS / 4 tile rows = MI 32-row MFMA tiles.
template <int ROWS, int MODE, bool WIDE>
__device__ __forceinline__ void dw_epilogue(const DwArgs &a, const f32x16 (&acc)[ROWS / 128][4], uint32_t k0t, uint32_t n0,
                                            uint32_t lane, uint32_t wave, FitAcc &fit) {
    constexpr int MI = ROWS / 128;
    const uint32_t f_row = lane & 31u, f_half = lane >> 5;
    const float s = a.sb ? to_scalar_regs(a.sb[0]) : 1.0f;
    const float b = a.sb ? to_scalar_regs(a.sb[1]) : 0.0f;
    const FmtParams fp = a.fp;
    bool seeded = false;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            // four weight rows at a time: their code dwords (and state) are fetched together
            uint32_t cw[4];
            f32x4 m4[4], v4[4];
            uint64_t e[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t q = 32 * mi + 8 * g + 4 * f_half + j;      // tile row (ROWS / 4) wave + q  ->  weight row 4 q + wave
                const uint32_t k = k0t + 4 * q + wave;
                e[j] = static_cast<uint64_t>(k) * a.N + n0 + 4 * f_row;
                cw[j] = a.codes[e[j] >> 2];
                if (MODE >= kStepMomentum) m4[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.st0 + e[j]));
                if (MODE == kStepAdam) v4[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.st1 + e[j]));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int v = 4 * g + j;
                pin(cw[j]);
                uint32_t out = 0;
                f32x4 grad;
#pragma unroll
                for (int ni = 0; ni < 4; ++ni) {
                    const float gr = acc[mi][ni][v];
                    grad[ni] = gr;
                    const float vt = decode_top(cw[j] << (24 - 8 * ni), fp);
                    const float sv = s * vt;
                    float x = sv + b;
                    float mm = MODE >= kStepMomentum ? m4[j][ni] : 0.0f, vv = MODE == kStepAdam ? v4[j][ni] : 0.0f;
                    x = apply_update<MODE>(x, gr, mm, vv, a.oc);
                    if (MODE >= kStepMomentum) m4[j][ni] = mm;
                    if (MODE == kStepAdam) v4[j][ni] = vv;
                    uint32_t code;
                    float tq;
                    encode<WIDE>(x, fp, code, tq);
                    if (!seeded) { fit.seed(tq); seeded = true; }
                    fit.add(x, tq);
                    out |= code << (8 * ni);
                }
                // keep the rows in program order: without this the compiler hoists the arithmetic of all
                // 128 elements above the serial fp64 accumulation and runs out of registers
                pin(fit.sV); pin(fit.sT); pin(fit.sVT); pin(fit.sTT); pin(fit.diff); pin(out);
                a.codes[e[j] >> 2] = out;
                if (MODE >= kStepMomentum) __builtin_nontemporal_store(m4[j], reinterpret_cast<f32x4 *>(a.st0 + e[j]));
                if (MODE == kStepAdam) __builtin_nontemporal_store(v4[j], reinterpret_cast<f32x4 *>(a.st1 + e[j]));
                if (a.dW_out) __builtin_nontemporal_store(grad, reinterpret_cast<f32x4 *>(a.dW_out + e[j]));
            }
        }
    }
}

// A wave's share of a finished tile: the epilogue and the wave's partial sums of the fit.
template <int ROWS, int MODE>
__device__ __forceinline__ void dw_finish_wave(const DwArgs &a, const f32x16 (&acc)[ROWS / 128][4], uint32_t k0t,
                                               uint32_t n0, uint32_t lane, uint32_t wave, uint32_t block) {
    FitAcc fit;
    fit.clear();
    if (a.fp.wide) dw_epilogue<ROWS, MODE, true>(a, acc, k0t, n0, lane, wave, fit);
    else dw_epilogue<ROWS, MODE, false>(a, acc, k0t, n0, lane, wave, fit);
    // the butterfly leaves the wave's totals in every lane; lane 0 stores them
    Partial *slot = a.ws + 4 * static_cast<uint64_t>(block) + wave;
    float tmin, tmax;
    fit.lane_range(tmin, tmax);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        fit.sV += __shfl_xor(fit.sV, off);
        fit.sT += __shfl_xor(fit.sT, off);
        fit.sVT += __shfl_xor(fit.sVT, off);
        fit.sTT += __shfl_xor(fit.sTT, off);
        tmin = fminf(tmin, __shfl_xor(tmin, off));
        tmax = fmaxf(tmax, __shfl_xor(tmax, off));
    }
    if (lane == 0) {
        Partial p;
        p.sV = fit.sV; p.sT = fit.sT; p.sVT = fit.sVT; p.sTT = fit.sTT;
        p.lV = p.lT = p.lVT = p.lTT = 0.0;               // 8-bit formats: plain fp64 sums
        p.tmin = tmin; p.tmax = tmax; p.pad[0] = p.pad[1] = 0;
        *slot = p;
    }
}

template <int ROWS, int MODE>
__global__ __launch_bounds__(256, ROWS == 256 ? 2 : 3) void dw_update_kernel(DwArgs a) {
    constexpr int MI = ROWS / 128;                        // 32-row MFMA tiles per wave
    constexpr int XP = ROWS / 128;                        // 4 x 4 patches of X per thread and step
    constexpr int QN = ROWS / 4;                          // groups of four weight rows in a tile
    constexpr int kDwAChunk = ROWS * 16;
    constexpr int kDwStageBytes = 4 * kDwAChunk + 4 * kDwBChunk;
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * kDwStageBytes];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t k0t = blockIdx.x * ROWS, n0 = blockIdx.y * kDwCols;
    const uint32_t K = a.K, N = a.N;

    // ---- roles in the loads: X patches (k group kq of 4 columns, m group mg of 4 rows; neighbouring threads
    // take the two halves of an m-chunk, so that their 8-byte LDS stores are adjacent), one dY patch
    struct Regs {
        u32x2 x[XP][4];
        u32x2 y[4];
    };
    Regs r;
    const uint32_t y_nq = tid & 31u, y_mg = tid >> 5;
    auto load_stage = [&](uint32_t m0) {
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const uint32_t idx = tid + 256 * p, kq = (idx >> 1) % QN, mg = 2 * ((idx >> 1) / QN) + (idx & 1u);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
                r.x[p][rr] = *reinterpret_cast<const u32x2 *>(a.X + static_cast<uint64_t>(m0 + 4 * mg + rr) * K + k0t + 4 * kq);
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            r.y[rr] = *reinterpret_cast<const u32x2 *>(a.dY + static_cast<uint64_t>(m0 + 4 * y_mg + rr) * N + n0 + 4 * y_nq);
    };
    auto store_stage = [&](uint8_t *ldsA) {
        uint8_t *ldsB = ldsA + 4 * kDwAChunk;
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const uint32_t idx = tid + 256 * p, kq = (idx >> 1) % QN, mg = 2 * ((idx >> 1) / QN) + (idx & 1u);
            const uint32_t chunk = mg >> 1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t row = QN * i + kq;
                *reinterpret_cast<u32x2 *>(ldsA + chunk * kDwAChunk + (dw_a_slot(row, chunk) << 4) + 8u * (mg & 1u)) =
                    patch_column(r.x[p], i);
            }
        }
        const uint32_t chunk = y_mg >> 1;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<u32x2 *>(ldsB + chunk * kDwBChunk + ((32u * i + y_nq) << 4) + 8u * (y_mg & 1u)) =
                patch_column(r.y, i);
    };

    f32x16 acc[MI][4];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const uint32_t f_row = lane & 31u, f_half = lane >> 5;
    auto multiply_stage = [&](const uint8_t *ldsA) {
        const uint8_t *ldsB = ldsA + 4 * kDwAChunk;
        bf16x8 fa[2][MI], fb[2][4];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const uint32_t chunk = 2 * ks + f_half;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const uint32_t row = QN * wave + 32 * mi + f_row;
                fa[ks][mi] = *reinterpret_cast<const bf16x8 *>(ldsA + chunk * kDwAChunk + (dw_a_slot(row, chunk) << 4));
            }
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                fb[ks][ni] = *reinterpret_cast<const bf16x8 *>(ldsB + chunk * kDwBChunk + ((32u * ni + f_row) << 4));
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][mi], fb[ks][ni], acc[mi][ni], 0, 0, 0);
    };

    // the loads of step ms + 2 are issued right after the barrier that ends round ms
    // this workgroup's share of the contraction: rows [m_begin, m_begin + nm * 32) of X and dY
    const uint32_t nm = a.M / kDwStep / a.nsplit;
    const uint32_t m_begin = blockIdx.z * nm * kDwStep;
    load_stage(m_begin);
    store_stage(lds);
    __syncthreads();
    if (nm > 1) load_stage(m_begin + kDwStep);
    uint32_t ms = 0;
    for (; ms + 2 < nm; ++ms) {
        const uint32_t cur = (ms & 1u) * kDwStageBytes;
        multiply_stage(lds + cur);
        store_stage(lds + (kDwStageBytes - cur));
        __syncthreads();
        load_stage(m_begin + (ms + 2) * kDwStep);
    }
    for (; ms < nm; ++ms) {
        const uint32_t cur = (ms & 1u) * kDwStageBytes;
        multiply_stage(lds + cur);
        if (ms + 1 < nm) {
            store_stage(lds + (kDwStageBytes - cur));
            __syncthreads();
        }
    }

    const uint32_t block = blockIdx.y * gridDim.x + blockIdx.x;     // tile index
    // ---- park the accumulators (accumulator layout, 16 bytes per lane and row): several splits of the
    // contraction, or a code width other than 8; the slab kernels add them up in split order and do the rest
    if (a.park) {
        constexpr uint32_t kTileFloats = ROWS * kDwCols;
        float *mine = a.partials + (static_cast<uint64_t>(block) * a.nsplit + blockIdx.z) * kTileFloats;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                __builtin_nontemporal_store(f32x4{acc[mi][0][v], acc[mi][1][v], acc[mi][2][v], acc[mi][3][v]},
                                            reinterpret_cast<f32x4 *>(mine) + ((mi * 16 + v) * 256 + tid));
        return;
    }

    dw_finish_wave<ROWS, MODE>(a, acc, k0t, n0, lane, wave, block);
}

// ---- wave-specialised variant (at most one tile per compute unit, long contraction) ---------------
// 16 waves: waves 0-7 only multiply (64 x 64 of the tile each), waves 8-15 only stage: each thread of
// them brings in one 4 x 4 patch of X per step, the threads of waves 12-15 also one patch of dY.  Three LDS
// stages; stage j is complete at barrier j, its fragments are read during round j + 1 and multiplied
// during round j + 2; global loads run three steps ahead.  Tile columns sit in LDS so that a multiplying
// wave's 64 columns are consecutive slots (column 64 h + 2 q + i at slot 64 h + 32 i + q).  The accumulators
// are always parked, in the layout of the four-wave kernel, and the slab kernels do the update.
constexpr int kDwWsStages = 3;
constexpr int kDwWsStageBytes = 4 * 256 * 16 + 4 * kDwBChunk;

__global__ __launch_bounds__(1024, 1) void dw_update_ws_kernel(DwArgs a) {
    constexpr int kDwAChunk = 256 * 16;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kDwWsStages * kDwWsStageBytes];
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t k0t = blockIdx.x * 256, n0 = blockIdx.y * kDwCols;
    const uint32_t K = a.K, N = a.N;
    const uint32_t nm = a.M / kDwStep / a.nsplit;           // this workgroup's share of the contraction, in steps
    const uint32_t m_begin = blockIdx.z * nm * kDwStep;

    if (wave < 8) {
        const uint32_t wm = wave >> 1, wh = wave & 1u;
        const uint32_t f_row = lane & 31u, f_half = lane >> 5;
        f32x16 acc[2][2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
        struct Frags {
            bf16x8 a[2], b[2];
        };
        auto read_frags = [&](const uint8_t *st, int ks, Frags &f) {
            const uint32_t chunk = 2 * ks + f_half;
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const uint32_t row = 64 * wm + 32 * mi + f_row;
                f.a[mi] = *reinterpret_cast<const bf16x8 *>(st + chunk * kDwAChunk + (dw_a_slot(row, chunk) << 4));
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                f.b[ni] = *reinterpret_cast<const bf16x8 *>(st + 4 * kDwAChunk + chunk * kDwBChunk +
                                                            ((64u * wh + 32u * ni + f_row) << 4));
        };
        auto multiply_frags = [&](const Frags &f) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mi], f.b[ni], acc[mi][ni], 0, 0, 0);
        };
        Frags f0, f1;
        __syncthreads();                                    // barrier 0: stage 0 is complete
        read_frags(lds, 0, f0);
        read_frags(lds, 1, f1);
        __syncthreads();                                    // barrier 1
        uint32_t nxt = kDwWsStageBytes;                     // LDS offset of stage j - 1
        for (uint32_t j = 2; j < nm + 2; ++j) {
            const bool more = j - 1 < nm;
            multiply_frags(f0);
            if (more) read_frags(lds + nxt, 0, f0);
            multiply_frags(f1);
            if (more) read_frags(lds + nxt, 1, f1);
            nxt = (nxt == (kDwWsStages - 1) * kDwWsStageBytes) ? 0u : nxt + kDwWsStageBytes;
            __syncthreads();                                // barrier j
        }
        // park: element (tile row, column c) goes where the four-wave kernel's lane (row's wave, c / 4) puts it
        const uint32_t block = blockIdx.y * gridDim.x + blockIdx.x;
        constexpr uint32_t kTileFloats = 256 * kDwCols;
        float *mine = a.partials + (static_cast<uint64_t>(block) * a.nsplit + blockIdx.z) * kTileFloats;
        const uint32_t owner = 64 * wm + 32 * f_half + 16 * wh + (f_row >> 1);
        const uint32_t sub = 2 * (f_row & 1u);
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                __builtin_nontemporal_store(f32x2{acc[mi][0][v], acc[mi][1][v]},
                                            reinterpret_cast<f32x2 *>(mine + (static_cast<uint32_t>(mi * 16 + v) * 256 + owner) * 4 + sub));
        return;
    }

    // ---- staging waves ---------------------------------------------------------------------------------
    const uint32_t pt = tid - 512u;
    const bool does_y = wave >= 12;
    const uint32_t x_kq = (pt >> 1) & 63u, x_mg = 2 * (pt >> 7) + (pt & 1u);
    const uint32_t wt = tid & 255u;
    const uint32_t y_nq = wt & 31u, y_mg = wt >> 5;
    struct Regs {
        u32x2 x[4], y[4];
    };
    Regs r[kDwWsStages];
    auto load_stage = [&](Regs &g, uint32_t m0) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            g.x[rr] = *reinterpret_cast<const u32x2 *>(a.X + static_cast<uint64_t>(m0 + 4 * x_mg + rr) * K + k0t + 4 * x_kq);
        if (!does_y) return;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            g.y[rr] = *reinterpret_cast<const u32x2 *>(a.dY + static_cast<uint64_t>(m0 + 4 * y_mg + rr) * N + n0 + 4 * y_nq);
    };
    auto store_stage = [&](const Regs &g, uint8_t *st) {
        const uint32_t xc = x_mg >> 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t row = 64 * i + x_kq;
            *reinterpret_cast<u32x2 *>(st + xc * kDwAChunk + (dw_a_slot(row, xc) << 4) + 8u * (x_mg & 1u)) = patch_column(g.x, i);
        }
        if (!does_y) return;
        const uint32_t yc = y_mg >> 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t c = 4 * y_nq + i;
            const uint32_t slot = (c & 64u) + 32u * (c & 1u) + ((c & 63u) >> 1);
            *reinterpret_cast<u32x2 *>(st + 4 * kDwAChunk + yc * kDwBChunk + (slot << 4) + 8u * (y_mg & 1u)) = patch_column(g.y, i);
        }
    };
#pragma unroll
    for (int u = 0; u < kDwWsStages; ++u)
        if (static_cast<uint32_t>(u) < nm) load_stage(r[u], m_begin + u * kDwStep);
    uint32_t j = 0;
    for (; j + kDwWsStages <= nm; j += kDwWsStages) {
#pragma unroll
        for (int u = 0; u < kDwWsStages; ++u) {
            store_stage(r[u], lds + u * kDwWsStageBytes);
            if (j + u + kDwWsStages < nm) load_stage(r[u], m_begin + (j + u + kDwWsStages) * kDwStep);
            __syncthreads();                                // barrier j + u
        }
    }
#pragma unroll
    for (int u = 0; u < kDwWsStages - 1; ++u)
        if (j + u < nm) {
            store_stage(r[u], lds + u * kDwWsStageBytes);
            __syncthreads();
        }
    __syncthreads();                                        // barriers nm and nm + 1: the multiplying waves drain
    __syncthreads();
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void dw_finalize_kernel(const Partial *__restrict__ ws, uint32_t nparts, uint64_t n,
                                                              int use_pvt, int exact, float *__restrict__ sb) {
    __shared__ double red[NW * 10];
    finalize_variable<NW>(ws, nparts, nullptr, n, use_pvt != 0, exact != 0, sb, red);
}

// one Partial per 16-row x 128-column slab (the finest grain any of the update kernels uses)
static size_t dw_fit_bytes(uint32_t N, uint32_t K) {
    return (static_cast<size_t>(K) * N / kTileElems * sizeof(Partial) + 255) / 256 * 256;
}

// Tile height and number of contraction splits for a problem size: 256-row tiles and no split when
// that already gives two workgroups per compute unit; otherwise split the M rows (each split at least
// 512 rows, at most 8 splits) and, if that is still not enough, take 128-row tiles.
DwConfig dw_config(uint32_t M, uint32_t N, uint32_t K) {
    DwConfig c{256, 1, 0};
    const uint64_t tiles256 = static_cast<uint64_t>(K / 256) * (N / kDwCols);
    // At most one workgroup per compute unit with at least 2048 rows of the contraction each, and at least
    // half of the compute units busy: the wave-specialised kernel.
    if (K % 256 == 0 && tiles256 <= 256) {
        uint32_t sp = 1;
        while (tiles256 * (2 * sp) <= 256 && sp < 8 && M % (2 * sp * kDwStep) == 0 && M / (2 * sp) >= 2048) sp *= 2;
        if (M / sp >= 2048 && tiles256 * sp >= 128) return DwConfig{256, sp, 1};
    }
    auto splits_for = [&](uint64_t tiles) {
        uint32_t sp = 1;
        while (tiles * sp < 512 && sp < 8 && M % (2 * sp * kDwStep) == 0 && M / (2 * sp) >= 512) sp *= 2;
        return sp;
    };
    c.nsplit = splits_for(tiles256);
    if (tiles256 * c.nsplit < 512) {
        c.rows = 128;
        c.nsplit = splits_for(2 * tiles256);
    }
    return c;
}

int launch_dw_update(const uint16_t *X, const uint16_t *dY, void *codes, const FmtParams &fp, float *sb, int use_pvt,
                     float *state0, float *state1, const omc_opt &opt, float *dW_out, uint32_t M, uint32_t N,
                     uint32_t K, void *ws, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const DwConfig cfg = dw_config(M, N, K);
    const uint32_t tiles = (K / cfg.rows) * (N / kDwCols);
    // workspace: the fit's partials (one per 16-row slab at most) | parked accumulators
    uint8_t *w8 = static_cast<uint8_t *>(ws);
    const size_t fit_bytes = dw_fit_bytes(N, K);
    const bool byte_codes = fp.bits == 8;
    DwArgs a{};
    a.X = X;
    a.dY = dY;
    a.codes = static_cast<uint32_t *>(codes);
    a.sb = sb;
    a.st0 = opt.kind >= OMC_MOMENTUM ? state0 : nullptr;
    a.st1 = opt.kind == OMC_ADAM ? state1 : nullptr;
    a.dW_out = dW_out;
    a.ws = reinterpret_cast<Partial *>(w8);
    a.partials = reinterpret_cast<float *>(w8 + fit_bytes);
    a.park = (cfg.nsplit > 1 || !byte_codes || cfg.ws) ? 1u : 0u;
    a.nsplit = cfg.nsplit;
    a.fp = fp;
    a.oc = OptConst{opt.lr, opt.momentum, opt.beta1, opt.beta2, opt.eps, opt.one_minus_beta1,
                    opt.one_minus_beta2, opt.bias_corr1, opt.bias_corr2};
    a.M = M;
    a.N = N;
    a.K = K;
    const dim3 grid(K / cfg.rows, N / kDwCols, cfg.nsplit);
#define OMC_DW_LAUNCH(ROWS)                                                                      \
    do {                                                                                         \
        if (opt.kind == OMC_SGD) dw_update_kernel<ROWS, kStepSgd><<<grid, dim3(256), 0, st>>>(a); \
        else if (opt.kind == OMC_MOMENTUM) dw_update_kernel<ROWS, kStepMomentum><<<grid, dim3(256), 0, st>>>(a); \
        else dw_update_kernel<ROWS, kStepAdam><<<grid, dim3(256), 0, st>>>(a);                    \
    } while (0)
    if (cfg.ws) dw_update_ws_kernel<<<grid, dim3(1024), 0, st>>>(a);
    else if (cfg.rows == 128) OMC_DW_LAUNCH(128);
    else OMC_DW_LAUNCH(256);
#undef OMC_DW_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return static_cast<int>(e);
    uint32_t nparts = 4u * tiles;
    if (a.park) {                                          // the slab kernels do the update, whatever the code width
        const uint32_t tx = K / cfg.rows;
        int rc;
        if (opt.kind == OMC_SGD) rc = launch_dw_generic_sgd(fp.bits, fp.variant == 2 || fp.variant == 3 ? 0u : fp.variant, cfg.rows, a, tiles, tx, st);
        else if (opt.kind == OMC_MOMENTUM) rc = launch_dw_generic_momentum(fp.bits, fp.variant == 2 || fp.variant == 3 ? 0u : fp.variant, cfg.rows, a, tiles, tx, st);
        else rc = launch_dw_generic_adam(fp.bits, fp.variant == 2 || fp.variant == 3 ? 0u : fp.variant, cfg.rows, a, tiles, tx, st);
        if (rc != 0) return rc;
        nparts = static_cast<uint32_t>(static_cast<uint64_t>(K) * N / kTileElems);
    }
    const uint64_t n = static_cast<uint64_t>(K) * N;
    // the width of the reduction depends on the sizes alone, so results do not depend on the run
    const int exact = variant_exact(fp.variant) ? 1 : 0;
    if (nparts <= 256) dw_finalize_kernel<1><<<dim3(1), dim3(64), 0, st>>>(a.ws, nparts, n, use_pvt, exact, sb);
    else if (nparts <= 2048) dw_finalize_kernel<4><<<dim3(1), dim3(256), 0, st>>>(a.ws, nparts, n, use_pvt, exact, sb);
    else dw_finalize_kernel<16><<<dim3(1), dim3(1024), 0, st>>>(a.ws, nparts, n, use_pvt, exact, sb);
    return static_cast<int>(hipGetLastError());
}

size_t dw_workspace_bytes(uint32_t bits, uint32_t M, uint32_t N, uint32_t K) {
    const DwConfig cfg = dw_config(M, N, K);
    const bool park = cfg.nsplit > 1 || bits != 8 || cfg.ws;
    const size_t partial_bytes = park ? static_cast<size_t>(cfg.nsplit) * K * N * sizeof(float) : 0;
    return dw_fit_bytes(N, K) + partial_bytes;
}

}  // namespace omc
