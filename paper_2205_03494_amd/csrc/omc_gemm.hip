// omc_dequant_gemm: C = A * decompress(W) with the weights expanded on chip (paper Sec. 2.1,
// forward path: the layer's parameters are decompressed on the fly and consumed at once).
//
// The affine per-variable transformation (Sec. 2.3) factors out of the contraction:
//     A (s Vt + b 1 1^T) = s (A Vt) + b rowsum(A) 1^T,
// and every code value Vt of a format with at most 7 mantissa bits is exactly a bfloat16, so the
// matrix cores run on exact images of the codes: bf16 x bf16 MFMA with fp32 accumulation.
//
// Tiling.  Workgroup = 4 waves, output tile 256 (M) x 128 (N), K step 32.  Wave w owns rows
// [64 w, 64 w + 64) and all 128 columns: 2 x 4 MFMA tiles of 32x32 (v_mfma_f32_32x32x16_bf16),
// 128 accumulator registers.  Both operands sit in LDS as [k-chunk of 8][row or column][16 bytes],
// which is what one lane of the MFMA consumes, so fragment reads are 16-byte, contiguous across
// lanes and free of bank conflicts.
//   A: global 16-byte pieces -> LDS, rows XOR-swizzled by the chunk so that the stores do not collide.
//   W: each thread takes a 4 (k) x 4 (n) patch of codes, decodes the 16 values in registers
//      (same bit-domain decode as the streaming kernels, fp32 -> top 16 bits, exact) and stores the
//      four k-values of each column as 8 bytes.  Column c = 4 cg + i is kept at slot 32 i + cg, so
//      that MFMA tile i covers the columns == i (mod 4): the stores of 16 neighbouring lanes then
//      fill 128 contiguous bytes, and in the epilogue a lane holds four adjacent columns of C,
//      one 16-byte store per row.
//      (S1E4M3 with bias 7: the hardware FP8 conversion decodes, after a pre-pass has excluded the one
//      code it reads differently.)
// The K loop is double-buffered in LDS: while the matrix cores work on one K step, the codes of the
// next one are decoded and stored into the other buffer; the global loads of the step after that are
// issued right after the barrier that ends a round (the 128-row variant, used when 256-row tiles
// would leave compute units idle, keeps two register sets and loads two steps ahead); one workgroup
// barrier per K step.  The row sums of A are taken inside the kernel from the staged pieces.
// omc_dequant_gemm_dx (dX = dY * Wbar^T) is the same kernel with the codes read along the other
// direction (TRANS): 16 consecutive codes of a weight row per thread, decoded into two k-chunks.
// A second kernel serves grids of at most one tile per compute unit with a long contraction: 16 waves per
// workgroup, eight that only multiply, four that only stage A and four that only stage W (see there).
#include <hip/hip_runtime.h>
#include "omc_internal.h"

#pragma clang fp contract(off)

namespace omc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#ifndef OMC_GEMM_WAVES
#define OMC_GEMM_WAVES 2
#endif
// LDS slot of an A row within its k-chunk plane: XOR with the chunk keeps the four planes' stores of
// one wave apart (measured against no swizzle and a rotation by 4 * chunk: both slower)
#define OMC_A_SLOT(row, chunk) ((row) ^ (2u * (chunk)))

constexpr int kBN = 128, kBK = 32;
constexpr int kWChunkBytes = kBN * 16;   // one k-chunk (8 bf16) of all columns

constexpr uint32_t kScanBlocks = 64;      // one flag word each; a GEMM wave reads them all with one load

// Pre-pass (S1E4M3 with bias 7 only): scan the codes for the top code, the one code whose value
// differs from the hardware FP8 conversion's (480 here, NaN there); flags[j] != 0 sends the GEMM to the
// generic decode.
__global__ __launch_bounds__(256) void gemm_scan_kernel(const uint32_t *__restrict__ codes, uint64_t code_dwords,
                                                        uint32_t *__restrict__ flags) {
    __shared__ uint32_t any_top[4];
    const uint32_t j = blockIdx.x;
    const uint64_t pieces = code_dwords / 4;                          // 16-byte pieces (streams are padded to 16 bytes)
    const uint64_t per = (pieces + kScanBlocks - 1) / kScanBlocks;
    const uint64_t lo = j * per, hi = (lo + per < pieces) ? lo + per : pieces;
    uint32_t found = 0;
    uint64_t q = lo + threadIdx.x;
    for (; q + 7 * 256 < hi; q += 8 * 256) {                // eight loads in flight per thread
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = reinterpret_cast<const u32x4 *>(codes)[q + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) found |= ((v[u][i] & 0x7f7f7f7fu) + 0x01010101u) & 0x80808080u;
    }
    for (; q < hi; q += 256) {
        const u32x4 v = reinterpret_cast<const u32x4 *>(codes)[q];
#pragma unroll
        for (int i = 0; i < 4; ++i) found |= ((v[i] & 0x7f7f7f7fu) + 0x01010101u) & 0x80808080u;
    }
    const bool w = __any(found != 0);
    if ((threadIdx.x & 63) == 0) any_top[threadIdx.x >> 6] = w ? 1u : 0u;
    __syncthreads();
    if (threadIdx.x == 0) flags[j] = any_top[0] | any_top[1] | any_top[2] | any_top[3];
}

// fp32 value of a code given with its sign bit at bit 31 (see the streaming kernels)
__device__ __forceinline__ uint32_t decode_bits(uint32_t top, const FmtParams &fp) {
    int32_t u = static_cast<int32_t>(top) >> fp.asr;
    u &= static_cast<int32_t>(fp.keep_mask);
    return __float_as_uint(__uint_as_float(static_cast<uint32_t>(u)) * fp.dec_scale);
}

// Four consecutive codes (elements e .. e+3 of the packed stream) as bytes-at-top of four words.
template <bool BYTE>
__device__ __forceinline__ void load_codes4(const uint32_t *__restrict__ codes, uint64_t total_dwords, uint64_t e,
                                            uint32_t B, uint32_t (&raw)[3], uint32_t &off) {
    if (BYTE) {
        raw[0] = codes[e >> 2];          // e is a multiple of 4
        off = 0;
    } else {
        const uint64_t bit = e * B;
        const uint64_t dw = bit >> 5;
        off = static_cast<uint32_t>(bit & 31u);
        if (dw + 3 <= total_dwords) {                       // one 12-byte load (dword-aligned) ...
            typedef uint32_t u32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));
            const u32x3_a4 t = *reinterpret_cast<const u32x3_a4 *>(codes + dw);
            raw[0] = t[0]; raw[1] = t[1]; raw[2] = t[2];
        } else {                                            // ... except at the very end of the stream
#pragma unroll
            for (int i = 0; i < 3; ++i) raw[i] = (dw + i < total_dwords) ? codes[dw + i] : 0u;
        }
    }
}
template <bool BYTE>
__device__ __forceinline__ uint32_t code_top_of(const uint32_t (&raw)[3], uint32_t off, uint32_t B, int i) {
    if (BYTE) return raw[0] << (24 - 8 * i);
    // the 64 bits that start at the first code (two funnel shifts by the lane's offset, shared by the four
    // codes), then a shift by i * B, which is the same in every lane; 4 B <= 64 for the widths the GEMM takes
    const uint32_t n0 = __builtin_amdgcn_alignbit(raw[1], raw[0], off);
    const uint32_t n1 = __builtin_amdgcn_alignbit(raw[2], raw[1], off);
    const uint64_t n = (static_cast<uint64_t>(n1) << 32) | n0;
    const uint32_t c = static_cast<uint32_t>(n >> (i * B));
    return c << (32 - B);
}

// The fp32 bit patterns of four consecutive codes (what load_codes4 fetched).  HW: the hardware FP8 conversion.
template <bool BYTE, bool HW>
__device__ __forceinline__ void decode_codes4(const uint32_t (&raw)[3], uint32_t off, const FmtParams &fp, uint32_t (&v)[4]) {
    if (HW) {
        const f32x2 c01 = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(raw[0]), false);
        const f32x2 c23 = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(raw[0]), true);
        v[0] = __float_as_uint(c01[0]); v[1] = __float_as_uint(c01[1]);
        v[2] = __float_as_uint(c23[0]); v[3] = __float_as_uint(c23[1]);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = decode_bits(code_top_of<BYTE>(raw, off, fp.bits, i), fp);
    }
}
// four fp32 bit patterns whose low 16 bits are zero, as four bf16 in 8 bytes
__device__ __forceinline__ u32x2 pack_bf16x4(uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3) {
    u32x2 out;
    out[0] = __builtin_amdgcn_perm(v1, v0, 0x07060302u);   // bf16(v0) | bf16(v1) << 16
    out[1] = __builtin_amdgcn_perm(v3, v2, 0x07060302u);
    return out;
}

// DEC: 0 = any code width, 1 = byte codes.  HW (byte codes of S1E4M3 / bias 7 only): hardware FP8 conversion.
// TRANS: the packed variable is [N x K] (output column major), i.e. C = A * W^T for the weights as
// stored: the input-gradient GEMM of the layer whose forward pass is the non-transposed one.
template <int BM, int DEC, bool HW, bool TRANS>
__device__ __forceinline__ void dequant_gemm_body(const uint16_t *__restrict__ A, const uint32_t *__restrict__ codes,
                                                  uint64_t total_dwords, const FmtParams &fp,
                                                  const float *__restrict__ sb, float *__restrict__ C, uint32_t N,
                                                  uint32_t K, uint8_t *lds) {
    constexpr bool BYTE = DEC != 0;
    constexpr int kAChunkBytes = BM * 16;                 // one k-chunk (8 bf16) of all rows
    constexpr int kStageBytes = 4 * kAChunkBytes + 4 * kWChunkBytes;
    constexpr int MI = BM / 128;                          // 32-row MFMA tiles per wave
    constexpr int AP = BM / 64;                           // 16-byte pieces of A per thread and stage

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    // consecutive workgroups share the W column block and walk down M
    const uint32_t m0 = blockIdx.x * BM, n0 = blockIdx.y * kBN;

    // ---- roles in the loads ------------------------------------------------------------------
    // A: piece q = tid + 256 p (p < AP): row = q / 4, chunk = q % 4
    // W: patch (kg, cg): kg = 2 wave + (lane & 1), cg = lane >> 1
    const uint32_t w_h = lane & 1u, w_cg = lane >> 1;
    const uint32_t w_kg = 2 * wave + w_h;
    const uint64_t w_col = n0 + 4 * w_cg;
    // W transposed: thread = (LDS slot, half of the K step); slot 32 i + cg holds column 4 cg + i, and the
    // thread takes that column's 16 consecutive k-values (contiguous in memory) as four groups of four
    const uint32_t t_slot = tid & 127u, t_h = tid >> 7;
    const uint64_t t_row = n0 + 4 * (t_slot & 31u) + (t_slot >> 5);

    // two register sets: global loads run two K steps ahead of the matrix cores
    struct StageRegs {
        u32x4 a[AP];
        uint32_t w_raw[4][3], w_off[4];
    };
    StageRegs r0, r1;                                      // r1 only in the two-ahead loop

    auto load_a_piece = [&](StageRegs &r, uint32_t k0, int p) {
        const uint32_t q = tid + 256 * p, row = q >> 2, chunk = q & 3u;
        r.a[p] = *reinterpret_cast<const u32x4 *>(A + static_cast<uint64_t>(m0 + row) * K + k0 + 8 * chunk);
    };
    auto load_w_row = [&](StageRegs &r, uint32_t k0, int rr) {
        const uint64_t e = TRANS ? t_row * K + k0 + 16 * t_h + 4 * rr
                                 : static_cast<uint64_t>(k0 + 4 * w_kg + rr) * N + w_col;
        load_codes4<BYTE>(codes, total_dwords, e, fp.bits, r.w_raw[rr], r.w_off[rr]);
    };
    auto load_stage = [&](StageRegs &r, uint32_t k0) {
#pragma unroll
        for (int p = 0; p < AP; ++p) load_a_piece(r, k0, p);
        if (TRANS && BYTE) {                                // the thread's 16 codes are one aligned 16-byte piece
            const u32x4 t = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(codes) + t_row * K + k0 + 16 * t_h);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                r.w_raw[rr][0] = t[rr];
                r.w_off[rr] = 0;
            }
            return;
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) load_w_row(r, k0, rr);
    };

    // Row sums of A for the b * rowsum(A) term, taken on the way: every piece of A passes through
    // store_a_piece exactly once, and a thread's piece p always belongs to the same row.
    float rsum[AP];
#pragma unroll
    for (int p = 0; p < AP; ++p) rsum[p] = 0.0f;
    const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
    auto store_a_piece = [&](const StageRegs &r, uint8_t *ldsA, int p) {
        const uint32_t q = tid + 256 * p, row = q >> 2, chunk = q & 3u;
        *reinterpret_cast<u32x4 *>(ldsA + chunk * kAChunkBytes + (OMC_A_SLOT(row, chunk) << 4)) = r.a[p];
        if (sb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w = r.a[p][i];               // (a bit_cast straight from the vector element reads element 0)
                rsum[p] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, rsum[p], false);
            }
        }
    };
    // decode the thread's 16 codes (four groups of four consecutive ones) and store them as 8-byte runs of four
    // k-values: non-transposed, group = weight row and the runs are the patch's columns; transposed, group = four
    // consecutive k-values of the thread's column and is a run itself
    auto store_w = [&](const StageRegs &r, uint8_t *ldsA) {
        uint8_t *ldsW = ldsA + 4 * kAChunkBytes;
        uint32_t v[4][4];
#pragma unroll
        for (int g = 0; g < 4; ++g) decode_codes4<BYTE, HW>(r.w_raw[g], r.w_off[g], fp, v[g]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (TRANS)
                *reinterpret_cast<u32x2 *>(ldsW + (2u * t_h + (i >> 1)) * kWChunkBytes + (t_slot << 4) + 8u * (i & 1)) =
                    pack_bf16x4(v[i][0], v[i][1], v[i][2], v[i][3]);
            else
                *reinterpret_cast<u32x2 *>(ldsW + wave * kWChunkBytes + ((32u * i + w_cg) << 4) + 8u * w_h) =
                    pack_bf16x4(v[0][i], v[1][i], v[2][i], v[3][i]);
        }
    };
    auto store_stage = [&](const StageRegs &r, uint8_t *ldsA) {
#pragma unroll
        for (int p = 0; p < AP; ++p) store_a_piece(r, ldsA, p);
        store_w(r, ldsA);
    };

    f32x16 acc[MI][4];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const uint32_t f_row = lane & 31u, f_half = lane >> 5;   // fragment roles
    struct Frags {
        bf16x8 a[MI], b[4];
    };
    auto read_frags = [&](const uint8_t *ldsA, int ks, Frags &f) {
        const uint8_t *ldsW = ldsA + 4 * kAChunkBytes;
        const uint32_t chunk = 2 * ks + f_half;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const uint32_t row = 32 * MI * wave + 32 * mi + f_row;
            f.a[mi] = *reinterpret_cast<const bf16x8 *>(ldsA + chunk * kAChunkBytes + (OMC_A_SLOT(row, chunk) << 4));
        }
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
            f.b[ni] = *reinterpret_cast<const bf16x8 *>(ldsW + chunk * kWChunkBytes + ((32u * ni + f_row) << 4));
    };
    auto multiply_frags = [&](const Frags &f) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mi], f.b[ni], acc[mi][ni], 0, 0, 0);
    };
    auto multiply_stage = [&](const uint8_t *ldsA) {
        if (BYTE) {                                         // all fragments of the K step first
            Frags f0, f1;
            read_frags(ldsA, 0, f0);
            read_frags(ldsA, 1, f1);
            multiply_frags(f0);
            multiply_frags(f1);
        } else {                                            // wider codes need the registers for the raw words
            Frags f;
            read_frags(ldsA, 0, f);
            multiply_frags(f);
            read_frags(ldsA, 1, f);
            multiply_frags(f);
        }
    };
    const uint32_t nk = K / kBK;
    if constexpr (BM == 256) {
    // One register set: the loads of K step ks+2 are issued right after the barrier that ends round
    // ks and have all of round ks+1 to arrive before they are decoded and stored.
    load_stage(r0, 0);
    store_stage(r0, lds);
    __syncthreads();
    if (nk > 1) load_stage(r0, kBK);
    uint32_t ks = 0;
    for (; ks + 2 < nk; ++ks) {
        const uint32_t cur = (ks & 1u) * kStageBytes;
        multiply_stage(lds + cur);
        store_stage(r0, lds + (kStageBytes - cur));
        __syncthreads();
        load_stage(r0, (ks + 2) * kBK);
    }
    for (; ks < nk; ++ks) {
        const uint32_t cur = (ks & 1u) * kStageBytes;
        multiply_stage(lds + cur);
        if (ks + 1 < nk) {
            store_stage(r0, lds + (kStageBytes - cur));
            __syncthreads();
        }
    }
    } else {
    // The 128-row tiling (three workgroups per compute unit) does better with loads two K steps ahead
    // in two register sets.  One steady-state round as straight-line code: fragments of both halves, the matrix instructions,
    // decode + LDS stores of the next K step, barrier, global loads of the step after the next two.
    auto steady_round = [&](const uint8_t *cur, uint8_t *nxt, StageRegs &r, uint32_t k_load) {
        multiply_stage(cur);
        store_stage(r, nxt);
        __syncthreads();
        load_stage(r, k_load);
    };

    uint8_t *buf0 = lds, *buf1 = lds + kStageBytes;
    load_stage(r0, 0);
    store_stage(r0, buf0);
    __syncthreads();
    if (nk > 1) load_stage(r0, kBK);
    if (nk > 2) load_stage(r1, 2 * kBK);
    // Invariant at the top of an even round `it`: buf0 holds K step it, r0 step it+1, r1 step it+2.
    uint32_t it = 0;
    for (; it + 4 < nk; it += 2) {                          // both rounds store and load unconditionally
        steady_round(buf0, buf1, r0, (it + 3) * kBK);
        steady_round(buf1, buf0, r1, (it + 4) * kBK);
    }
    for (; it < nk; it += 2) {
        multiply_stage(buf0);
        if (it + 1 < nk) store_stage(r0, buf1);            // nobody reads buf1 any more (barrier of the round before)
        __syncthreads();
        if (it + 3 < nk) load_stage(r0, (it + 3) * kBK);
        if (it + 1 < nk) {
            multiply_stage(buf1);
            if (it + 2 < nk) store_stage(r1, buf0);
            __syncthreads();
            if (it + 4 < nk) load_stage(r1, (it + 4) * kBK);
        }
    }
    }

    // ---- epilogue: C = s * acc + b * rowsum --------------------------------------------------------
    const float s = sb ? sb[0] : 1.0f;
    const float b = sb ? sb[1] : 0.0f;
    // the four threads that hold the pieces of a row add up their parts and publish the row sum in LDS
    // (the stage buffers are free once everybody is past the last matrix instruction's fragment reads)
    float *rowsum_lds = reinterpret_cast<float *>(lds);
    if (sb) {
        __syncthreads();
#pragma unroll
        for (int p = 0; p < AP; ++p) {
            float t = rsum[p];
            t += __shfl_xor(t, 1);
            t += __shfl_xor(t, 2);
            if ((tid & 3u) == 0) rowsum_lds[(tid >> 2) + 64 * p] = t;
        }
        __syncthreads();
    }
    // a lane's accumulators cover rows in runs of four: fetch all row sums it needs in one batch
    f32x4 rs[MI][4];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t row = 32 * MI * wave + 32 * mi + 8 * g + 4 * f_half;
            rs[mi][g] = sb ? *reinterpret_cast<const f32x4 *>(rowsum_lds + row) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = m0 + 32 * MI * wave + 32 * mi + 8 * (v >> 2) + 4 * f_half + (v & 3);
            const float add = sb ? b * rs[mi][v >> 2][v & 3] : 0.0f;
            f32x4 out;
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) out[ni] = s * acc[mi][ni][v] + add;
            __builtin_nontemporal_store(out, reinterpret_cast<f32x4 *>(C + static_cast<uint64_t>(row) * N + n0 + 4 * f_row));
        }
    }
}

// ---- S1E4M3 forward kernel ---------------------------------------------------------------------------
// The forward product on hardware-convertible byte codes (S1E4M3, bias 7, no top code: see the pre-pass) takes a
// kernel of its own, built on three facts that were measured on this part.  (1) In the 4 x 1 wave layout the 64 rows
// of A that a wave multiplies belong to it alone, so staging A in LDS buys no reuse and only costs LDS bandwidth (the
// tile kernel above moves 80 KB through LDS per K step, more than the matrix instructions leave time for): here every
// lane loads its A fragments (8 consecutive k of its row, 16 bytes) straight from global memory into registers, two K
// steps ahead in three register sets.  (2) gfx950 converts two FP8 codes into a packed pair of bfloat16 in one
// instruction (v_cvt_scalef32_pk_bf16_fp8, scale 1), so a thread's 16 codes become 32 bytes of bf16 with eight
// conversions and no byte shuffles, stored row-major [k][n] as loaded.  (3) The transposing LDS read
// (ds_read_b64_tr_b16) then delivers the B fragments: within a block of 16 lanes, lane 4 q + e receives element e of
// the 8-byte chunks that lanes q, q + 4, q + 8, q + 12 point at, so four lanes pointing at four consecutive k rows of
// the same four columns hand each of 16 lanes one column's four k values.  Rows are 320 bytes apart (16 banks), which
// keeps the four rows of a read on different banks.  About 30 vector instructions per K step and wave instead of
// about 100, and 48 KB instead of 80 KB through LDS.  W of step j + 1 is decoded and stored during step j; the
// fragments of the first half of step j + 1 are read under the second half of step j; one barrier per K step.
constexpr int kF8RowBytes = kBN * 2 + 64;
constexpr int kF8WBytes = kBK * kF8RowBytes;               // 10 KB per stage, two stages

// TRANS (dX = dY * Wbar^T; the packed variable is [N x K]): the contraction runs along the codes' contiguous direction, so
// a thread's 16 codes are 16 consecutive k of one output column and need no transposition at all: they are stored as two
// 16-byte k-chunks in the [k-chunk][column][16 B] layout of the tile kernel and read back with plain 16-byte loads.
template <bool TRANS>
__device__ __forceinline__ void dequant_gemm_fp8_body(const uint16_t *__restrict__ A, const uint8_t *__restrict__ codes,
                                                      const float *__restrict__ sb, float *__restrict__ C, uint32_t N,
                                                      uint32_t K, uint8_t *sW0, uint8_t *sW1, float *rowsum_lds) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    constexpr int BM = 256;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t m0 = blockIdx.x * BM, n0 = blockIdx.y * kBN;
    const uint32_t nk = K / kBK;                              // >= 2
    const uint32_t f_row = lane & 31u, f_half = lane >> 5;

    // A: lane (row, half) takes 8 consecutive k of its row per fragment
    const uint8_t *a_base = reinterpret_cast<const uint8_t *>(A) + static_cast<uint64_t>(m0) * K * 2;
    uint32_t a_off[2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) a_off[mi] = (64 * wave + 32 * mi + f_row) * K * 2 + f_half * 16;
    struct ASet {
        u32x4 f[2][2];                                        // [half of the K step][mi]
    };
    auto load_a = [&](uint32_t step, ASet &r) {
        const uint8_t *p = a_base + step * (kBK * 2);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) r.f[ks][mi] = *reinterpret_cast<const u32x4 *>(p + a_off[mi] + 32 * ks);
    };
    // W: thread = (k row, 16 consecutive codes); TRANS: thread = (output column, which 16 of the step's 32 k)
    const uint32_t w_row = TRANS ? (tid >> 1) : (tid >> 3), w_piece = TRANS ? (tid & 1u) : (tid & 7u);
    const uint8_t *w_base = TRANS ? codes + static_cast<uint64_t>(n0) * K : codes + n0;
    const uint32_t w_off = TRANS ? w_row * K + 16 * w_piece : w_row * N + 16 * w_piece;
    auto load_w = [&](uint32_t step) {
        return *reinterpret_cast<const u32x4 *>(w_base + (TRANS ? static_cast<uint64_t>(step) * kBK
                                                                : static_cast<uint64_t>(step) * kBK * N) + w_off);
    };
    auto store_w = [&](const u32x4 &c, uint8_t *sW) {
        uint32_t o[8];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            o[2 * d] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c[d], 1.0f, false));
            o[2 * d + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c[d], 1.0f, true));
        }
        if (TRANS) {      // k-chunks 2 piece and 2 piece + 1 of column w_row; the column slot is XORed with 8 piece so that
                          // the two threads of a column, whose chunks lie 4 KB apart, hit different banks
            uint8_t *dst = sW + (2 * w_piece) * kWChunkBytes + ((w_row ^ (8u * w_piece)) << 4);
            *reinterpret_cast<u32x4 *>(dst) = u32x4{o[0], o[1], o[2], o[3]};
            *reinterpret_cast<u32x4 *>(dst + kWChunkBytes) = u32x4{o[4], o[5], o[6], o[7]};
            return;
        }
        uint8_t *dst = sW + w_row * kF8RowBytes + w_piece * 32;
        *reinterpret_cast<u32x4 *>(dst) = u32x4{o[0], o[1], o[2], o[3]};
        *reinterpret_cast<u32x4 *>(dst + 16) = u32x4{o[4], o[5], o[6], o[7]};
    };
    // transposing read: block b = lane >> 4 (b & 1: which 16 of the 32 columns, b >> 1: which 8 of the 16 k),
    // source lane L = lane & 15: L & 3 = group of four columns, L >> 2 = k row
    const uint32_t tb = lane >> 4, tL = lane & 15u;
    const uint32_t fb_base = (8 * (tb >> 1) + (tL >> 2)) * kF8RowBytes + (16 * (tb & 1u) + 4 * (tL & 3u)) * 2;
    struct BSet {
        bf16x8 b[4];
    };
    auto read_b = [&](const uint8_t *sW, int ks, BSet &f) {
        if (TRANS) {
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                f.b[ni] = *reinterpret_cast<const bf16x8 *>(sW + (2 * ks + f_half) * kWChunkBytes + (((32u * ni + f_row) ^ (8u * ks)) << 4));
            return;
        }
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            const uint8_t *p = sW + fb_base + (16 * ks) * kF8RowBytes + 64 * ni;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 4 * kF8RowBytes));
            const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            f.b[ni] = __builtin_bit_cast(bf16x8, both);
        }
    };

    f32x16 acc[2][4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    float rsum[2] = {0.0f, 0.0f};
    const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
    const bool want_rs = sb != nullptr;
    auto multiply = [&](const ASet &a, int ks, const BSet &f) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.f[ks][mi]), f.b[ni], acc[mi][ni], 0, 0, 0);
        if (want_rs) {                                       // row sums of A for the b * rowsum(A) term, on the way
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t x = a.f[ks][mi][i];
                    rsum[mi] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x), ones, rsum[mi], false);
                }
        }
    };

    ASet a0, a1, a2;
    u32x4 wq0, wq1;
    BSet f0, f1;
    load_a(0, a0); wq0 = load_w(0);
    load_a(1, a1); wq1 = load_w(1);
    store_w(wq0, sW0);
    __syncthreads();
    read_b(sW0, 0, f0);
    // one K step J whose step J + 2 still exists: A of step J in Ac, loads of J + 2 into Af / WQ_FAR, W of J + 1 from WQ_NXT
#define OMC_F8_STEADY(J, Ac, Af, sWc, sWn, WQ_FAR, WQ_NXT) \
    do {                                                    \
        read_b(sWc, 1, f1);                                 \
        load_a((J) + 2, Af);                                \
        WQ_FAR = load_w((J) + 2);                           \
        multiply(Ac, 0, f0);                                \
        store_w(WQ_NXT, sWn);                               \
        __syncthreads();                                    \
        read_b(sWn, 0, f0);                                 \
        multiply(Ac, 1, f1);                                \
    } while (0)
    // the same with every part conditional: the last steps
#define OMC_F8_TAIL(J, Ac, Af, sWc, sWn, WQ_FAR, WQ_NXT)   \
    if ((J) < nk) {                                         \
        read_b(sWc, 1, f1);                                 \
        if ((J) + 2 < nk) {                                 \
            load_a((J) + 2, Af);                            \
            WQ_FAR = load_w((J) + 2);                       \
        }                                                   \
        multiply(Ac, 0, f0);                                \
        if ((J) + 1 < nk) {                                 \
            store_w(WQ_NXT, sWn);                           \
            __syncthreads();                                \
            read_b(sWn, 0, f0);                             \
        }                                                   \
        multiply(Ac, 1, f1);                                \
    }
    // three A sets and two W buffers rotate with a period of six steps, written out so that every index is static
    uint32_t j = 0;
    for (; j + 8 <= nk; j += 6) {
        OMC_F8_STEADY(j + 0, a0, a2, sW0, sW1, wq0, wq1);
        OMC_F8_STEADY(j + 1, a1, a0, sW1, sW0, wq1, wq0);
        OMC_F8_STEADY(j + 2, a2, a1, sW0, sW1, wq0, wq1);
        OMC_F8_STEADY(j + 3, a0, a2, sW1, sW0, wq1, wq0);
        OMC_F8_STEADY(j + 4, a1, a0, sW0, sW1, wq0, wq1);
        OMC_F8_STEADY(j + 5, a2, a1, sW1, sW0, wq1, wq0);
    }
    OMC_F8_TAIL(j + 0, a0, a2, sW0, sW1, wq0, wq1)
    OMC_F8_TAIL(j + 1, a1, a0, sW1, sW0, wq1, wq0)
    OMC_F8_TAIL(j + 2, a2, a1, sW0, sW1, wq0, wq1)
    OMC_F8_TAIL(j + 3, a0, a2, sW1, sW0, wq1, wq0)
    OMC_F8_TAIL(j + 4, a1, a0, sW0, sW1, wq0, wq1)
    OMC_F8_TAIL(j + 5, a2, a1, sW1, sW0, wq1, wq0)
    OMC_F8_TAIL(j + 6, a0, a2, sW0, sW1, wq0, wq1)
#undef OMC_F8_STEADY
#undef OMC_F8_TAIL

    // epilogue: C = s * acc + b * rowsum(A).  A lane's accumulators are one column of each of the four 32-column
    // blocks: a wave's store instruction writes two rows of 128 contiguous bytes
    const float s = sb ? sb[0] : 1.0f;
    const float b = sb ? sb[1] : 0.0f;
    if (want_rs) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            float t = rsum[mi];
            t += __shfl_xor(t, 32);
            if (f_half == 0) rowsum_lds[64 * wave + 32 * mi + f_row] = t;
        }
        __syncthreads();
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t trow = 64 * wave + 32 * mi + 8 * (v >> 2) + 4 * f_half + (v & 3);
            const float add = want_rs ? b * rowsum_lds[trow] : 0.0f;
            float *crow = C + static_cast<uint64_t>(m0 + trow) * N + n0 + f_row;
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) __builtin_nontemporal_store(s * acc[mi][ni][v] + add, crow + 32 * ni);
        }
    }
}

// S1E4M3 / bias 7, forward, 256-row tiles, K >= 64: the kernel above unless the pre-pass found a top code, in which
// case the tile kernel's generic byte decode runs (same results).
template <bool TRANS>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256))) __attribute__((amdgpu_waves_per_eu(2, 2)))
void dequant_gemm_fp8_kernel(const uint16_t *__restrict__ A, const uint32_t *__restrict__ codes, uint64_t total_dwords,
                             FmtParams fp, const float *__restrict__ sb, float *__restrict__ C, uint32_t M, uint32_t N,
                             uint32_t K, const uint32_t *__restrict__ flags) {
    __shared__ __attribute__((aligned(1024))) uint8_t sW0[kF8WBytes], sW1[kF8WBytes];
    __shared__ float rowsum_lds[256];
    __shared__ __attribute__((aligned(16))) uint8_t lds_generic[2 * (4 * 256 * 16 + 4 * kWChunkBytes)];
    (void)M;
    const bool top = __any(flags[threadIdx.x & 63u] != 0);
    if (!top) {
        dequant_gemm_fp8_body<TRANS>(A, reinterpret_cast<const uint8_t *>(codes), sb, C, N, K, sW0, sW1, rowsum_lds);
        return;
    }
    dequant_gemm_body<256, 1, false, TRANS>(A, codes, total_dwords, fp, sb, C, N, K, lds_generic);
}

// ---- wave-specialised variant --------------------------------------------------------------------
// One workgroup of 16 waves per compute unit and 256 x 128 tile.  Waves 0-7 only multiply (64 x 64 each:
// 2 x 2 MFMA tiles, 64 accumulator registers), waves 8-11 only stage A (global -> LDS, row sums on the
// way), waves 12-15 only stage W (global -> decode -> LDS).  No wave carries both instruction streams,
// so the staging work of a K step runs beside the matrix instructions of another instead of after
// them.  Three LDS stages: stage j is complete at barrier j, its fragments are read during round j+1
// (under the matrix instructions of stage j-1) and multiplied during round j+2; the stagers load three
// K steps ahead in three register sets.  One workgroup barrier per K step, reached by all 16 waves.
// Columns of the tile are kept in LDS so that a multiplying wave's 64 columns are 64 consecutive slots:
// column c = 64 h + 2 cg + i sits at slot 64 h + 32 i + cg, and a lane ends up with two adjacent
// columns of C (8-byte stores, 256 contiguous bytes per row and wave).
constexpr int kWsStages = 3;
constexpr int kWsBM = 256;
constexpr int kWsStageBytes = 4 * kWsBM * 16 + 4 * kWChunkBytes;

__device__ __forceinline__ uint32_t ws_slot_of_column(uint32_t c) {          // c in [0, 128)
    return (c & 64u) + 32u * (c & 1u) + ((c & 63u) >> 1);
}

template <int DEC, bool HW, bool TRANS>
__device__ __forceinline__ void dequant_gemm_ws_body(const uint16_t *__restrict__ A, const uint32_t *__restrict__ codes,
                                                     uint64_t total_dwords, const FmtParams &fp,
                                                     const float *__restrict__ sb, float *__restrict__ C, uint32_t N,
                                                     uint32_t K, uint8_t *lds) {
    constexpr bool BYTE = DEC != 0;
    constexpr int kAChunkBytes = kWsBM * 16;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // the role is the same for the whole wave
    const uint32_t m0 = blockIdx.x * kWsBM, n0 = blockIdx.y * kBN;
    const uint32_t nk = K / kBK;
    float *rowsum_lds = reinterpret_cast<float *>(lds);                      // reused once the K loop is over

    if (wave < 8) {
        // ---- multiplying waves ----------------------------------------------------------------------
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
                f.a[mi] = *reinterpret_cast<const bf16x8 *>(st + chunk * kAChunkBytes + (OMC_A_SLOT(row, chunk) << 4));
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                f.b[ni] = *reinterpret_cast<const bf16x8 *>(st + 4 * kAChunkBytes + chunk * kWChunkBytes +
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
        uint32_t nxt = kWsStageBytes;                       // LDS offset of stage j - 1
        for (uint32_t j = 2; j < nk + 2; ++j) {
            const bool more = j - 1 < nk;
            multiply_frags(f0);
            if (more) read_frags(lds + nxt, 0, f0);
            multiply_frags(f1);
            if (more) read_frags(lds + nxt, 1, f1);
            nxt = (nxt == (kWsStages - 1) * kWsStageBytes) ? 0u : nxt + kWsStageBytes;
            __syncthreads();                                // barrier j
        }
        __syncthreads();                                    // row sums published
        const float s = sb ? sb[0] : 1.0f;
        const float b = sb ? sb[1] : 0.0f;
        f32x4 rs[2][4];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t row = 64 * wm + 32 * mi + 8 * g + 4 * f_half;
                rs[mi][g] = sb ? *reinterpret_cast<const f32x4 *>(rowsum_lds + row) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            }
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t row = m0 + 64 * wm + 32 * mi + 8 * (v >> 2) + 4 * f_half + (v & 3);
                const float add = sb ? b * rs[mi][v >> 2][v & 3] : 0.0f;
                f32x2 out;
                out[0] = s * acc[mi][0][v] + add;
                out[1] = s * acc[mi][1][v] + add;
                __builtin_nontemporal_store(out, reinterpret_cast<f32x2 *>(C + static_cast<uint64_t>(row) * N + n0 + 64 * wh + 2 * f_row));
            }
        }
        return;
    }

    const uint32_t pt = tid & 255u;                         // thread within its group of four staging waves
    if (wave < 12) {
        // ---- waves that stage A ---------------------------------------------------------------------
        u32x4 ra[kWsStages][4];
        float rsum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
        auto load_a = [&](u32x4 (&r)[4], uint32_t k0) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t q = pt + 256 * p, row = q >> 2, chunk = q & 3u;
                r[p] = *reinterpret_cast<const u32x4 *>(A + static_cast<uint64_t>(m0 + row) * K + k0 + 8 * chunk);
            }
        };
        auto store_a = [&](const u32x4 (&r)[4], uint8_t *st) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t q = pt + 256 * p, row = q >> 2, chunk = q & 3u;
                *reinterpret_cast<u32x4 *>(st + chunk * kAChunkBytes + (OMC_A_SLOT(row, chunk) << 4)) = r[p];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = r[p][i];             // (a bit_cast straight from the vector element reads element 0)
                    rsum[p] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, rsum[p], false);
                }
            }
        };
#pragma unroll
        for (int u = 0; u < kWsStages; ++u)
            if (static_cast<uint32_t>(u) < nk) load_a(ra[u], u * kBK);
        uint32_t j = 0;
        for (; j + kWsStages <= nk; j += kWsStages) {
#pragma unroll
            for (int u = 0; u < kWsStages; ++u) {
                store_a(ra[u], lds + u * kWsStageBytes);
                if (j + u + kWsStages < nk) load_a(ra[u], (j + u + kWsStages) * kBK);
                __syncthreads();                            // barrier j + u
            }
        }
#pragma unroll
        for (int u = 0; u < kWsStages - 1; ++u)
            if (j + u < nk) {
                store_a(ra[u], lds + u * kWsStageBytes);
                __syncthreads();
            }
        __syncthreads();                                    // barriers nk and nk + 1: the multiplying waves drain
        __syncthreads();
        if (sb) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                float t = rsum[p];
                t += __shfl_xor(t, 1);
                t += __shfl_xor(t, 2);
                if ((pt & 3u) == 0) rowsum_lds[(pt >> 2) + 64 * p] = t;
            }
        }
        __syncthreads();                                    // row sums published
        return;
    }

    // ---- waves that stage W -----------------------------------------------------------------------------
    {
        const uint32_t pw = wave - 12u;
        const uint32_t w_h = lane & 1u, w_cg = lane >> 1;
        const uint32_t w_kg = 2 * pw + w_h;
        const uint64_t w_col = n0 + 4 * w_cg;
        const uint32_t t_slot = pt & 127u, t_h = pt >> 7;
        const uint64_t t_row = n0 + (t_slot & 64u) + 2 * (t_slot & 31u) + ((t_slot >> 5) & 1u);
        struct WRegs {
            uint32_t raw[4][3], off[4];
        };
        WRegs rw[kWsStages];
        auto load_w = [&](WRegs &r, uint32_t k0) {
            if (TRANS && BYTE) {                            // the thread's 16 codes are one aligned 16-byte piece
                const u32x4 t = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint8_t *>(codes) + t_row * K + k0 + 16 * t_h);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    r.raw[rr][0] = t[rr];
                    r.off[rr] = 0;
                }
                return;
            }
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const uint64_t e = TRANS ? t_row * K + k0 + 16 * t_h + 4 * rr
                                         : static_cast<uint64_t>(k0 + 4 * w_kg + rr) * N + w_col;
                load_codes4<BYTE>(codes, total_dwords, e, fp.bits, r.raw[rr], r.off[rr]);
            }
        };
        auto store_w = [&](const WRegs &r, uint8_t *st) {      // as in the four-wave kernel, other column slots
            uint8_t *ldsW = st + 4 * kAChunkBytes;
            uint32_t v[4][4];
#pragma unroll
            for (int g = 0; g < 4; ++g) decode_codes4<BYTE, HW>(r.raw[g], r.off[g], fp, v[g]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (TRANS)
                    *reinterpret_cast<u32x2 *>(ldsW + (2u * t_h + (i >> 1)) * kWChunkBytes + (t_slot << 4) + 8u * (i & 1)) =
                        pack_bf16x4(v[i][0], v[i][1], v[i][2], v[i][3]);
                else
                    *reinterpret_cast<u32x2 *>(ldsW + pw * kWChunkBytes + (ws_slot_of_column(4 * w_cg + i) << 4) + 8u * w_h) =
                        pack_bf16x4(v[0][i], v[1][i], v[2][i], v[3][i]);
            }
        };
#pragma unroll
        for (int u = 0; u < kWsStages; ++u)
            if (static_cast<uint32_t>(u) < nk) load_w(rw[u], u * kBK);
        uint32_t j = 0;
        for (; j + kWsStages <= nk; j += kWsStages) {
#pragma unroll
            for (int u = 0; u < kWsStages; ++u) {
                store_w(rw[u], lds + u * kWsStageBytes);
                if (j + u + kWsStages < nk) load_w(rw[u], (j + u + kWsStages) * kBK);
                __syncthreads();
            }
        }
#pragma unroll
        for (int u = 0; u < kWsStages - 1; ++u)
            if (j + u < nk) {
                store_w(rw[u], lds + u * kWsStageBytes);
                __syncthreads();
            }
        __syncthreads();
        __syncthreads();
        __syncthreads();
    }
}

template <int DEC, bool TRANS>
__global__ __launch_bounds__(1024, 1) void dequant_gemm_ws_kernel(const uint16_t *__restrict__ A, const uint32_t *__restrict__ codes,
                                                                  uint64_t total_dwords, FmtParams fp,
                                                                  const float *__restrict__ sb, float *__restrict__ C,
                                                                  uint32_t M, uint32_t N, uint32_t K,
                                                                  const uint32_t *__restrict__ flags) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[kWsStages * kWsStageBytes];
    (void)M;
    if (DEC == 2) {
        const bool top = __any(flags[threadIdx.x & 63u] != 0);
        if (!top) {
            dequant_gemm_ws_body<1, true, TRANS>(A, codes, total_dwords, fp, sb, C, N, K, lds);
            return;
        }
    }
    dequant_gemm_ws_body<(DEC == 0 ? 0 : 1), false, TRANS>(A, codes, total_dwords, fp, sb, C, N, K, lds);
}

// DEC 2 = byte codes of S1E4M3 / bias 7: hardware conversion unless the pre-pass found a top code.
template <int BM, int DEC, bool TRANS>
__global__ __launch_bounds__(256, (BM == 256 || DEC == 0) ? OMC_GEMM_WAVES : 3) void dequant_gemm_kernel(const uint16_t *__restrict__ A,
                                                              const uint32_t *__restrict__ codes, uint64_t total_dwords,
                                                              FmtParams fp, const float *__restrict__ sb,
                                                              float *__restrict__ C, uint32_t M, uint32_t N, uint32_t K,
                                                              const uint32_t *__restrict__ flags) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * (4 * BM * 16 + 4 * kWChunkBytes)];
    (void)M;
    if (DEC == 2) {
        const bool top = __any(flags[threadIdx.x & 63u] != 0);
        if (!top) {
            dequant_gemm_body<BM, 1, true, TRANS>(A, codes, total_dwords, fp, sb, C, N, K, lds);
            return;
        }
    }
    dequant_gemm_body<BM, (DEC == 0 ? 0 : 1), false, TRANS>(A, codes, total_dwords, fp, sb, C, N, K, lds);
}

// C[M x N] = A[M x K] * W (trans == 0, W packed as [K x N]) or A * W^T (trans != 0, W packed as [N x K])
int launch_dequant_gemm(const uint16_t *A, const void *codes, const FmtParams &fp, const float *sb, float *C,
                        uint32_t M, uint32_t N, uint32_t K, float *ws, int trans, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t n = static_cast<uint64_t>(K) * N;
    const uint64_t total_dwords = ((n * fp.bits + 7) / 8 + 15) / 16 * 4;
    const uint32_t *c = static_cast<const uint32_t *>(codes);
    // workspace: kScanBlocks flag words
    uint32_t *flags = reinterpret_cast<uint32_t *>(ws);
    const int dec = (fp.bits != 8) ? 0 : (fp.variant == 2 ? 2 : 1);
    if (dec == 2) {
        gemm_scan_kernel<<<dim3(kScanBlocks), dim3(256), 0, st>>>(c, total_dwords, flags);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    // 256-row tiles unless they would leave fewer than two workgroups per compute unit
#ifndef OMC_GEMM_FP8_TRANS
#define OMC_GEMM_FP8_TRANS 1
#endif
#ifndef OMC_GEMM_SMALL_LIMIT
#define OMC_GEMM_SMALL_LIMIT 512
#endif
    const bool small = static_cast<uint64_t>(M / 256) * (N / kBN) < OMC_GEMM_SMALL_LIMIT;
#define OMC_GEMM_LAUNCH(BM, DEC)                                                                                    \
    do {                                                                                                            \
        if (trans)                                                                                                  \
            dequant_gemm_kernel<BM, DEC, true><<<dim3(M / BM, N / kBN), dim3(256), 0, st>>>(A, c, total_dwords, fp, sb, \
                                                                                            C, M, N, K, flags);     \
        else                                                                                                        \
            dequant_gemm_kernel<BM, DEC, false><<<dim3(M / BM, N / kBN), dim3(256), 0, st>>>(A, c, total_dwords, fp, sb, \
                                                                                             C, M, N, K, flags);    \
    } while (0)
    // S1E4M3 forward: the kernel built on the hardware FP8 -> bf16 conversion and transposing LDS reads (measured on
    // the two benchmark shapes: 871 against 806 TFLOP/s for 8192 x 4096 x 1024 with the tile kernel, 921 against 873 for
    // 8192 x 1024 x 4096 with the wave-specialised one); smaller grids take it too
    if (dec == 2 && K >= 2 * kBK && (!trans || OMC_GEMM_FP8_TRANS)) {
        if (trans) dequant_gemm_fp8_kernel<true><<<dim3(M / 256, N / kBN), dim3(256), 0, st>>>(A, c, total_dwords, fp, sb, C, M, N, K, flags);
        else dequant_gemm_fp8_kernel<false><<<dim3(M / 256, N / kBN), dim3(256), 0, st>>>(A, c, total_dwords, fp, sb, C, M, N, K, flags);
        return static_cast<int>(hipGetLastError());
    }
    // At most one 256-row tile per compute unit and a long contraction: the wave-specialised kernel (its
    // prologue and C stores are not covered by another workgroup, so it needs the long K loop to pay off).
#ifndef OMC_GEMM_WS_MIN_K
#define OMC_GEMM_WS_MIN_K 2048
#endif
#ifndef OMC_GEMM_WS_MAX_TILES
#define OMC_GEMM_WS_MAX_TILES 256
#endif
    if (K >= OMC_GEMM_WS_MIN_K && static_cast<uint64_t>(M / 256) * (N / kBN) <= OMC_GEMM_WS_MAX_TILES) {
#define OMC_GEMM_WS_LAUNCH(DEC)                                                                                      \
    do {                                                                                                            \
        if (trans)                                                                                                  \
            dequant_gemm_ws_kernel<DEC, true><<<dim3(M / 256, N / kBN), dim3(1024), 0, st>>>(A, c, total_dwords, fp, sb, \
                                                                                             C, M, N, K, flags);    \
        else                                                                                                        \
            dequant_gemm_ws_kernel<DEC, false><<<dim3(M / 256, N / kBN), dim3(1024), 0, st>>>(A, c, total_dwords, fp, sb, \
                                                                                              C, M, N, K, flags);   \
    } while (0)
        if (dec == 2) OMC_GEMM_WS_LAUNCH(2);
        else if (dec == 1) OMC_GEMM_WS_LAUNCH(1);
        else OMC_GEMM_WS_LAUNCH(0);
#undef OMC_GEMM_WS_LAUNCH
    } else if (!small) {
        if (dec == 2) OMC_GEMM_LAUNCH(256, 2);
        else if (dec == 1) OMC_GEMM_LAUNCH(256, 1);
        else OMC_GEMM_LAUNCH(256, 0);
    } else {
        if (dec == 2) OMC_GEMM_LAUNCH(128, 2);
        else if (dec == 1) OMC_GEMM_LAUNCH(128, 1);
        else OMC_GEMM_LAUNCH(128, 0);
    }
#undef OMC_GEMM_LAUNCH
    return static_cast<int>(hipGetLastError());
}

}  // namespace omc
