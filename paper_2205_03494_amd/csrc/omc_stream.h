// Device side of the streaming kernels: unpack / decode / transform / update / round / pack
// for one 2048-element tile per wavefront (paper Sec. 2.1 cycle, Sec. 2.2 format, Sec. 2.3 fit).
//
// Data movement.  Every global access is coalesced: a wave reads or writes whole contiguous
// runs (packed codes as dwords, fp32 streams as 16-byte pieces).  Each lane, however, works on
// 32 *consecutive* elements, because 32 codes of any width B are exactly B dwords: all shift
// amounts are then compile-time constants and no dword is shared between lanes.  The change of
// ownership between the two layouts goes through LDS (one wave, one private LDS region), with
// padding / XOR swizzles chosen so that both sides are free of bank conflicts.
//
// Arithmetic.  fp32 operations are written one per statement and the file is compiled with
// contraction off, so that each is rounded on its own.  Rounding to the format is done in the
// value domain of fp32 itself: adding and subtracting 2^(ex+23-M) rounds to M mantissa bits
// with the hardware's nearest-even rule, and a clamped exponent gives gradual underflow.
#pragma once
#include <hip/hip_runtime.h>
#include "omc_internal.h"

#pragma clang fp contract(off)

namespace omc {

enum Mode : int { kCompress = 0, kDecompress = 1, kStepSgd = 2, kStepMomentum = 3, kStepAdam = 4 };

struct OptConst {
    float lr, momentum, beta1, beta2, eps, omb1, omb2, bc1, bc2;
};

// ---- LDS layouts ----------------------------------------------------------------------------
// Packed tile of 64*B dwords.  Lane l owns dwords [l*B, l*B+B).  With B = 2^t * odd, a stride of
// B dwords between lanes hits only every 2^t-th bank, so one spare dword is inserted after
// every 32*odd dwords: lane l's run starts at l*B + (l >> (5 - t)).
template <int B>
struct CodeLds {
    static constexpr int t = (B % 2) ? 0 : (B % 4) ? 1 : (B % 8) ? 2 : (B % 16) ? 3 : (B % 32) ? 4 : 5;
    static constexpr int odd = B >> t;
    static constexpr bool padded = (t > 0);
    __device__ static __forceinline__ uint32_t lane_base(uint32_t lane) {
        return padded ? lane * B + (lane >> (5 - t)) : lane * B;
    }
    __device__ static __forceinline__ uint32_t flat(uint32_t p) {  // p: dword index in the tile
        return padded ? p + p / (32u * odd) : p;
    }
};

// fp32 tile of 2048 floats handled as 512 pieces of 16 bytes.  Lane l owns pieces [8l, 8l+8);
// piece k of lane l is stored at 8l + (k ^ (l & 7)) so that eight lanes reading "their k-th
// piece" cover all banks.
__device__ __forceinline__ uint32_t piece_slot_flat(uint32_t j, uint32_t lane) {
    // piece q = 64 j + lane belongs to lane' = q >> 3 = 8 j + (lane >> 3), position k = lane & 7
    return j * 64u + (lane & ~7u) + ((lane & 7u) ^ ((lane >> 3) & 7u));
}
__device__ __forceinline__ uint32_t piece_slot_own(uint32_t k, uint32_t lane) {
    return lane * 8u + (k ^ (lane & 7u));
}

__device__ __forceinline__ void lds_fence() { __syncthreads(); }  // one wave per workgroup

// ---- global <-> registers, coalesced ---------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void load_f32_pieces(const float *__restrict__ src, uint32_t valid,
                                                uint32_t lane, float4 (&g)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t e = (j * 64u + lane) * 4u;
        if (FULL) {
            g[j] = *reinterpret_cast<const float4 *>(src + e);
        } else {
            g[j].x = (e + 0 < valid) ? src[e + 0] : 0.0f;
            g[j].y = (e + 1 < valid) ? src[e + 1] : 0.0f;
            g[j].z = (e + 2 < valid) ? src[e + 2] : 0.0f;
            g[j].w = (e + 3 < valid) ? src[e + 3] : 0.0f;
        }
    }
}

template <bool FULL>
__device__ __forceinline__ void store_f32_pieces(float *__restrict__ dst, uint32_t valid,
                                                 uint32_t lane, const float4 (&g)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t e = (j * 64u + lane) * 4u;
        if (FULL) {
            *reinterpret_cast<float4 *>(dst + e) = g[j];
        } else {
            if (e + 0 < valid) dst[e + 0] = g[j].x;
            if (e + 1 < valid) dst[e + 1] = g[j].y;
            if (e + 2 < valid) dst[e + 2] = g[j].z;
            if (e + 3 < valid) dst[e + 3] = g[j].w;
        }
    }
}

// coalesced pieces -> each lane's 32 consecutive floats
__device__ __forceinline__ void pieces_to_lanes(const float4 (&g)[8], float (&r)[32], uint32_t *lds,
                                                uint32_t lane) {
    float4 *l4 = reinterpret_cast<float4 *>(lds);
#pragma unroll
    for (int j = 0; j < 8; ++j) l4[piece_slot_flat(j, lane)] = g[j];
    lds_fence();
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float4 t = l4[piece_slot_own(k, lane)];
        r[4 * k + 0] = t.x; r[4 * k + 1] = t.y; r[4 * k + 2] = t.z; r[4 * k + 3] = t.w;
    }
    lds_fence();
}

// each lane's 32 consecutive floats -> coalesced pieces
__device__ __forceinline__ void lanes_to_pieces(const float (&r)[32], float4 (&g)[8], uint32_t *lds,
                                                uint32_t lane) {
    float4 *l4 = reinterpret_cast<float4 *>(lds);
#pragma unroll
    for (int k = 0; k < 8; ++k)
        l4[piece_slot_own(k, lane)] = make_float4(r[4 * k + 0], r[4 * k + 1], r[4 * k + 2], r[4 * k + 3]);
    lds_fence();
#pragma unroll
    for (int j = 0; j < 8; ++j) g[j] = l4[piece_slot_flat(j, lane)];
    lds_fence();
}

template <int B, bool FULL>
__device__ __forceinline__ void load_code_dwords(const uint32_t *__restrict__ src, uint64_t dwords_left,
                                                 uint32_t lane, uint32_t (&cw)[B]) {
#pragma unroll
    for (int j = 0; j < B; ++j) {
        uint32_t p = j * 64u + lane;
        cw[j] = (FULL || p < dwords_left) ? src[p] : 0u;
    }
}

template <int B, bool FULL>
__device__ __forceinline__ void store_code_dwords(uint32_t *__restrict__ dst, uint64_t dwords_left,
                                                  uint32_t lane, const uint32_t (&cw)[B]) {
#pragma unroll
    for (int j = 0; j < B; ++j) {
        uint32_t p = j * 64u + lane;
        if (FULL || p < dwords_left) dst[p] = cw[j];
    }
}

template <int B>
__device__ __forceinline__ void code_dwords_to_lanes(const uint32_t (&cw)[B], uint32_t (&w)[B],
                                                     uint32_t *lds, uint32_t lane) {
#pragma unroll
    for (int j = 0; j < B; ++j) lds[CodeLds<B>::flat(j * 64u + lane)] = cw[j];
    lds_fence();
    const uint32_t base = CodeLds<B>::lane_base(lane);
#pragma unroll
    for (int j = 0; j < B; ++j) w[j] = lds[base + j];
    lds_fence();
}

template <int B>
__device__ __forceinline__ void lanes_to_code_dwords(const uint32_t (&o)[B], uint32_t (&cw)[B],
                                                     uint32_t *lds, uint32_t lane) {
    const uint32_t base = CodeLds<B>::lane_base(lane);
#pragma unroll
    for (int j = 0; j < B; ++j) lds[base + j] = o[j];
    lds_fence();
#pragma unroll
    for (int j = 0; j < B; ++j) cw[j] = lds[CodeLds<B>::flat(j * 64u + lane)];
    lds_fence();
}

// ---- codec ------------------------------------------------------------------------------------
// Element i of a lane's B dwords, returned with its sign bit at bit 31 (lower bits: the rest of
// the code, then unrelated bits that the decoder masks away).
template <int B>
__device__ __forceinline__ uint32_t code_at_top(const uint32_t (&w)[B], int i) {
    const int p = i * B, idx = p >> 5, off = p & 31;
    if (off + B <= 32) return w[idx] << (32 - B - off);
    return __builtin_amdgcn_alignbit(w[(idx + 1 < B) ? idx + 1 : idx], w[idx], off + B - 32);
}

// Sec. 2.2 value of a code.  Align [sign | e | m] with the fp32 fields, drop everything else,
// and scale by 2^(127 - bias); an e == 0 code becomes an fp32 subnormal whose product with the
// scale is exactly the format's subnormal value.
__device__ __forceinline__ float decode_top(uint32_t t, const FmtParams &fp) {
    int32_t u = static_cast<int32_t>(t) >> fp.asr;
    u &= static_cast<int32_t>(fp.keep_mask);
    return __uint_as_float(static_cast<uint32_t>(u)) * fp.dec_scale;
}

// Nearest code to x (ties to even significand, saturating) and the value tq of that code.
__device__ __forceinline__ void encode(float x, const FmtParams &fp, uint32_t &code, float &tq) {
    const uint32_t xb = __float_as_uint(x);
    // |x| clamped to the largest magnitude, compared as integers so that Inf and NaN saturate too
    const uint32_t ab = min(xb & 0x7fffffffu, __float_as_uint(fp.maxval));
    const float a = __uint_as_float(ab);
    const uint32_t exb = max(ab, fp.min_norm_bits) & 0x7f800000u;  // binade of a, at least the first normal one
    float r;
    if (fp.wide) {
        const int k = static_cast<int>(exb >> 23) - fp.exp_adj;    // ulp = 2^k
        r = ldexpf(rintf(ldexpf(a, -k)), k);
    } else {
        const float magic = __uint_as_float(exb + fp.magic_off);   // 2^(ex + 23 - M)
        const float t = a + magic;                                  // rounds a to a multiple of 2^(ex - M)
        r = t - magic;
    }
    const float scaled = r * fp.enc_scale;                          // exponent field becomes e, subnormals included
    const uint32_t mag = __float_as_uint(scaled) >> fp.sh;
    code = mag | ((xb >> 31) << (fp.bits - 1));
    tq = __uint_as_float(__float_as_uint(r) | (xb & 0x80000000u));
}

template <int B>
__device__ __forceinline__ void pack_at(uint32_t (&o)[B], int i, uint32_t code) {
    const int p = i * B, idx = p >> 5, off = p & 31;
    if (off == 0) o[idx] = code; else o[idx] |= code << off;
    if (off + B > 32) o[(idx + 1 < B) ? idx + 1 : idx] = code >> (32 - off);
}

// ---- parameter update (see omc.h for the exact forms) -------------------------------------------
template <int MODE>
__device__ __forceinline__ float apply_update(float w, float g, float &m, float &v, const OptConst &oc) {
    if (MODE == kStepSgd) {
        const float d = oc.lr * g;
        return w - d;
    } else if (MODE == kStepMomentum) {
        const float mm = oc.momentum * m;
        const float mn = mm + g;
        m = mn;
        const float d = oc.lr * mn;
        return w - d;
    } else {
        const float m1 = oc.beta1 * m;
        const float m2 = oc.omb1 * g;
        const float mn = m1 + m2;
        const float v1 = oc.beta2 * v;
        const float v2 = oc.omb2 * g;
        const float v3 = v2 * g;
        const float vn = v1 + v3;
        m = mn;
        v = vn;
        const float mhat = mn / oc.bc1;
        const float vhat = vn / oc.bc2;
        const float num = oc.lr * mhat;
        const float rt = sqrtf(vhat);
        const float den = rt + oc.eps;
        const float d = num / den;
        return w - d;
    }
}

// ---- fit accumulators -----------------------------------------------------------------------------
struct FitAcc {
    double sV, sT, sVT, sTT;
    float tmin, tmax;
    __device__ __forceinline__ void clear() {
        sV = sT = sVT = sTT = 0.0;
        tmin = __builtin_huge_valf();
        tmax = -__builtin_huge_valf();
    }
    __device__ __forceinline__ void add(float x, float tq) {
        const double dx = static_cast<double>(x), dt = static_cast<double>(tq);
        sV += dx;
        sT += dt;
        sVT = fma(dx, dt, sVT);   // the product of two fp32 values is exact in fp64
        sTT = fma(dt, dt, sTT);
        tmin = fminf(tmin, tq);
        tmax = fmaxf(tmax, tq);
    }
    // butterfly over the 64 lanes; every lane ends with the same totals, in an order that does
    // not depend on scheduling
    __device__ __forceinline__ void wave_reduce() {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            sV += __shfl_xor(sV, off);
            sT += __shfl_xor(sT, off);
            sVT += __shfl_xor(sVT, off);
            sTT += __shfl_xor(sTT, off);
            tmin = fminf(tmin, __shfl_xor(tmin, off));
            tmax = fmaxf(tmax, __shfl_xor(tmax, off));
        }
    }
};

// ---- one tile ---------------------------------------------------------------------------------------
struct TileArgs {
    uint32_t *codes;          // variable's packed stream (nullptr for fp32 input of kCompress: unused)
    uint64_t total_dwords;    // its length in dwords
    const float *vin;         // kCompress: values to compress
    float *vout;              // kDecompress: output
    const float *grad;        // step modes
    float *st0, *st1;         // step modes
    float s, b;               // transformation in force for decoding
    uint64_t n;
};

template <int B, int MODE, bool FULL>
__device__ __forceinline__ void do_tile(const TileArgs &a, const FmtParams &fp, const OptConst &oc,
                                        uint64_t e0, uint32_t valid, uint32_t lane, uint32_t *lds,
                                        FitAcc &acc) {
    const uint64_t dw0 = (e0 >> 5) * B;                   // first dword of the tile
    const uint64_t dw_left = a.total_dwords - dw0;

    // 1. all global loads first, so that they are in flight together
    uint32_t cw[B];
    float4 gq[8], mq[8], vq[8];
    if (MODE != kCompress) load_code_dwords<B, FULL>(a.codes + dw0, dw_left, lane, cw);
    if (MODE == kCompress) load_f32_pieces<FULL>(a.vin + e0, valid, lane, gq);
    if (MODE >= kStepSgd) load_f32_pieces<FULL>(a.grad + e0, valid, lane, gq);
    if (MODE >= kStepMomentum) load_f32_pieces<FULL>(a.st0 + e0, valid, lane, mq);
    if (MODE == kStepAdam) load_f32_pieces<FULL>(a.st1 + e0, valid, lane, vq);

    // 2. hand every lane its 32 consecutive elements
    uint32_t w[B];
    float rg[32], rm[32], rv[32];
    if (MODE != kCompress) code_dwords_to_lanes<B>(cw, w, lds, lane);
    if (MODE == kCompress || MODE >= kStepSgd) pieces_to_lanes(gq, rg, lds, lane);
    if (MODE >= kStepMomentum) pieces_to_lanes(mq, rm, lds, lane);
    if (MODE == kStepAdam) pieces_to_lanes(vq, rv, lds, lane);

    // 3. the cycle, element by element
    uint32_t o[B];
#pragma unroll
    for (int j = 0; j < B; ++j) o[j] = 0u;
    const uint32_t first = lane * kLaneElems;
#pragma unroll
    for (int i = 0; i < kLaneElems; ++i) {
        float x;
        if (MODE != kCompress) {
            const float vt = decode_top(code_at_top<B>(w, i), fp);
            const float sv = a.s * vt;
            x = sv + a.b;
        } else {
            x = rg[i];
        }
        if (MODE == kDecompress) {
            rg[i] = x;
            continue;
        }
        if (MODE >= kStepSgd) {
            float mdummy = 0.0f, vdummy = 0.0f;
            x = apply_update<MODE>(x, rg[i], MODE >= kStepMomentum ? rm[i] : mdummy,
                                   MODE == kStepAdam ? rv[i] : vdummy, oc);
        }
        const bool live = FULL || (first + i < valid);
        if (!live) x = 0.0f;                             // padding elements pack as zero bits
        uint32_t code;
        float tq;
        encode(x, fp, code, tq);
        pack_at<B>(o, i, code);
        if (live) acc.add(x, tq);
    }

    // 4. back to the coalesced layouts and out
    if (MODE == kDecompress) {
        lanes_to_pieces(rg, gq, lds, lane);
        store_f32_pieces<FULL>(a.vout + e0, valid, lane, gq);
        return;
    }
    if (MODE >= kStepMomentum) {
        lanes_to_pieces(rm, mq, lds, lane);
        store_f32_pieces<FULL>(a.st0 + e0, valid, lane, mq);
    }
    if (MODE == kStepAdam) {
        lanes_to_pieces(rv, vq, lds, lane);
        store_f32_pieces<FULL>(a.st1 + e0, valid, lane, vq);
    }
    lanes_to_code_dwords<B>(o, cw, lds, lane);
    store_code_dwords<B, FULL>(a.codes + dw0, dw_left, lane, cw);
}

// One work item: up to kTilesPerChunk tiles of one variable, reduced into one Partial.
template <int B, int MODE>
__device__ __forceinline__ void do_chunk(const TileArgs &a, const FmtParams &fp, const OptConst &oc,
                                         uint32_t chunk, uint32_t *lds, Partial *partial_out) {
    const uint32_t lane = threadIdx.x;
    FitAcc acc;
    acc.clear();
    const uint64_t begin = static_cast<uint64_t>(chunk) * kChunkElems;
    for (int t = 0; t < kTilesPerChunk; ++t) {
        const uint64_t e0 = begin + static_cast<uint64_t>(t) * kTileElems;
        if (e0 >= a.n) break;
        const uint64_t left = a.n - e0;
        if (left >= kTileElems)
            do_tile<B, MODE, true>(a, fp, oc, e0, kTileElems, lane, lds, acc);
        else
            do_tile<B, MODE, false>(a, fp, oc, e0, static_cast<uint32_t>(left), lane, lds, acc);
    }
    if (MODE != kDecompress) {
        acc.wave_reduce();
        if (lane == 0) {
            Partial p;
            p.sV = acc.sV; p.sT = acc.sT; p.sVT = acc.sVT; p.sTT = acc.sTT;
            p.tmin = acc.tmin; p.tmax = acc.tmax; p.pad[0] = p.pad[1] = 0;
            *partial_out = p;
        }
    }
}

// ---- finalize: per-variable (s, b) from the partials (paper Sec. 2.3) -----------------------------
struct DD {  // unevaluated sum hi + lo
    double hi, lo;
};
__device__ __forceinline__ DD dd_add(DD a, double x) {
    const double s = a.hi + x;
    const double bb = s - a.hi;
    const double err = (a.hi - (s - bb)) + (x - bb);
    const double lo = a.lo + err;
    DD r;
    r.hi = s + lo;
    r.lo = lo - (r.hi - s);
    return r;
}
__device__ __forceinline__ DD dd_add(DD a, DD b) { return dd_add(dd_add(a, b.hi), b.lo); }
__device__ __forceinline__ DD dd_shfl_xor(DD a, int off) {
    DD r;
    r.hi = __shfl_xor(a.hi, off);
    r.lo = __shfl_xor(a.lo, off);
    return r;
}

// Called by one full wave.  Sums the variable's partials in a fixed order with compensated
// additions, evaluates the closed form in fp64 and stores (s, b) as fp32.
__device__ __forceinline__ void finalize_variable(const Partial *__restrict__ parts, uint32_t nparts,
                                                  uint64_t n, bool use_pvt, float *sb_out) {
    const uint32_t lane = threadIdx.x;
    if (!use_pvt) {
        if (lane == 0) { sb_out[0] = 1.0f; sb_out[1] = 0.0f; }
        return;
    }
    DD sV{0, 0}, sT{0, 0}, sVT{0, 0}, sTT{0, 0};
    float tmin = __builtin_huge_valf(), tmax = -__builtin_huge_valf();
    bool finite = true;
    for (uint32_t i = lane; i < nparts; i += 64) {
        const Partial p = parts[i];
        finite = finite && isfinite(p.sV);
        if (finite) {
            sV = dd_add(sV, p.sV);
            sT = dd_add(sT, p.sT);
            sVT = dd_add(sVT, p.sVT);
            sTT = dd_add(sTT, p.sTT);
        }
        tmin = fminf(tmin, p.tmin);
        tmax = fmaxf(tmax, p.tmax);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        sV = dd_add(sV, dd_shfl_xor(sV, off));
        sT = dd_add(sT, dd_shfl_xor(sT, off));
        sVT = dd_add(sVT, dd_shfl_xor(sVT, off));
        sTT = dd_add(sTT, dd_shfl_xor(sTT, off));
        tmin = fminf(tmin, __shfl_xor(tmin, off));
        tmax = fmaxf(tmax, __shfl_xor(tmax, off));
        finite = __shfl_xor(static_cast<int>(finite), off) && finite;
    }
    if (lane != 0) return;
    if (!finite) {                                   // a non-finite input value poisons the fit
        sb_out[0] = __builtin_nanf("");
        sb_out[1] = __builtin_nanf("");
        return;
    }
    const double SV = sV.hi, ST = sT.hi, SVT = sVT.hi, STT = sTT.hi;
    const double dn = static_cast<double>(n);
    double s;
    if (tmin == tmax) {                              // all decompressed values equal: degenerate case
        s = 1.0;
    } else {
        const double p1 = dn * SVT;
        const double p2 = SV * ST;
        const double num = p1 - p2;
        const double q1 = dn * STT;
        const double q2 = ST * ST;
        const double den = q1 - q2;
        s = num / den;
    }
    const double sst = s * ST;
    const double b = (SV - sst) / dn;
    sb_out[0] = static_cast<float>(s);
    sb_out[1] = static_cast<float>(b);
}

// ---- dispatch over the code width ---------------------------------------------------------------------
#define OMC_FOR_EACH_BITS(X)                                                                       \
    X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17) X(18)  \
    X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30) X(31) X(32)

}  // namespace omc
