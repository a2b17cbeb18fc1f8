// Device side of the streaming kernels: unpack / decode / transform / update / round / pack
// (paper Sec. 2.1 cycle, Sec. 2.2 format, Sec. 2.3 fit).
//
// Work split.  A variable of n elements is cut into full tiles of 2048 elements (64 lanes x 32)
// plus, when n is not a multiple of 2048, one ragged tail.  Full tiles are processed by kernels
// templated on the code width B, with no bounds checks at all; tails by a small generic kernel.
//
// Data movement of the full-tile path.  Every global access is coalesced and 16 bytes per lane.
// Each lane, however, works on 32 *consecutive* elements, because 32 codes of any width B are
// exactly B dwords: all shift amounts are then compile-time constants and no dword is shared
// between lanes.  The change of ownership between the two layouts goes through LDS (one wave,
// one private LDS region), with padding / XOR swizzles chosen so that both sides are free of
// bank conflicts.
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

// Native 16-byte vectors (first-class values for the optimizer, unlike the HIP struct types).
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Mode : int { kCompress = 0, kDecompress = 1, kStepSgd = 2, kStepMomentum = 3, kStepAdam = 4 };

struct OptConst {
    float lr, momentum, beta1, beta2, eps, omb1, omb2, bc1, bc2;
};

// Per-mode tuning: occupancy target (waves per SIMD; bounds the register budget the compiler may
// use) and whether the next tile's loads are issued before the current tile is computed.
#ifndef OMC_TUNE_WAVES_LIGHT
#define OMC_TUNE_WAVES_LIGHT 3
#endif
#ifndef OMC_TUNE_SCHED_GROUP
#define OMC_TUNE_SCHED_GROUP 4
#endif
#ifndef OMC_TUNE_PREFETCH
#define OMC_TUNE_PREFETCH 1
#endif
#ifndef OMC_TUNE_WAVES_MOMENTUM
#define OMC_TUNE_WAVES_MOMENTUM 2
#endif
#ifndef OMC_TUNE_WAVES_ADAM
#define OMC_TUNE_WAVES_ADAM 2
#endif
#ifndef OMC_TUNE_DIRECT
#define OMC_TUNE_DIRECT 1
#endif
#ifndef OMC_TUNE_ADAM_WIDE_BITS
#define OMC_TUNE_ADAM_WIDE_BITS 13
#endif
#ifndef OMC_TUNE_PREFETCH_HEAVY
#define OMC_TUNE_PREFETCH_HEAVY 0
#endif
template <int MODE, int B>
struct Tuning {
    static constexpr int light = (B <= 12) ? OMC_TUNE_WAVES_LIGHT : (OMC_TUNE_WAVES_LIGHT > 3 ? 3 : OMC_TUNE_WAVES_LIGHT);
    // Adam on codes of OMC_TUNE_ADAM_WIDE_BITS bits or more does not fit 256 registers without spilling (and
    // scratch is memory traffic): one wave per SIMD with the next tile's loads in flight instead
    // byte-multiple code widths: lanes own 4-element groups, fp32 streams skip the LDS transposition
    // (not for 8-bit momentum: the registers it saves raise that kernel's occupancy from two to three waves
    // per SIMD, which measures 2 % slower there)
    static constexpr bool direct = (B % 8 == 0) && (OMC_TUNE_DIRECT != 0) && !(MODE == kStepMomentum && B == 8);
    static constexpr bool adam_wide = MODE == kStepAdam && B >= OMC_TUNE_ADAM_WIDE_BITS;
    static constexpr int waves = adam_wide ? 1 : (MODE == kStepAdam) ? OMC_TUNE_WAVES_ADAM
                                 : (MODE == kStepMomentum) ? OMC_TUNE_WAVES_MOMENTUM : light;
    // momentum: measured with every stream coming from HBM, the next tile's loads in flight during the arithmetic
    // are worth 0.3 - 1.4 % at every code width (11 bit: 303 -> 300 us on 115 M elements)
    static constexpr bool prefetch = (MODE <= kStepSgd) ? (OMC_TUNE_PREFETCH != 0)
                                     : (adam_wide || MODE == kStepMomentum || OMC_TUNE_PREFETCH_HEAVY != 0);
};

// A value that is the same in every lane (read through a vector load, e.g. from the plan) moved
// to scalar registers, so that it does not occupy a vector register per field.
template <typename T>
__device__ __forceinline__ T to_scalar_regs(const T &v) {
    static_assert(sizeof(T) % 4 == 0, "dword-sized types only");
    uint32_t tmp[sizeof(T) / 4];
    __builtin_memcpy(tmp, &v, sizeof(T));
#pragma unroll
    for (unsigned i = 0; i < sizeof(T) / 4; ++i) tmp[i] = __builtin_amdgcn_readfirstlane(tmp[i]);
    T out;
    __builtin_memcpy(&out, tmp, sizeof(T));
    return out;
}

// An empty, ordered asm statement that "modifies" a register.  Work that produces the value must
// precede it and work that consumes it must follow, and such statements keep their program order:
// placed at the start and end of a group of elements they keep the compiler from hoisting every
// element's arithmetic ahead of the (serial) fp64 accumulation, which would hold two live
// registers per element for the whole tile.
template <typename T>
__device__ __forceinline__ void pin(T &v) {
    asm volatile("" : "+v"(v));
}

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

// ---- global <-> registers, coalesced, full tiles only --------------------------------------------
// Streams that are read once per step are loaded with the non-temporal hint: the lines are not
// kept in the L2 / memory-side cache, which is worth more than 20 % of achieved HBM bandwidth here.
// Optimizer state is read and rewritten in place once per step: non-temporal on *both* the load
// and the store (either alone does nothing) lifts a no-compute kernel with the momentum byte mix
// from 69 % to 86 % of peak.
#ifndef OMC_TUNE_NT_LOADS
#define OMC_TUNE_NT_LOADS 1      // bit 0: gradients / values to compress; bit 1: packed codes (loads and stores)
#endif
#ifndef OMC_TUNE_NT_STATE
#define OMC_TUNE_NT_STATE 1      // optimizer state and decompressed output, loads and stores
#endif
// Cache hints of a work item's in-place streams.  Packed codes are read and rewritten by every step
// and come back from the memory-side cache at the next step if they still sit there: KEEP marks a
// work item whose codes are meant to stay (the host grants this to as many items as fit), the
// others carry the non-temporal hint and stream past.  The conversions (compress / decompress) keep
// the codes cached, as every step after them reads them.  Optimizer state is always non-temporal:
// keeping part of it cached instead was measured to be slower, not faster.
template <int MODE, bool KEEP>
struct StreamHints {
    static constexpr bool nt_codes = (MODE >= kStepSgd) ? !KEEP : (OMC_TUNE_NT_LOADS & 2) != 0;
    static constexpr bool nt_state = OMC_TUNE_NT_STATE != 0;
};

template <bool NT>
__device__ __forceinline__ void load_f32_pieces(const float *__restrict__ src, uint32_t lane, f32x4 (&g)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(src) + (j * 64u + lane);
        g[j] = NT ? __builtin_nontemporal_load(p) : *p;
    }
}

template <bool NT>
__device__ __forceinline__ void store_f32_pieces(float *__restrict__ dst, uint32_t lane, const f32x4 (&g)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        f32x4 *p = reinterpret_cast<f32x4 *>(dst) + (j * 64u + lane);
        if (NT) __builtin_nontemporal_store(g[j], p); else *p = g[j];
    }
}

// coalesced pieces -> each lane's 32 consecutive floats
__device__ __forceinline__ void pieces_to_lanes(const f32x4 (&g)[8], float (&r)[32], uint32_t *lds,
                                                uint32_t lane) {
    f32x4 *l4 = reinterpret_cast<f32x4 *>(lds);
#pragma unroll
    for (int j = 0; j < 8; ++j) l4[piece_slot_flat(j, lane)] = g[j];
    lds_fence();
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        f32x4 t = l4[piece_slot_own(k, lane)];
        r[4 * k + 0] = t.x; r[4 * k + 1] = t.y; r[4 * k + 2] = t.z; r[4 * k + 3] = t.w;
    }
    lds_fence();
}

// each lane's 32 consecutive floats -> coalesced pieces
__device__ __forceinline__ void lanes_to_pieces(const float (&r)[32], f32x4 (&g)[8], uint32_t *lds,
                                                uint32_t lane) {
    f32x4 *l4 = reinterpret_cast<f32x4 *>(lds);
#pragma unroll
    for (int k = 0; k < 8; ++k)
        l4[piece_slot_own(k, lane)] = f32x4{r[4 * k + 0], r[4 * k + 1], r[4 * k + 2], r[4 * k + 3]};
    lds_fence();
#pragma unroll
    for (int j = 0; j < 8; ++j) g[j] = l4[piece_slot_flat(j, lane)];
    lds_fence();
}

// Packed tile as 16-byte pieces: 16*B of them, piece q = 64 j + lane in round j.
template <int B>
struct CodePieces {
    static constexpr int total = 16 * B;
    static constexpr int rounds = (total + 63) / 64;
    __device__ static __forceinline__ bool in_tile(int j, uint32_t q) {
        return (j * 64 + 64 <= total) || q < static_cast<uint32_t>(total);
    }
};

template <int B, bool NT = (OMC_TUNE_NT_LOADS & 2) != 0>
__device__ __forceinline__ void load_code_pieces(const uint32_t *__restrict__ src, uint32_t lane,
                                                 u32x4 (&cq)[CodePieces<B>::rounds]) {
#pragma unroll
    for (int j = 0; j < CodePieces<B>::rounds; ++j) {
        const uint32_t q = j * 64u + lane;
        if (CodePieces<B>::in_tile(j, q))
            cq[j] = NT ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src) + q)
                       : reinterpret_cast<const u32x4 *>(src)[q];
        else
            cq[j] = u32x4{0u, 0u, 0u, 0u};
    }
}

template <int B, bool NT = (OMC_TUNE_NT_LOADS & 2) != 0>
__device__ __forceinline__ void store_code_pieces(uint32_t *__restrict__ dst, uint32_t lane,
                                                  const u32x4 (&cq)[CodePieces<B>::rounds]) {
#pragma unroll
    for (int j = 0; j < CodePieces<B>::rounds; ++j) {
        const uint32_t q = j * 64u + lane;
        if (CodePieces<B>::in_tile(j, q)) {
            if (NT) __builtin_nontemporal_store(cq[j], reinterpret_cast<u32x4 *>(dst) + q);
            else reinterpret_cast<u32x4 *>(dst)[q] = cq[j];
        }
    }
}

// coalesced pieces -> each lane's B consecutive dwords
template <int B>
__device__ __forceinline__ void code_pieces_to_lanes(const u32x4 (&cq)[CodePieces<B>::rounds], uint32_t (&w)[B],
                                                     uint32_t *lds, uint32_t lane) {
#pragma unroll
    for (int j = 0; j < CodePieces<B>::rounds; ++j) {
        const uint32_t q = j * 64u + lane;
        if (CodePieces<B>::in_tile(j, q)) {
            const uint32_t a = CodeLds<B>::flat(4u * q);   // a piece never straddles a spare dword
            lds[a + 0] = cq[j].x; lds[a + 1] = cq[j].y; lds[a + 2] = cq[j].z; lds[a + 3] = cq[j].w;
        }
    }
    lds_fence();
    const uint32_t base = CodeLds<B>::lane_base(lane);
#pragma unroll
    for (int j = 0; j < B; ++j) w[j] = lds[base + j];
    lds_fence();
}

// each lane's B consecutive dwords -> coalesced pieces
template <int B>
__device__ __forceinline__ void lanes_to_code_pieces(const uint32_t (&o)[B], u32x4 (&cq)[CodePieces<B>::rounds],
                                                     uint32_t *lds, uint32_t lane) {
    const uint32_t base = CodeLds<B>::lane_base(lane);
#pragma unroll
    for (int j = 0; j < B; ++j) lds[base + j] = o[j];
    lds_fence();
#pragma unroll
    for (int j = 0; j < CodePieces<B>::rounds; ++j) {
        const uint32_t q = j * 64u + lane;
        if (CodePieces<B>::in_tile(j, q)) {
            const uint32_t a = CodeLds<B>::flat(4u * q);
            cq[j] = u32x4{lds[a + 0], lds[a + 1], lds[a + 2], lds[a + 3]};
        } else {
            cq[j] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    lds_fence();
}

// Byte-multiple code widths (B = 8 k): a lane that owns the four consecutive elements of each of its
// eight 16-byte fp32 pieces (elements 256 j + 4 lane ..) owns whole dwords of the packed tile too,
// k of them per piece: tile dwords k (64 j + lane) + h, h < k, in the lane-local order j k + h that the
// element loops expect.  The fp32 streams then need no transposition at all; the codes still pass
// through LDS, so that their global accesses stay 16 bytes per lane.
template <int B>
__device__ __forceinline__ void code_pieces_to_strided_lanes(const u32x4 (&cq)[CodePieces<B>::rounds], uint32_t (&w)[B],
                                                             uint32_t *lds, uint32_t lane) {
    constexpr uint32_t k = B / 8;
    u32x4 *l4 = reinterpret_cast<u32x4 *>(lds);
#pragma unroll
    for (int r = 0; r < CodePieces<B>::rounds; ++r) l4[r * 64u + lane] = cq[r];   // rounds * 64 == 16 B pieces exactly
    lds_fence();
#pragma unroll
    for (uint32_t j = 0; j < 8; ++j)
#pragma unroll
        for (uint32_t h = 0; h < k; ++h) w[j * k + h] = lds[k * (64u * j + lane) + h];
    lds_fence();
}

template <int B>
__device__ __forceinline__ void strided_lanes_to_code_pieces(const uint32_t (&o)[B], u32x4 (&cq)[CodePieces<B>::rounds],
                                                             uint32_t *lds, uint32_t lane) {
    constexpr uint32_t k = B / 8;
#pragma unroll
    for (uint32_t j = 0; j < 8; ++j)
#pragma unroll
        for (uint32_t h = 0; h < k; ++h) lds[k * (64u * j + lane) + h] = o[j * k + h];
    lds_fence();
    const u32x4 *l4 = reinterpret_cast<const u32x4 *>(lds);
#pragma unroll
    for (int r = 0; r < CodePieces<B>::rounds; ++r) cq[r] = l4[r * 64u + lane];
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
template <bool WIDE>
__device__ __forceinline__ void encode(float x, const FmtParams &fp, uint32_t &code, float &tq) {
    const uint32_t xb = __float_as_uint(x);
    // |x| clamped to the largest magnitude, compared as integers so that Inf and NaN saturate too
    const uint32_t ab = min(xb & 0x7fffffffu, __float_as_uint(fp.maxval));
    const float a = __uint_as_float(ab);
    const uint32_t exb = max(ab, fp.min_norm_bits) & 0x7f800000u;  // binade of a, at least the first normal one
    float r;
    if (WIDE) {
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
// Unevaluated sum hi + lo of two doubles, and the additions that keep one (Knuth's two-sum for the
// error of an addition; used by the wide-mantissa kernels and by the finalize).
struct DD {
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
// s += x with the rounding error of the addition added to l
__device__ __forceinline__ void sum_with_error(double &s, double &l, double x) {
    const double t = s + x;
    const double bb = t - s;
    const double e = (s - (t - bb)) + (x - bb);
    s = t;
    l += e;
}

// The four sums of Sec. 2.3 over the elements a lane has seen.  Every term is exact in fp64 (an fp32
// value, or the product of two).  EXACT = false: plain fp64 additions; a lane adds 32 to 128 terms and
// their rounding errors stay some 2^-50 of the sums, which moves the fp32 result of the closed form only
// when that result lies within ~1e-16 of a rounding boundary -- as long as b is a visible fraction of
// the values, i.e. for formats of fewer than 16 mantissa bits.  EXACT = true (16 mantissa bits and more,
// where b = (SUM V - s SUM Vt) / n cancels to ~2^-M of the values): every addition's error is kept in a
// second word (lV ..), so that sum + error carries about 106 bits and its rounding to fp64 is the
// correctly rounded sum, as the definition of the fit asks for.
struct FitAcc {
    double sV, sT, sVT, sTT;
    double lV, lT, lVT, lTT;
    uint32_t t0;     // bit pattern of the first decompressed value this lane saw
    uint32_t diff;   // OR of (bits ^ t0) over all values this lane saw
    bool have;
    __device__ __forceinline__ void clear() {
        sV = sT = sVT = sTT = 0.0;
        lV = lT = lVT = lTT = 0.0;
        t0 = 0u;
        diff = 0u;
        have = false;
    }
    template <bool EXACT = false>
    __device__ __forceinline__ void add(float x, float tq) {
        const double dx = static_cast<double>(x), dt = static_cast<double>(tq);
        if constexpr (EXACT) {
            sum_with_error(sV, lV, dx);
            sum_with_error(sT, lT, dt);
            sum_with_error(sVT, lVT, dx * dt);   // the product of two fp32 values is exact in fp64
            sum_with_error(sTT, lTT, dt * dt);
        } else {
            sV += dx;
            sT += dt;
            sVT = fma(dx, dt, sVT);              // one rounding: the product itself is exact
            sTT = fma(dt, dt, sTT);
        }
        diff |= __float_as_uint(tq) ^ t0;
    }
    template <bool EXACT = false>
    __device__ __forceinline__ void pin_sums() {
        asm volatile("" : "+v"(sV), "+v"(sT), "+v"(sVT), "+v"(sTT), "+v"(diff));
        if constexpr (EXACT) asm volatile("" : "+v"(lV), "+v"(lT), "+v"(lVT), "+v"(lTT));
    }
    __device__ __forceinline__ void seed(float tq) {   // before the first add
        if (!have) t0 = __float_as_uint(tq);
        have = true;
    }
    // Range of the decompressed values as (min, max): exact when all of the lane's values are
    // equal (+0 and -0 count as equal), otherwise (-inf, +inf), which is all the fit needs.
    __device__ __forceinline__ void lane_range(float &tmin, float &tmax) const {
        const float inf = __builtin_huge_valf();
        if (!have) { tmin = inf; tmax = -inf; return; }
        const bool equal = diff == 0u || (diff == 0x80000000u && (t0 & 0x7fffffffu) == 0u);
        tmin = equal ? __uint_as_float(t0) : -inf;
        tmax = equal ? __uint_as_float(t0) : inf;
    }
    // butterfly over the 64 lanes; every lane ends with the same totals, in an order that does
    // not depend on scheduling; lane 0 stores them
    template <bool EXACT = false>
    __device__ __forceinline__ void reduce_and_store(Partial *out) {
        float tmin, tmax;
        lane_range(tmin, tmax);
        if constexpr (EXACT) {
            DD dV{sV, lV}, dT{sT, lT}, dVT{sVT, lVT}, dTT{sTT, lTT};
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                dV = dd_add(dV, dd_shfl_xor(dV, off));
                dT = dd_add(dT, dd_shfl_xor(dT, off));
                dVT = dd_add(dVT, dd_shfl_xor(dVT, off));
                dTT = dd_add(dTT, dd_shfl_xor(dTT, off));
                tmin = fminf(tmin, __shfl_xor(tmin, off));
                tmax = fmaxf(tmax, __shfl_xor(tmax, off));
            }
            sV = dV.hi; lV = dV.lo; sT = dT.hi; lT = dT.lo; sVT = dVT.hi; lVT = dVT.lo; sTT = dTT.hi; lTT = dTT.lo;
        } else {
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
        if ((threadIdx.x & 63u) == 0) {
            Partial p;
            p.sV = sV; p.sT = sT; p.sVT = sVT; p.sTT = sTT;
            p.lV = EXACT ? lV : 0.0; p.lT = EXACT ? lT : 0.0; p.lVT = EXACT ? lVT : 0.0; p.lTT = EXACT ? lTT : 0.0;
            p.tmin = tmin; p.tmax = tmax; p.pad[0] = p.pad[1] = 0;
            *out = p;
        }
    }
};

// ---- one variable as the kernels see it ---------------------------------------------------------------
struct TileArgs {
    uint32_t *codes;          // variable's packed stream
    uint64_t total_dwords;    // its length in dwords
    const float *vin;         // kCompress: values to compress
    float *vout;              // kDecompress: output
    const float *grad;        // step modes
    float *st0, *st1;         // step modes
    float s, b;               // transformation in force for decoding
    uint64_t n;
};

// Registers that receive a tile's global loads (coalesced layout).
template <int B, int MODE>
struct Stage {
    u32x4 cq[CodePieces<B>::rounds];
    f32x4 gq[8], mq[8], vq[8];
};

template <int B, int MODE, bool KEEP>
__device__ __forceinline__ void issue_loads(const TileArgs &a, uint64_t e0, uint32_t lane, Stage<B, MODE> &st) {
    const uint64_t dw0 = (e0 >> 5) * B;                   // first dword of the tile
    constexpr bool nt_codes = StreamHints<MODE, KEEP>::nt_codes, nt_state = StreamHints<MODE, KEEP>::nt_state;
    if (MODE != kCompress) load_code_pieces<B, nt_codes>(a.codes + dw0, lane, st.cq);
    constexpr bool nt_in = (OMC_TUNE_NT_LOADS & 1) != 0;
    if (MODE == kCompress) load_f32_pieces<nt_in>(a.vin + e0, lane, st.gq);
    if (MODE >= kStepSgd) load_f32_pieces<nt_in>(a.grad + e0, lane, st.gq);
    if (MODE >= kStepMomentum) load_f32_pieces<nt_state>(a.st0 + e0, lane, st.mq);
    if (MODE == kStepAdam) load_f32_pieces<nt_state>(a.st1 + e0, lane, st.vq);
}

// The cycle over a lane's 32 elements, generic formats: decode -> transform -> update -> round ->
// pack, and the fit's sums.  w: the lane's B code dwords; rg / rm / rv: gradient (or the values to
// compress) and optimizer state, updated in place; o: the lane's B output dwords.
template <int B, int MODE, bool WIDE, bool EXACT = false>
__device__ __forceinline__ void cycle_generic(const TileArgs &a, const FmtParams &fp, const OptConst &oc,
                                              uint32_t (&w)[B], float (&rg)[32], float (&rm)[32], float (&rv)[32],
                                              uint32_t (&o)[B], FitAcc &acc) {
#pragma unroll
    for (int j = 0; j < B; ++j) o[j] = 0u;
#pragma unroll
    for (int i = 0; i < kLaneElems; ++i) {
#if OMC_TUNE_SCHED_GROUP > 0
        if (i % OMC_TUNE_SCHED_GROUP == 0) {              // group start: pin the group's inputs
            constexpr int G = OMC_TUNE_SCHED_GROUP;
            if (MODE != kCompress) {
#pragma unroll
                for (int j = (i * B) >> 5; j <= (((i + G) * B - 1) >> 5); ++j) pin(w[j]);
            }
            if (MODE != kDecompress) {
#pragma unroll
                for (int e = i; e < i + G; ++e) pin(rg[e]);
            }
            if (MODE >= kStepMomentum) {
#pragma unroll
                for (int e = i; e < i + G; ++e) pin(rm[e]);
            }
            if (MODE == kStepAdam) {
#pragma unroll
                for (int e = i; e < i + G; ++e) pin(rv[e]);
            }
        }
#endif
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
        uint32_t code;
        float tq;
        encode<WIDE>(x, fp, code, tq);
        pack_at<B>(o, i, code);
        if (i == 0) acc.seed(tq);
        acc.template add<EXACT>(x, tq);
#if OMC_TUNE_SCHED_GROUP > 0
        if ((i + 1) % OMC_TUNE_SCHED_GROUP == 0) {        // group end: pin what the group produced
            constexpr int G = OMC_TUNE_SCHED_GROUP;
            pin(acc.sV); pin(acc.sT); pin(acc.sVT); pin(acc.sTT); pin(acc.diff);
            if constexpr (EXACT) { pin(acc.lV); pin(acc.lT); pin(acc.lVT); pin(acc.lTT); }
            pin(o[((i + 1) * B - 1) >> 5]);
            if (MODE >= kStepMomentum) {
#pragma unroll
                for (int e = i + 1 - G; e <= i; ++e) pin(rm[e]);
            }
            if (MODE == kStepAdam) {
#pragma unroll
                for (int e = i + 1 - G; e <= i; ++e) pin(rv[e]);
            }
        }
#endif
    }
}

// gfx950 OCP FP8 (E4M3) conversions; the selectors must be literal constants for the builtins, the
// switches below fold away once the surrounding loops are unrolled.
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float fp8_to_f32(int w, int byte) {
    switch (byte) {
        case 0: return __builtin_amdgcn_cvt_f32_fp8(w, 0);
        case 1: return __builtin_amdgcn_cvt_f32_fp8(w, 1);
        case 2: return __builtin_amdgcn_cvt_f32_fp8(w, 2);
        default: return __builtin_amdgcn_cvt_f32_fp8(w, 3);
    }
}
__device__ __forceinline__ int f32x2_to_fp8_half(float x0, float x1, int old, int half) {
    return half ? __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, old, true) : __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, old, false);
}
__device__ __forceinline__ f32x2 fp8_half_to_f32x2(int w, int half) {
    return half ? __builtin_amdgcn_cvt_pk_f32_fp8(w, true) : __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
}

// The same cycle for S1E4M3 with bias 7.  That format is OCP FP8 E4M3 in every code but the top
// one (0x7F / 0xFF: 480 here, NaN there), and gfx950 converts OCP FP8 in hardware: one
// instruction decodes a byte, one rounds and packs two values (nearest even, gradual underflow;
// without saturation every overflow yields exactly the top code, which is also what this format
// wants), one decodes two codes back for the fit.  13 vector instructions per element instead
// of 30.  What the hardware cannot give is the *value* of a top code: it reads back as NaN, and a
// NaN input picks a different sign bit.  Both cases leave a NaN in the lane's sums, so the caller
// checks for that and redoes such a tile with cycle_generic.  Returns false when a redo is needed.
// New optimizer state goes to rm / rv only when the result is good.
template <int MODE>
__device__ __forceinline__ bool cycle_ocp_e4m3(const TileArgs &a, const OptConst &oc, uint32_t (&w)[8],
                                               float (&rg)[32], float (&rm)[32], float (&rv)[32],
                                               uint32_t (&o)[8], FitAcc &acc) {
    const FitAcc saved = acc;
    float nm[32], nv[32];
#pragma unroll
    for (int j = 0; j < 8; ++j) {                          // one code dword = 4 elements
        pin(w[j]);
#pragma unroll
        for (int e = 4 * j; e < 4 * j + 4; ++e) {
            if (MODE != kDecompress) pin(rg[e]);
            if (MODE >= kStepMomentum) pin(rm[e]);
            if (MODE == kStepAdam) pin(rv[e]);
        }
        int packed = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {                      // one 16-bit half = 2 elements
            float x[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int i = 4 * j + 2 * h + q;
                if (MODE != kCompress) {
                    const float vt = fp8_to_f32(static_cast<int>(w[j]), 2 * h + q);
                    const float sv = a.s * vt;
                    x[q] = sv + a.b;
                } else {
                    x[q] = rg[i];
                }
                if (MODE >= kStepSgd) {
                    float m = MODE >= kStepMomentum ? rm[i] : 0.0f, v = MODE == kStepAdam ? rv[i] : 0.0f;
                    x[q] = apply_update<MODE>(x[q], rg[i], m, v, oc);
                    if (MODE >= kStepMomentum) nm[i] = m;
                    if (MODE == kStepAdam) nv[i] = v;
                }
            }
            packed = f32x2_to_fp8_half(x[0], x[1], packed, h);
            const f32x2 t = fp8_half_to_f32x2(packed, h);
            if (j == 0 && h == 0) acc.seed(t.x);
            acc.add(x[0], t.x);
            acc.add(x[1], t.y);
        }
        o[j] = static_cast<uint32_t>(packed);
        pin(acc.sV); pin(acc.sT); pin(acc.sVT); pin(acc.sTT); pin(acc.diff);
        pin(o[j]);
    }
    const bool bad = (acc.sV != acc.sV) || (acc.sT != acc.sT);
    if (__any(bad)) {
        acc = saved;
        return false;
    }
    if (MODE >= kStepMomentum) {
#pragma unroll
        for (int i = 0; i < 32; ++i) rm[i] = nm[i];
    }
    if (MODE == kStepAdam) {
#pragma unroll
        for (int i = 0; i < 32; ++i) rv[i] = nv[i];
    }
    return true;
}

// The same cycle for S1E2M3 with bias 1.  That format is the 6-bit E2M3 element type of the OCP
// microscaling formats, code for code (no Inf / NaN codes, gradual underflow, saturating
// nearest-even conversion), and gfx950 converts 32 such elements per lane in one instruction in
// each direction, with exactly this library's packing (element k in bits [6k, 6k+6) of six
// dwords): one instruction decodes the lane's tile, one rounds and packs it (its two 16-float
// operands interleave: even elements, odd elements), one more decodes the new codes for the fit.
// Probed against the oracle: identical for every code and position, every tie, subnormal and
// overflow, and for +-Inf; only a NaN input is not covered (sign handling), and a NaN leaves a NaN in
// the lane's sums, so such a tile is redone with cycle_generic.  Returns false when a redo is needed.
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x32 __attribute__((ext_vector_type(32)));
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
template <int MODE>
__device__ __forceinline__ bool cycle_mx_fp6(const TileArgs &a, const OptConst &oc, uint32_t (&w)[6],
                                             float (&rg)[32], float (&rm)[32], float (&rv)[32],
                                             uint32_t (&o)[6], FitAcc &acc) {
    const FitAcc saved = acc;
    float nm[32], nv[32];
    f32x16 xe, xo;                                         // new values: even and odd elements
    if (MODE != kCompress) {
        const u32x6 cw = {w[0], w[1], w[2], w[3], w[4], w[5]};
        const f32x32 vt = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(cw, 1.0f);
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const float sv = a.s * vt[i];
            float x = sv + a.b;
            if (MODE >= kStepSgd) {
                float m = MODE >= kStepMomentum ? rm[i] : 0.0f, v = MODE == kStepAdam ? rv[i] : 0.0f;
                x = apply_update<MODE>(x, rg[i], m, v, oc);
                if (MODE >= kStepMomentum) nm[i] = m;
                if (MODE == kStepAdam) nv[i] = v;
            }
            if (i & 1) xo[i >> 1] = x; else xe[i >> 1] = x;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            if (i & 1) xo[i >> 1] = rg[i]; else xe[i >> 1] = rg[i];
        }
    }
    const u32x6 nw = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(xe, xo, 1.0f);
    const f32x32 tq = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(nw, 1.0f);
    acc.seed(tq[0]);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        acc.add((i & 1) ? xo[i >> 1] : xe[i >> 1], tq[i]);
        if (i % 4 == 3) { pin(acc.sV); pin(acc.sT); pin(acc.sVT); pin(acc.sTT); pin(acc.diff); }
    }
    const bool bad = (acc.sV != acc.sV);
    if (__any(bad)) {
        acc = saved;
        return false;
    }
#pragma unroll
    for (int j = 0; j < 6; ++j) o[j] = nw[j];
    if (MODE >= kStepMomentum) {
#pragma unroll
        for (int i = 0; i < 32; ++i) rm[i] = nm[i];
    }
    if (MODE == kStepAdam) {
#pragma unroll
        for (int i = 0; i < 32; ++i) rv[i] = nv[i];
    }
    return true;
}

// Everything after the loads of the full tile at e0 have been issued into `st`.  When PREFETCH,
// the loads of the next tile are issued into the same registers as soon as they are free, so
// that they are in flight while this tile is computed.
template <int B, int MODE, int VARIANT, bool PREFETCH, bool KEEP>
__device__ __forceinline__ void finish_tile(const TileArgs &a, const FmtParams &fp, const OptConst &oc,
                                            uint64_t e0, uint32_t lane, uint32_t *lds, Stage<B, MODE> &st,
                                            FitAcc &acc) {
    // hand every lane its 32 elements: consecutive ones, or (byte-multiple code widths) the four
    // consecutive elements of each of its eight 16-byte pieces, which the fp32 loads delivered already
    constexpr bool kDirect = Tuning<MODE, B>::direct;
    uint32_t w[B];
    float rg[32], rm[32], rv[32];
    if constexpr (kDirect) {
        if (MODE != kCompress) code_pieces_to_strided_lanes<B>(st.cq, w, lds, lane);
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (MODE == kCompress || MODE >= kStepSgd) rg[4 * j + i] = st.gq[j][i];
                if (MODE >= kStepMomentum) rm[4 * j + i] = st.mq[j][i];
                if (MODE == kStepAdam) rv[4 * j + i] = st.vq[j][i];
            }
    } else {
        if (MODE != kCompress) code_pieces_to_lanes<B>(st.cq, w, lds, lane);
        if (MODE == kCompress || MODE >= kStepSgd) pieces_to_lanes(st.gq, rg, lds, lane);
        if (MODE >= kStepMomentum) pieces_to_lanes(st.mq, rm, lds, lane);
        if (MODE == kStepAdam) pieces_to_lanes(st.vq, rv, lds, lane);
    }

    if (PREFETCH) issue_loads<B, MODE, KEEP>(a, e0 + kTileElems, lane, st);

    uint32_t o[B];
    if constexpr (VARIANT == 2 && B == 8 && MODE != kDecompress) {
        if (!cycle_ocp_e4m3<MODE>(a, oc, w, rg, rm, rv, o, acc))
            cycle_generic<B, MODE, false>(a, fp, oc, w, rg, rm, rv, o, acc);
    } else if constexpr (VARIANT == 3 && B == 6 && MODE != kDecompress) {
        if (!cycle_mx_fp6<MODE>(a, oc, w, rg, rm, rv, o, acc))
            cycle_generic<B, MODE, false>(a, fp, oc, w, rg, rm, rv, o, acc);
    } else {
        cycle_generic<B, MODE, variant_wide(VARIANT), variant_exact(VARIANT)>(a, fp, oc, w, rg, rm, rv, o, acc);
    }

    // back to the coalesced layouts and out
    auto to_pieces = [&](const float (&r)[32], f32x4 (&out)[8]) {
        if constexpr (kDirect) {
#pragma unroll
            for (int j = 0; j < 8; ++j) out[j] = f32x4{r[4 * j + 0], r[4 * j + 1], r[4 * j + 2], r[4 * j + 3]};
        } else {
            lanes_to_pieces(r, out, lds, lane);
        }
    };
    if (MODE == kDecompress) {
        f32x4 out[8];
        to_pieces(rg, out);
        store_f32_pieces<OMC_TUNE_NT_STATE != 0>(a.vout + e0, lane, out);
        return;
    }
    if (MODE >= kStepMomentum) {
        f32x4 out[8];
        to_pieces(rm, out);
        store_f32_pieces<StreamHints<MODE, KEEP>::nt_state>(a.st0 + e0, lane, out);
    }
    if (MODE == kStepAdam) {
        f32x4 out[8];
        to_pieces(rv, out);
        store_f32_pieces<StreamHints<MODE, KEEP>::nt_state>(a.st1 + e0, lane, out);
    }
    u32x4 cout[CodePieces<B>::rounds];
    if constexpr (kDirect) strided_lanes_to_code_pieces<B>(o, cout, lds, lane);
    else lanes_to_code_pieces<B>(o, cout, lds, lane);
    store_code_pieces<B, StreamHints<MODE, KEEP>::nt_codes>(a.codes + (e0 >> 5) * B, lane, cout);
}

// One work item of the full-tile kernels: tiles [chunk * tiles, (chunk + 1) * tiles) of one variable, as far
// as full tiles go, reduced into one Partial.  The caller guarantees at least one full tile.  `tiles` is
// tiles_per_chunk(B) for the work items of a plan; the single-variable calls pass a larger number for huge
// variables, so that the finalize has at most a few thousand partial sums to add.
template <int B, int MODE, int VARIANT, bool KEEP = true>
__device__ __forceinline__ void do_chunk(const TileArgs &a, const FmtParams &fp, const OptConst &oc,
                                         uint32_t chunk, uint32_t *lds, Partial *partial_out,
                                         uint32_t tiles = tiles_per_chunk(B)) {
    const uint32_t lane = threadIdx.x;
    FitAcc acc;
    acc.clear();
    const uint64_t first_tile = static_cast<uint64_t>(chunk) * tiles;
    const uint64_t full_tiles = a.n / kTileElems;
    const uint32_t ntiles = static_cast<uint32_t>((full_tiles - first_tile < tiles) ? full_tiles - first_tile : tiles);
    const uint64_t begin = first_tile * kTileElems;
    Stage<B, MODE> st;
    issue_loads<B, MODE, KEEP>(a, begin, lane, st);
    for (uint32_t t = 0; t + 1 < ntiles; ++t) {
        const uint64_t e0 = begin + static_cast<uint64_t>(t) * kTileElems;
        finish_tile<B, MODE, VARIANT, Tuning<MODE, B>::prefetch, KEEP>(a, fp, oc, e0, lane, lds, st, acc);
        if (!Tuning<MODE, B>::prefetch) issue_loads<B, MODE, KEEP>(a, e0 + kTileElems, lane, st);
    }
    finish_tile<B, MODE, VARIANT, false, KEEP>(a, fp, oc, begin + static_cast<uint64_t>(ntiles - 1) * kTileElems,
                                               lane, lds, st, acc);
    if (MODE != kDecompress) acc.template reduce_and_store<variant_exact(VARIANT)>(partial_out);
}

// ---- the ragged tail of a variable ----------------------------------------------------------------------
// Elements [e0, n) with e0 a multiple of 2048 and n - e0 < 2048, by one wave.  Same ownership as
// a full tile (lane l: elements e0 + 32 l ...), same arithmetic, but the code width is a run-time
// value, every access is bounds-checked and goes straight to global memory.  Lanes past the end
// write zero bits up to the end of the (16-byte padded) packed buffer.  The sums of the fit are kept
// with their rounding errors for the formats whose full-tile kernels do so (fp.variant).
template <int MODE, bool WIDE>
__device__ __forceinline__ void do_tail(const TileArgs &a, const FmtParams &fp, const OptConst &oc,
                                        Partial *partial_out) {
    const uint32_t lane = threadIdx.x;
    const uint32_t B = fp.bits;
    const uint64_t e0 = (a.n / kTileElems) * kTileElems;
    const uint64_t lane_e0 = e0 + static_cast<uint64_t>(lane) * kLaneElems;
    const uint64_t lane_dw0 = (lane_e0 >> 5) * B;            // the lane's first dword
    const uint32_t cmask = (B == 32) ? 0xffffffffu : ((1u << B) - 1u);
    const bool exact = variant_exact(fp.variant);
    FitAcc acc;
    acc.clear();
    uint64_t outbits = 0;
    uint32_t fill = 0, outidx = 0;
    for (uint32_t i = 0; i < kLaneElems; ++i) {
        const uint64_t e = lane_e0 + i;
        const bool live = e < a.n;
        float x;
        if (MODE != kCompress) {
            const uint32_t bit = i * B, idx = bit >> 5, off = bit & 31u;
            const uint64_t d = lane_dw0 + idx;
            const uint32_t lo = (d < a.total_dwords) ? a.codes[d] : 0u;
            const uint32_t hi = (idx + 1 < B && d + 1 < a.total_dwords) ? a.codes[d + 1] : 0u;
            const uint64_t both = (static_cast<uint64_t>(hi) << 32) | lo;
            const uint32_t code = static_cast<uint32_t>(both >> off) & cmask;
            const float vt = decode_top(code << (32u - B), fp);
            const float sv = a.s * vt;
            x = sv + a.b;
        } else {
            x = live ? a.vin[e] : 0.0f;
        }
        if (MODE == kDecompress) {
            if (live) a.vout[e] = x;
            continue;
        }
        if (MODE >= kStepSgd) {
            float g = live ? a.grad[e] : 0.0f;
            float m = (MODE >= kStepMomentum && live) ? a.st0[e] : 0.0f;
            float v = (MODE == kStepAdam && live) ? a.st1[e] : 0.0f;
            x = apply_update<MODE>(x, g, m, v, oc);
            if (MODE >= kStepMomentum && live) a.st0[e] = m;
            if (MODE == kStepAdam && live) a.st1[e] = v;
        }
        if (!live) x = 0.0f;                                  // padding elements pack as zero bits
        uint32_t code;
        float tq;
        encode<WIDE>(x, fp, code, tq);
        if (live) {
            acc.seed(tq);
            if (exact) acc.add<true>(x, tq); else acc.add<false>(x, tq);
        }
        outbits |= static_cast<uint64_t>(code) << fill;
        fill += B;
        if (fill >= 32u) {                                    // one more dword of the lane is complete
            const uint64_t d = lane_dw0 + outidx;
            if (d < a.total_dwords) a.codes[d] = static_cast<uint32_t>(outbits);
            outbits >>= 32;
            fill -= 32u;
            ++outidx;
        }
    }
    if (MODE != kDecompress) {
        if (exact) acc.reduce_and_store<true>(partial_out); else acc.reduce_and_store<false>(partial_out);
    }
}

// ---- finalize: per-variable (s, b) from the partials (paper Sec. 2.3) -----------------------------
// Called by a whole workgroup of NW waves (blockDim.x == 64 * NW).  Sums the variable's partials
// (a run of `nparts` from the full-tile kernels and, if `tail` is not null, one more from the tail
// kernel) with compensated additions in an order fixed by (nparts, NW) alone: thread t takes
// partials t, t + 64 NW, ...; lanes combine by a butterfly; waves combine in index order.  Then the
// closed form in fp64, stored as fp32.  `red` is LDS scratch of NW * 10 doubles.  `exact`: the partials
// carry error words (formats of 16 or more mantissa bits), which are added as well.
template <int NW>
__device__ __forceinline__ void finalize_variable(const Partial *__restrict__ parts, uint32_t nparts,
                                                  const Partial *__restrict__ tail, uint64_t n, bool use_pvt,
                                                  bool exact, float *sb_out, double *red) {
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    if (!use_pvt) {
        if (tid == 0) { sb_out[0] = 1.0f; sb_out[1] = 0.0f; }
        return;
    }
    DD sV{0, 0}, sT{0, 0}, sVT{0, 0}, sTT{0, 0};
    float tmin = __builtin_huge_valf(), tmax = -__builtin_huge_valf();
    bool finite = true;
    const uint32_t total = nparts + (tail ? 1u : 0u);
    // a lane's partials are fetched eight at a time before they are added (same order of additions; the
    // loads of a batch are in flight together instead of one memory round trip per partial)
    constexpr uint32_t kBatch = 8, kStride = 64 * NW;
    for (uint32_t i0 = tid; i0 < total; i0 += kBatch * kStride) {
        Partial p[kBatch];
#pragma unroll
        for (uint32_t u = 0; u < kBatch; ++u) {
            const uint32_t i = i0 + u * kStride;
            if (i < total) p[u] = (i < nparts) ? parts[i] : *tail;
        }
#pragma unroll
        for (uint32_t u = 0; u < kBatch; ++u) {
            if (i0 + u * kStride >= total) break;
            finite = finite && isfinite(p[u].sV);
            if (finite) {
                sV = dd_add(sV, p[u].sV);
                sT = dd_add(sT, p[u].sT);
                sVT = dd_add(sVT, p[u].sVT);
                sTT = dd_add(sTT, p[u].sTT);
                if (exact) {                        // the error words of the wide-mantissa kernels (zero otherwise)
                    sV = dd_add(sV, p[u].lV);
                    sT = dd_add(sT, p[u].lT);
                    sVT = dd_add(sVT, p[u].lVT);
                    sTT = dd_add(sTT, p[u].lTT);
                }
            }
            tmin = fminf(tmin, p[u].tmin);
            tmax = fmaxf(tmax, p[u].tmax);
        }
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
    if (NW > 1) {
        if (lane == 0) {
            double *r = red + wave * 10;
            r[0] = sV.hi; r[1] = sV.lo; r[2] = sT.hi; r[3] = sT.lo; r[4] = sVT.hi; r[5] = sVT.lo;
            r[6] = sTT.hi; r[7] = sTT.lo;
            r[8] = static_cast<double>(tmin);
            r[9] = finite ? static_cast<double>(tmax) : __builtin_nan("");   // NaN marks a poisoned wave
        }
        __syncthreads();
        if (tid != 0) return;
        for (int w = 1; w < NW; ++w) {
            const double *r = red + w * 10;
            sV = dd_add(sV, DD{r[0], r[1]});
            sT = dd_add(sT, DD{r[2], r[3]});
            sVT = dd_add(sVT, DD{r[4], r[5]});
            sTT = dd_add(sTT, DD{r[6], r[7]});
            tmin = fminf(tmin, static_cast<float>(r[8]));
            if (r[9] != r[9]) finite = false; else tmax = fmaxf(tmax, static_cast<float>(r[9]));
        }
    } else if (tid != 0) {
        return;
    }
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

// One workgroup of NW waves per variable: new (s, b) of every quantized variable of a plan.
template <int NW>
__global__ __launch_bounds__(64 * NW) void finalize_plan_kernel(const uint8_t *__restrict__ plan, uint64_t var_off,
                                                                const Partial *__restrict__ ws,
                                                                float *__restrict__ sb_table) {
    __shared__ double red[NW * 10];
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(plan + var_off);
    const PlanVar pv = to_scalar_regs(vars[blockIdx.x]);
    if (!(pv.flags & OMC_VAR_QUANTIZED)) return;
    finalize_variable<NW>(pv.nitems ? ws + pv.first_item : ws, pv.nitems,
                          pv.tail_item != kNoItem ? ws + pv.tail_item : nullptr, pv.n,
                          !(pv.flags & OMC_VAR_NO_PVT), variant_exact(pv.fp.variant), sb_table + 2 * static_cast<uint64_t>(pv.sb_index), red);
}
constexpr int kFinalizeWaves = 4;

// ---- dispatch over the code width ---------------------------------------------------------------------
#define OMC_FOR_EACH_BITS(X)                                                                       \
    X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17) X(18)  \
    X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30) X(31) X(32)

}  // namespace omc
