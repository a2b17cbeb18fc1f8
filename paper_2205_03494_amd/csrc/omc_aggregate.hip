// omc_aggregate_mean: the server's side of a federated round (paper Sec. 1: the clients' trained
// models come back and are aggregated; Sec. 2.5: every client quantizes its own subset of the
// variables).  out[i] = (v_0[i] + v_1[i] + ... + v_{R-1}[i]) / R over the clients' decompressed
// values, summed in client order in fp32, every operation rounded once.  One pass: each client's
// copy is read once in the form it arrived in (packed codes or fp32), the mean is written once.
#include "omc_stream.h"

#ifndef OMC_TUNE_AGG_NT
#define OMC_TUNE_AGG_NT 1      // the clients' codes are read once per round: non-temporal
#endif

namespace omc {

#ifndef OMC_AGG_WAVES
#define OMC_AGG_WAVES 4
#endif

struct AggArgs {
    const uint8_t *plan;                 // device copy of the aggregation plan blob
    uint64_t var_off, src_off, item_off;
    uint32_t first_item, nitems;
    uint32_t flat_first, flat_nitems;    // items of all-fp32 variables appended to a full-tile launch
    uint32_t nreplicas;
    float count;                         // R as a float
    AggPointers p;
    float *out;
};

// Variables that are fp32 at every client: 16-byte pieces, coalesced, bounds-checked at the end.
__device__ __forceinline__ void aggregate_flat_item(const AggArgs &aa, uint32_t item) {
    const PlanItem it = to_scalar_regs(reinterpret_cast<const PlanItem *>(aa.plan + aa.item_off)[item]);
    const AggVar av = to_scalar_regs(reinterpret_cast<const AggVar *>(aa.plan + aa.var_off)[it.var]);
    const AggSrc *src = reinterpret_cast<const AggSrc *>(aa.plan + aa.src_off) + static_cast<uint64_t>(it.var) * aa.nreplicas;
    const uint32_t lane = threadIdx.x;
    float *dst = aa.out + av.aux_offset;
    const uint64_t begin = static_cast<uint64_t>(it.chunk) * kChunkElems;
    for (int j = 0; j < kChunkElems / 256; ++j) {
        const uint64_t e = begin + (static_cast<uint64_t>(j) * 64 + lane) * 4;
        if (e >= av.n) break;
        const bool full = e + 4 <= av.n;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (uint32_t r = 0; r < aa.nreplicas; ++r) {
            const float *v = reinterpret_cast<const float *>(aa.p.arena[r] + to_scalar_regs(src[r].data_offset));
            float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (full) {
                const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(v + e));
                x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
            } else {
                for (int c = 0; c < 4; ++c)
                    if (e + c < av.n) x[c] = v[e + c];
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = (r == 0) ? x[c] : acc[c] + x[c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = acc[c] / aa.count;
        if (full) {
            __builtin_nontemporal_store(f32x4{acc[0], acc[1], acc[2], acc[3]}, reinterpret_cast<f32x4 *>(dst + e));
        } else {
            for (int c = 0; c < 4; ++c)
                if (e + c < av.n) dst[e + c] = acc[c];
        }
    }
}

// Full tiles of a variable that at least one client quantized (code width B).  A lane owns 32
// consecutive elements; a client's tile reaches that layout through LDS from coalesced 16-byte
// pieces, whether it holds codes or fp32 values.
template <int B>
__global__ __launch_bounds__(64, OMC_AGG_WAVES) void aggregate_kernel(AggArgs aa) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    if (blockIdx.x >= aa.nitems) {
        aggregate_flat_item(aa, aa.flat_first + (blockIdx.x - aa.nitems));
        return;
    }
    const uint32_t lane = threadIdx.x;
    const uint32_t item = aa.first_item + blockIdx.x;
    const PlanItem it = to_scalar_regs(reinterpret_cast<const PlanItem *>(aa.plan + aa.item_off)[item]);
    const AggVar av = to_scalar_regs(reinterpret_cast<const AggVar *>(aa.plan + aa.var_off)[it.var]);
    const AggSrc *src = reinterpret_cast<const AggSrc *>(aa.plan + aa.src_off) + static_cast<uint64_t>(it.var) * aa.nreplicas;
    const FmtParams fp = av.fp;
    const uint64_t first_tile = static_cast<uint64_t>(it.chunk) * tiles_per_chunk(B);
    const uint64_t full_tiles = av.n / kTileElems;
    const uint32_t ntiles = static_cast<uint32_t>(
        (full_tiles - first_tile < tiles_per_chunk(B)) ? full_tiles - first_tile : tiles_per_chunk(B));
    for (uint32_t t = 0; t < ntiles; ++t) {
        const uint64_t e0 = (first_tile + t) * kTileElems;
        float acc[32];
        for (uint32_t r = 0; r < aa.nreplicas; ++r) {
            const AggSrc s = to_scalar_regs(src[r]);
            float val[32];
            if (s.quantized) {
                const uint32_t *codes = reinterpret_cast<const uint32_t *>(aa.p.arena[r] + s.data_offset);
                const float sc = to_scalar_regs(aa.p.sb[r][2 * static_cast<uint64_t>(it.var)]);
                const float of = to_scalar_regs(aa.p.sb[r][2 * static_cast<uint64_t>(it.var) + 1]);
                u32x4 cq[CodePieces<B>::rounds];
                load_code_pieces<B, OMC_TUNE_AGG_NT != 0>(codes + (e0 >> 5) * B, lane, cq);
                uint32_t w[B];
                code_pieces_to_lanes<B>(cq, w, lds, lane);
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const float vt = decode_top(code_at_top<B>(w, i), fp);
                    const float sv = sc * vt;
                    val[i] = sv + of;
                }
            } else {
                const float *v = reinterpret_cast<const float *>(aa.p.arena[r] + s.data_offset);
                f32x4 g[8];
                load_f32_pieces<true>(v + e0, lane, g);
                pieces_to_lanes(g, val, lds, lane);
            }
            if (r == 0) {
#pragma unroll
                for (int i = 0; i < 32; ++i) acc[i] = val[i];
            } else {
#pragma unroll
                for (int i = 0; i < 32; ++i) acc[i] = acc[i] + val[i];
            }
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = acc[i] / aa.count;
        f32x4 o[8];
        lanes_to_pieces(acc, o, lds, lane);
        store_f32_pieces<true>(aa.out + av.aux_offset + e0, lane, o);
    }
}

// Byte codes need no transposition: a lane takes dwords of four codes at the same element offsets as
// its 16-byte pieces of the fp32 copies and of the output (slab of 1024 elements: piece j of lane l =
// elements 256 j + 4 l ..).  Everything stays coalesced and LDS is not used.  S1E4M3 / bias 7 is
// decoded by the hardware's FP8 conversion; its one deviating code (the top code reads as NaN) leaves a
// NaN in the sum, and such a slab is redone with the generic decode.
template <bool HW>
__device__ __forceinline__ void aggregate_byte_slab(const AggArgs &aa, const AggSrc *src, uint32_t var, const FmtParams &fp,
                                                    uint64_t e0, uint32_t lane, f32x4 (&acc)[4]) {
    // (fetching the code dwords of all copies before the first decode, to have more loads in flight,
    // was measured: 499 us instead of 334 us on the benchmark set; one copy at a time it is)
    for (uint32_t r = 0; r < aa.nreplicas; ++r) {
        const AggSrc s = to_scalar_regs(src[r]);
        f32x4 val[4];
        if (s.quantized) {
            const uint32_t *c = reinterpret_cast<const uint32_t *>(aa.p.arena[r] + s.data_offset) + (e0 >> 2);
            const float sc = to_scalar_regs(aa.p.sb[r][2 * static_cast<uint64_t>(var)]);
            const float of = to_scalar_regs(aa.p.sb[r][2 * static_cast<uint64_t>(var) + 1]);
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = OMC_TUNE_AGG_NT ? __builtin_nontemporal_load(c + (64 * j + lane)) : c[64 * j + lane];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float vt[4];
                if (HW) {
                    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(w[j]), false);
                    const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(w[j]), true);
                    vt[0] = lo[0]; vt[1] = lo[1]; vt[2] = hi[0]; vt[3] = hi[1];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) vt[i] = decode_top(w[j] << (24 - 8 * i), fp);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float sv = sc * vt[i];
                    val[j][i] = sv + of;
                }
            }
        } else {
            const f32x4 *v = reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(aa.p.arena[r] + s.data_offset) + e0);
#pragma unroll
            for (int j = 0; j < 4; ++j) val[j] = __builtin_nontemporal_load(v + (64 * j + lane));
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[j][i] = (r == 0) ? val[j][i] : acc[j][i] + val[j][i];
    }
}

__global__ __launch_bounds__(64, 8) void aggregate_byte_kernel(AggArgs aa) {
    if (blockIdx.x >= aa.nitems) {
        aggregate_flat_item(aa, aa.flat_first + (blockIdx.x - aa.nitems));
        return;
    }
    const uint32_t lane = threadIdx.x;
    const uint32_t item = aa.first_item + blockIdx.x;
    const PlanItem it = to_scalar_regs(reinterpret_cast<const PlanItem *>(aa.plan + aa.item_off)[item]);
    const AggVar av = to_scalar_regs(reinterpret_cast<const AggVar *>(aa.plan + aa.var_off)[it.var]);
    const AggSrc *src = reinterpret_cast<const AggSrc *>(aa.plan + aa.src_off) + static_cast<uint64_t>(it.var) * aa.nreplicas;
    const FmtParams fp = av.fp;
    const uint64_t first_tile = static_cast<uint64_t>(it.chunk) * tiles_per_chunk(8);
    const uint64_t full_tiles = av.n / kTileElems;
    const uint32_t ntiles = static_cast<uint32_t>(
        (full_tiles - first_tile < tiles_per_chunk(8)) ? full_tiles - first_tile : tiles_per_chunk(8));
    const bool hw = fp.variant == 2;
    for (uint32_t sl = 0; sl < 2 * ntiles; ++sl) {
        const uint64_t e0 = first_tile * kTileElems + static_cast<uint64_t>(sl) * 1024;
        f32x4 acc[4];
        bool done = false;
        if (hw) {
            aggregate_byte_slab<true>(aa, src, it.var, fp, e0, lane, acc);
            bool bad = false;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) bad = bad || (acc[j][i] != acc[j][i]);
            done = !__any(bad);
        }
        if (!done) aggregate_byte_slab<false>(aa, src, it.var, fp, e0, lane, acc);
        f32x4 *dst = reinterpret_cast<f32x4 *>(aa.out + av.aux_offset + e0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = acc[j][i] / aa.count;
            __builtin_nontemporal_store(o, dst + (64 * j + lane));
        }
    }
}

// Ragged tails of those variables: one wave each, run-time code width, every access checked.
__global__ __launch_bounds__(64) void aggregate_tail_kernel(AggArgs aa) {
    const uint32_t lane = threadIdx.x;
    const uint32_t item = aa.first_item + blockIdx.x;
    const PlanItem it = to_scalar_regs(reinterpret_cast<const PlanItem *>(aa.plan + aa.item_off)[item]);
    const AggVar av = to_scalar_regs(reinterpret_cast<const AggVar *>(aa.plan + aa.var_off)[it.var]);
    const AggSrc *src = reinterpret_cast<const AggSrc *>(aa.plan + aa.src_off) + static_cast<uint64_t>(it.var) * aa.nreplicas;
    const FmtParams fp = av.fp;
    const uint32_t B = fp.bits;
    const uint32_t cmask = (B == 32) ? 0xffffffffu : ((1u << B) - 1u);
    const uint64_t e0 = (av.n / kTileElems) * kTileElems;
    const uint64_t lane_e0 = e0 + static_cast<uint64_t>(lane) * kLaneElems;
    const uint64_t lane_dw0 = (lane_e0 >> 5) * B;
    for (uint32_t i = 0; i < kLaneElems; ++i) {
        const uint64_t e = lane_e0 + i;
        if (e >= av.n) break;
        float acc = 0.0f;
        for (uint32_t r = 0; r < aa.nreplicas; ++r) {
            const AggSrc s = to_scalar_regs(src[r]);
            float x;
            if (s.quantized) {
                const uint32_t *codes = reinterpret_cast<const uint32_t *>(aa.p.arena[r] + s.data_offset);
                const uint32_t bit = i * B, idx = bit >> 5, off = bit & 31u;
                const uint64_t d = lane_dw0 + idx;
                const uint32_t lo = (d < av.total_dwords) ? codes[d] : 0u;
                const uint32_t hi = (idx + 1 < B && d + 1 < av.total_dwords) ? codes[d + 1] : 0u;
                const uint64_t both = (static_cast<uint64_t>(hi) << 32) | lo;
                const uint32_t code = static_cast<uint32_t>(both >> off) & cmask;
                const float vt = decode_top(code << (32u - B), fp);
                const float sv = aa.p.sb[r][2 * static_cast<uint64_t>(it.var)] * vt;
                x = sv + aa.p.sb[r][2 * static_cast<uint64_t>(it.var) + 1];
            } else {
                x = reinterpret_cast<const float *>(aa.p.arena[r] + s.data_offset)[e];
            }
            acc = (r == 0) ? x : acc + x;
        }
        aa.out[av.aux_offset + e] = acc / aa.count;
    }
}

// flat items alone (no full-tile launch to ride on)
__global__ __launch_bounds__(64) void aggregate_flat_kernel(AggArgs aa) {
    aggregate_flat_item(aa, aa.flat_first + blockIdx.x);
}

int launch_aggregate_mean(const AggHeader *ah, const void *agg_dev, const AggPointers &ptrs, float *out,
                          void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(reinterpret_cast<const uint8_t *>(ah) + ah->group_off);
    AggArgs aa{};
    aa.plan = static_cast<const uint8_t *>(agg_dev);
    aa.var_off = ah->var_off;
    aa.src_off = ah->src_off;
    aa.item_off = ah->item_off;
    aa.nreplicas = ah->nreplicas;
    aa.count = static_cast<float>(ah->nreplicas);
    aa.p = ptrs;
    aa.out = out;
    const PlanGroup *flat = nullptr;
    for (uint32_t gi = 0; gi < ah->ngroups; ++gi)
        if (groups[gi].kind == kGroupFp32 && groups[gi].nitems > 0) flat = &groups[gi];
    bool flat_done = (flat == nullptr);
    for (uint32_t gi = 0; gi < ah->ngroups; ++gi) {
        const PlanGroup &g = groups[gi];
        if (g.nitems == 0 || g.kind == kGroupFp32) continue;
        aa.first_item = g.first_item;
        aa.nitems = g.nitems;
        aa.flat_first = 0;
        aa.flat_nitems = 0;
        if (g.kind == kGroupTail) {
            aggregate_tail_kernel<<<dim3(g.nitems), dim3(64), 0, st>>>(aa);
        } else {
            if (!flat_done) {
                aa.flat_first = flat->first_item;
                aa.flat_nitems = flat->nitems;
                flat_done = true;
            }
            const dim3 grid(g.nitems + aa.flat_nitems);
            if (g.bits == 8) {
                aggregate_byte_kernel<<<grid, dim3(64), 0, st>>>(aa);
                const hipError_t e8 = hipGetLastError();
                if (e8 != hipSuccess) return static_cast<int>(e8);
                continue;
            }
            switch (g.bits) {
#define X(BITS) case BITS: aggregate_kernel<BITS><<<grid, dim3(64), 0, st>>>(aa); break;
                OMC_FOR_EACH_BITS(X)
#undef X
                default: return static_cast<int>(hipErrorInvalidValue);
            }
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    if (!flat_done) {
        aa.flat_first = flat->first_item;
        aa.flat_nitems = flat->nitems;
        aggregate_flat_kernel<<<dim3(flat->nitems), dim3(64), 0, st>>>(aa);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    return 0;
}

}  // namespace omc
