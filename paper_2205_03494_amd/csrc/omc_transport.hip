// Device side of omc_transport_pack (paper Sec. 1: parameters are kept and transported in compressed
// form) and the (s, b) bookkeeping of omc_reselect (Sec. 2.5).  Pure data movement: no arithmetic of the
// method happens here.
#include "omc_stream.h"

namespace omc {

constexpr int kMetaThreads = 256;

// One workgroup: walks the plan's variable table in order, gives every variable its 16-byte aligned place
// in the payload (a running sum of the sizes), writes the message's variable table and (s, b) table, and
// finally the header with the checksum over both.
__global__ __launch_bounds__(kMetaThreads) void transport_meta_kernel(const uint8_t *__restrict__ plan, uint64_t var_off,
                                                                       const float *__restrict__ sb_table,
                                                                       uint8_t *__restrict__ msg, TransportHeader th) {
    __shared__ uint64_t scan[kMetaThreads];
    __shared__ uint64_t carry;
    const uint32_t tid = threadIdx.x;
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(plan + var_off);
    TransportVar *out = reinterpret_cast<TransportVar *>(msg + sizeof(TransportHeader));
    float *sb_out = reinterpret_cast<float *>(msg + th.sb_off);
    if (tid == 0) carry = 0;
    __syncthreads();
    uint64_t hash_sum = 0;
    for (uint32_t base = 0; base < th.nvars; base += kMetaThreads) {
        const uint32_t i = base + tid;
        uint64_t bytes = 0;
        PlanVar pv{};
        if (i < th.nvars) {
            pv = vars[i];
            bytes = (pv.flags & OMC_VAR_QUANTIZED) ? pv.total_dwords * 4 : (4 * pv.n + 15) / 16 * 16;
        }
        scan[tid] = bytes;
        __syncthreads();
        for (int off = 1; off < kMetaThreads; off <<= 1) {       // inclusive scan of the sizes
            const uint64_t add = tid >= static_cast<uint32_t>(off) ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += add;
            __syncthreads();
        }
        if (i < th.nvars) {
            TransportVar tv;
            tv.payload_offset = carry + scan[tid] - bytes;
            tv.aux_offset = pv.aux_offset;
            tv.n = pv.n;
            const bool q = (pv.flags & OMC_VAR_QUANTIZED) != 0;
            tv.exp_bits = q ? static_cast<uint8_t>(pv.fp.exp_bits) : 8;
            tv.man_bits = q ? static_cast<uint8_t>(pv.fp.man_bits) : 23;
            tv.exp_bias = q ? static_cast<int16_t>(pv.fp.bias) : 127;
            tv.flags = pv.flags;
            out[i] = tv;
            hash_sum += transport_var_hash(i, tv);
            sb_out[2 * static_cast<uint64_t>(i)] = q ? sb_table[2 * static_cast<uint64_t>(pv.sb_index)] : 1.0f;
            sb_out[2 * static_cast<uint64_t>(i) + 1] = q ? sb_table[2 * static_cast<uint64_t>(pv.sb_index) + 1] : 0.0f;
        }
        __syncthreads();
        if (tid == kMetaThreads - 1) carry += scan[tid];
        __syncthreads();
    }
    scan[tid] = hash_sum;
    __syncthreads();
    for (int off = kMetaThreads / 2; off >= 1; off >>= 1) {
        if (tid < static_cast<uint32_t>(off)) scan[tid] += scan[tid + off];
        __syncthreads();
    }
    if (tid == 0) {
        th.checksum = transport_header_hash(th, scan[0]);
        *reinterpret_cast<TransportHeader *>(msg) = th;
    }
}

// Workgroup (i, y) copies runs of 1024 16-byte pieces, y, y + gridDim.y, ..., of variable i from the arena to
// the place the meta kernel gave it (read back from the message's own table).
constexpr uint32_t kPackSlices = 64;
__global__ __launch_bounds__(256) void transport_pack_kernel(const uint8_t *__restrict__ plan, uint64_t var_off,
                                                             const uint8_t *__restrict__ arena, uint8_t *__restrict__ msg,
                                                             uint64_t payload_off) {
    const PlanVar *vars = reinterpret_cast<const PlanVar *>(plan + var_off);
    const uint32_t i = blockIdx.x;
    const PlanVar pv = to_scalar_regs(vars[i]);
    const TransportVar *tvs = reinterpret_cast<const TransportVar *>(msg + sizeof(TransportHeader));
    const uint64_t dst_off = to_scalar_regs(tvs[i].payload_offset);
    const bool q = (pv.flags & OMC_VAR_QUANTIZED) != 0;
    const uint64_t bytes = q ? pv.total_dwords * 4 : 4 * pv.n;
    const uint64_t full = bytes / 16;
    const u32x4 *src = reinterpret_cast<const u32x4 *>(arena + pv.data_offset);
    u32x4 *dst = reinterpret_cast<u32x4 *>(msg + payload_off + dst_off);
    // four pieces per thread in flight; a slice's run of 4 * 256 pieces is contiguous
    constexpr uint32_t kBatch = 4;
    for (uint64_t p0 = static_cast<uint64_t>(blockIdx.y) * (256 * kBatch); p0 < full; p0 += 256ull * kBatch * gridDim.y) {
        u32x4 x[kBatch];
#pragma unroll
        for (uint32_t u = 0; u < kBatch; ++u) {
            const uint64_t p = p0 + u * 256 + threadIdx.x;
            if (p < full) x[u] = __builtin_nontemporal_load(src + p);
        }
#pragma unroll
        for (uint32_t u = 0; u < kBatch; ++u) {
            const uint64_t p = p0 + u * 256 + threadIdx.x;
            if (p < full) __builtin_nontemporal_store(x[u], dst + p);
        }
    }
    if (blockIdx.y == 0 && threadIdx.x == 0 && bytes % 16) {      // an fp32 variable whose size is no multiple of four
        const uint32_t *s = reinterpret_cast<const uint32_t *>(src + full);
        uint32_t *d = reinterpret_cast<uint32_t *>(dst + full);
        const uint32_t left = static_cast<uint32_t>(bytes % 16) / 4;
        for (uint32_t k = 0; k < 4; ++k) d[k] = k < left ? s[k] : 0u;
    }
}

int launch_transport_pack(const PlanHeader *ph, const void *plan_dev, const void *arena, const float *sb_table,
                          void *msg_dev, const TransportHeader &th, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    transport_meta_kernel<<<dim3(1), dim3(kMetaThreads), 0, st>>>(static_cast<const uint8_t *>(plan_dev), ph->var_off, sb_table,
                                                                  static_cast<uint8_t *>(msg_dev), th);
    int rc = static_cast<int>(hipGetLastError());
    if (rc != 0) return rc;
    transport_pack_kernel<<<dim3(ph->nvars, kPackSlices), dim3(256), 0, st>>>(
        static_cast<const uint8_t *>(plan_dev), ph->var_off, static_cast<const uint8_t *>(arena),
        static_cast<uint8_t *>(msg_dev), th.payload_off);
    return static_cast<int>(hipGetLastError());
}

// (s, b) of the variables that omc_reselect only moves: copied for those that stay quantized, (1, 0) for
// those that are fp32 afterwards; the entries of newly quantized variables are written by their fit.
__global__ __launch_bounds__(256) void reselect_sb_kernel(const uint32_t *__restrict__ actions, uint32_t nvars,
                                                          const float *__restrict__ sb_old, float *__restrict__ sb_new) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= nvars) return;
    const uint32_t a = actions[i];
    if (a == kRsCopyQuantized) {
        sb_new[2 * static_cast<uint64_t>(i)] = sb_old[2 * static_cast<uint64_t>(i)];
        sb_new[2 * static_cast<uint64_t>(i) + 1] = sb_old[2 * static_cast<uint64_t>(i) + 1];
    } else if (a != kRsToQuantized) {
        sb_new[2 * static_cast<uint64_t>(i)] = 1.0f;
        sb_new[2 * static_cast<uint64_t>(i) + 1] = 0.0f;
    }
}

int launch_reselect_sb(const uint32_t *actions_dev, uint32_t nvars, const float *sb_old, float *sb_new, void *stream) {
    reselect_sb_kernel<<<dim3((nvars + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(actions_dev, nvars, sb_old, sb_new);
    return static_cast<int>(hipGetLastError());
}

}  // namespace omc
