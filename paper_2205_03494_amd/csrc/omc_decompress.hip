// omc_decompress: packed codes + (s, b) -> fp32.
#include "omc_stream.h"

namespace omc {

template <int B>
__global__ __launch_bounds__(64, (Tuning<kDecompress, B>::waves)) void decompress_kernel(
    const uint32_t *__restrict__ codes, VarArgs va, const float *__restrict__ sb, float *__restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    TileArgs a{};
    a.codes = const_cast<uint32_t *>(codes);   // never written in this mode
    a.total_dwords = va.total_dwords;
    a.vout = out;
    a.n = va.n;
    a.s = sb ? to_scalar_regs(sb[0]) : 1.0f;
    a.b = sb ? to_scalar_regs(sb[1]) : 0.0f;
    OptConst oc{};
    do_chunk<B, kDecompress, 0>(a, va.fp, oc, blockIdx.x, lds, nullptr);
}

__global__ __launch_bounds__(64) void decompress_tail_kernel(const uint32_t *__restrict__ codes, VarArgs va,
                                                             const float *__restrict__ sb, float *__restrict__ out) {
    TileArgs a{};
    a.codes = const_cast<uint32_t *>(codes);
    a.total_dwords = va.total_dwords;
    a.vout = out;
    a.n = va.n;
    a.s = sb ? to_scalar_regs(sb[0]) : 1.0f;
    a.b = sb ? to_scalar_regs(sb[1]) : 0.0f;
    OptConst oc{};
    do_tail<kDecompress, false>(a, va.fp, oc, nullptr);
}

int launch_decompress(const void *codes, const VarArgs &va, const float *sb, float *out, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t nchunks = static_cast<uint32_t>((va.n / kTileElems + kTilesPerChunk - 1) / kTilesPerChunk);
    const uint32_t *c = static_cast<const uint32_t *>(codes);
    if (nchunks > 0) {
        switch (va.fp.bits) {
#define X(BITS)                                                                        \
    case BITS:                                                                         \
        decompress_kernel<BITS><<<dim3(nchunks), dim3(64), 0, st>>>(c, va, sb, out);   \
        break;
            OMC_FOR_EACH_BITS(X)
#undef X
            default:
                return static_cast<int>(hipErrorInvalidValue);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    if (va.n % kTileElems) {
        decompress_tail_kernel<<<dim3(1), dim3(64), 0, st>>>(c, va, sb, out);
        return static_cast<int>(hipGetLastError());
    }
    return 0;
}

}  // namespace omc
