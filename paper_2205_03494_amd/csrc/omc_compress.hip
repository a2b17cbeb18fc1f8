// omc_compress: fp32 variable -> packed codes + partial sums of the fit, then (s, b).
#include "omc_stream.h"

namespace omc {

template <int B>
__global__ __launch_bounds__(64) void compress_kernel(const float *__restrict__ v, uint32_t *__restrict__ codes,
                                                      VarArgs va, Partial *__restrict__ ws) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    TileArgs a{};
    a.codes = codes;
    a.total_dwords = va.total_dwords;
    a.vin = v;
    a.n = va.n;
    a.s = 1.0f;
    a.b = 0.0f;
    OptConst oc{};
    do_chunk<B, kCompress>(a, va.fp, oc, blockIdx.x, lds, ws + blockIdx.x);
}

__global__ __launch_bounds__(64) void finalize_single_kernel(const Partial *__restrict__ ws, uint32_t nparts,
                                                             uint64_t n, int use_pvt, float *__restrict__ sb) {
    finalize_variable(ws, nparts, n, use_pvt != 0, sb);
}

int launch_compress(const float *v, const VarArgs &va, int use_pvt, void *codes, float *sb, Partial *ws,
                    void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t nchunks = static_cast<uint32_t>((va.n + kChunkElems - 1) / kChunkElems);
    switch (va.fp.bits) {
#define X(BITS)                                                                                     \
    case BITS:                                                                                      \
        compress_kernel<BITS><<<dim3(nchunks), dim3(64), 0, st>>>(v, static_cast<uint32_t *>(codes), va, ws); \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return static_cast<int>(e);
    finalize_single_kernel<<<dim3(1), dim3(64), 0, st>>>(ws, nchunks, va.n, use_pvt, sb);
    return static_cast<int>(hipGetLastError());
}

}  // namespace omc
