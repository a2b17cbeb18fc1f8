// omc_compress: fp32 variable -> packed codes + partial sums of the fit, then (s, b).
#include "omc_stream.h"

namespace omc {

template <int B, int VARIANT>
__global__ __launch_bounds__(64, (Tuning<kCompress, B>::waves)) void compress_kernel(
    const float *__restrict__ v, uint32_t *__restrict__ codes, VarArgs va, Partial *__restrict__ ws) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kLdsDwords];
    TileArgs a{};
    a.codes = codes;
    a.total_dwords = va.total_dwords;
    a.vin = v;
    a.n = va.n;
    a.s = 1.0f;
    a.b = 0.0f;
    OptConst oc{};
    do_chunk<B, kCompress, VARIANT>(a, va.fp, oc, blockIdx.x, lds, ws + blockIdx.x);
}

template <bool WIDE>
__global__ __launch_bounds__(64) void compress_tail_kernel(const float *__restrict__ v, uint32_t *__restrict__ codes,
                                                           VarArgs va, Partial *__restrict__ tail_partial) {
    TileArgs a{};
    a.codes = codes;
    a.total_dwords = va.total_dwords;
    a.vin = v;
    a.n = va.n;
    a.s = 1.0f;
    a.b = 0.0f;
    OptConst oc{};
    do_tail<kCompress, WIDE>(a, va.fp, oc, tail_partial);
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void finalize_single_kernel(const Partial *__restrict__ ws, uint32_t nparts,
                                                                  int has_tail, uint64_t n, int use_pvt,
                                                                  float *__restrict__ sb) {
    __shared__ double red[NW * 10];
    finalize_variable<NW>(ws, nparts, has_tail ? ws + nparts : nullptr, n, use_pvt != 0, sb, red);
}

int launch_compress(const float *v, const VarArgs &va, int use_pvt, void *codes, float *sb, Partial *ws,
                    void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t nchunks = static_cast<uint32_t>((va.n / kTileElems + kTilesPerChunk - 1) / kTilesPerChunk);
    const bool has_tail = (va.n % kTileElems) != 0;
    uint32_t *c = static_cast<uint32_t *>(codes);
    if (nchunks > 0 && va.fp.variant == 2) {
        compress_kernel<8, 2><<<dim3(nchunks), dim3(64), 0, st>>>(v, c, va, ws);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    } else if (nchunks > 0) {
        switch (va.fp.bits) {
#define X(BITS)                                                                                 \
    case BITS:                                                                                  \
        if (va.fp.variant == 1) compress_kernel<BITS, 1><<<dim3(nchunks), dim3(64), 0, st>>>(v, c, va, ws); \
        else compress_kernel<BITS, 0><<<dim3(nchunks), dim3(64), 0, st>>>(v, c, va, ws);        \
        break;
            OMC_FOR_EACH_BITS(X)
#undef X
            default:
                return static_cast<int>(hipErrorInvalidValue);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    if (has_tail) {
        if (va.fp.wide) compress_tail_kernel<true><<<dim3(1), dim3(64), 0, st>>>(v, c, va, ws + nchunks);
        else compress_tail_kernel<false><<<dim3(1), dim3(64), 0, st>>>(v, c, va, ws + nchunks);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return static_cast<int>(e);
    }
    // the width of the reduction depends on the size alone, so results do not depend on the run
    if (nchunks <= 256)
        finalize_single_kernel<1><<<dim3(1), dim3(64), 0, st>>>(ws, nchunks, has_tail ? 1 : 0, va.n, use_pvt, sb);
    else
        finalize_single_kernel<16><<<dim3(1), dim3(1024), 0, st>>>(ws, nchunks, has_tail ? 1 : 0, va.n, use_pvt, sb);
    return static_cast<int>(hipGetLastError());
}

}  // namespace omc
