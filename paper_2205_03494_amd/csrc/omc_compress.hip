// omc_compress / omc_compress_set: fp32 values -> packed codes + partial sums of the fit, then (s, b).
#include <mutex>

#include "omc_codec_impl.h"

namespace omc {

template <int NW>
__global__ __launch_bounds__(64 * NW) void finalize_single_kernel(const Partial *__restrict__ ws, uint32_t nparts,
                                                                  int has_tail, uint64_t n, int use_pvt, int exact,
                                                                  float *__restrict__ sb) {
    __shared__ double red[NW * 10];
    finalize_variable<NW>(ws, nparts, has_tail ? ws + nparts : nullptr, n, use_pvt != 0, exact != 0, sb, red);
}

// Variants 0 / 1 (add-subtract or ldexp rounding) and, for code widths that can hold 16 mantissa bits,
// 4 / 5 (the same with error-carrying sums).
template <int BITS>
static void launch_generic_variant(uint32_t variant, uint32_t grid, const CodecArgs &ca, hipStream_t st) {
    if constexpr (BITS >= 18) {
        if (variant == 4) { codec_kernel<BITS, kCompress, 4><<<dim3(grid), dim3(64), 0, st>>>(ca); return; }
        if (variant == 5) { codec_kernel<BITS, kCompress, 5><<<dim3(grid), dim3(64), 0, st>>>(ca); return; }
    }
    if (variant == 1) codec_kernel<BITS, kCompress, 1><<<dim3(grid), dim3(64), 0, st>>>(ca);
    else codec_kernel<BITS, kCompress, 0><<<dim3(grid), dim3(64), 0, st>>>(ca);
}

// One full-tile launch: `grid` workgroups of the kernel for (bits, variant).
static int launch_full(uint32_t bits, uint32_t variant, uint32_t grid, const CodecArgs &ca, hipStream_t st) {
    if (bits == 8 && variant == 2) {
        codec_kernel<8, kCompress, 2><<<dim3(grid), dim3(64), 0, st>>>(ca);
        return static_cast<int>(hipGetLastError());
    }
    if (bits == 6 && variant == 3) {
        codec_kernel<6, kCompress, 3><<<dim3(grid), dim3(64), 0, st>>>(ca);
        return static_cast<int>(hipGetLastError());
    }
    switch (bits) {
#define X(BITS)                                                                                  \
    case BITS:                                                                                   \
        launch_generic_variant<BITS>(variant, grid, ca, st);                                     \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

static int launch_tail(bool wide, uint32_t grid, const CodecArgs &ca, hipStream_t st) {
    if (wide) codec_tail_kernel<kCompress, true><<<dim3(grid), dim3(64), 0, st>>>(ca);
    else codec_tail_kernel<kCompress, false><<<dim3(grid), dim3(64), 0, st>>>(ca);
    return static_cast<int>(hipGetLastError());
}

// Full tiles per work item of a single variable: the plan's figure, doubled until at most kMaxSingleItems work
// items are left (a 64 M-element variable: 2048 items of 16 tiles), so that all of them are resident at once and the
// finalize adds a few thousand partial sums at most.  Depends on the size alone.
uint32_t single_tiles_per_item(uint32_t bits, uint64_t n) {
#ifndef OMC_TUNE_SINGLE_ITEMS
#define OMC_TUNE_SINGLE_ITEMS 2048
#endif
    constexpr uint64_t kMaxSingleItems = OMC_TUNE_SINGLE_ITEMS;
    const uint64_t full_tiles = n / kTileElems;
    uint64_t tiles = tiles_per_chunk(bits);
    if ((full_tiles + tiles - 1) / tiles > kMaxSingleItems) tiles = (full_tiles + kMaxSingleItems - 1) / kMaxSingleItems;
    return static_cast<uint32_t>(tiles);
}

int launch_compress(const float *v, const VarArgs &va, int use_pvt, void *codes, float *sb, Partial *ws,
                    void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t tiles = single_tiles_per_item(va.fp.bits, va.n);
    const uint32_t nchunks = static_cast<uint32_t>((va.n / kTileElems + tiles - 1) / tiles);
    const bool has_tail = (va.n % kTileElems) != 0;
    CodecArgs ca{};
    ca.arena = static_cast<uint8_t *>(codes);
    ca.single.n = va.n;
    ca.single.total_dwords = va.total_dwords;
    ca.single.fp = va.fp;
    ca.single_tiles = tiles;
    ca.single_tail = has_tail ? 1u : 0u;
    ca.vin = v;
    ca.ws = ws;
    ca.nitems = nchunks + (has_tail ? 1u : 0u);            // the ragged tail is the launch's last workgroup
    int rc = launch_full(va.fp.bits, va.fp.variant, ca.nitems, ca, st);
    if (rc != 0) return rc;
    // the width of the reduction depends on the size alone, so results do not depend on the run
    const int exact = variant_exact(va.fp.variant) ? 1 : 0;
    if (nchunks <= 256)
        finalize_single_kernel<1><<<dim3(1), dim3(64), 0, st>>>(ws, nchunks, has_tail ? 1 : 0, va.n, use_pvt, exact, sb);
    else
        finalize_single_kernel<4><<<dim3(1), dim3(256), 0, st>>>(ws, nchunks, has_tail ? 1 : 0, va.n, use_pvt, exact, sb);
    return static_cast<int>(hipGetLastError());
}

// ---- a workspace that nobody has to allocate ------------------------------------------------------
// omc_compress_noalloc serves callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid it): the partial sums of the fit go to this
// file-scope device array instead of a caller's workspace.  Every GPU the library runs on holds its
// own copy of the array, at its own address, until the process ends.  In host code the array's name
// is only a handle for the runtime's symbol lookup, not a device address: the address is asked for
// once per device (that device current) and all host-side uses go through the pointer kept here.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices] = {nullptr};    // per device: address of that device's copy of `scratch`
}  // namespace

int static_scratch(void **ptr_out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<int>(e);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return static_cast<int>(e);
        if (!p) return static_cast<int>(hipErrorInvalidSymbol);
        scratch_ptr[dev] = p;
    }
    *ptr_out = scratch_ptr[dev];
    return 0;
}

int launch_compress_set(const float *values, const PlanHeader *ph, const void *plan_dev, void *arena,
                        float *sb_table, Partial *ws, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *ph_bytes = reinterpret_cast<const uint8_t *>(ph);
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(ph_bytes + ph->group_off);
    CodecArgs ca{};
    ca.arena = static_cast<uint8_t *>(arena);
    ca.plan = static_cast<const uint8_t *>(plan_dev);
    ca.var_off = ph->var_off;
    ca.item_off = ph->item_off;
    ca.vin = values;
    ca.ws = ws;
    const PlanGroup *fp32_group = nullptr;
    bool any_full = false;
    for (uint32_t gi = 0; gi < ph->ngroups; ++gi) {
        if (groups[gi].kind == kGroupFp32 && groups[gi].nitems > 0) fp32_group = &groups[gi];
        if (groups[gi].kind == kGroupFull && groups[gi].nitems > 0) any_full = true;
    }
    bool fp32_done = (fp32_group == nullptr);
    for (uint32_t gi = 0; gi < ph->ngroups; ++gi) {
        const PlanGroup &g = groups[gi];
        if (g.nitems == 0 || g.kind == kGroupFp32) continue;
        ca.first_item = g.first_item;
        ca.nitems = g.nitems;
        ca.fp32_first = 0;
        ca.fp32_nitems = 0;
        int rc;
        if (g.kind == kGroupFull) {
            if (!fp32_done) {                          // the fp32 copies ride along with the first full-tile launch
                ca.fp32_first = fp32_group->first_item;
                ca.fp32_nitems = fp32_group->nitems;
                fp32_done = true;
            }
            rc = launch_full(g.bits, g.wide, g.nitems + ca.fp32_nitems, ca, st);
        } else {
            rc = launch_tail(g.wide != 0, g.nitems, ca, st);
        }
        if (rc != 0) return rc;
    }
    if (!fp32_done) {                                  // no full-tile launch to ride on: a launch of copies alone
        (void)any_full;
        ca.first_item = 0;
        ca.nitems = 0;
        ca.fp32_first = fp32_group->first_item;
        ca.fp32_nitems = fp32_group->nitems;
        codec_kernel<8, kCompress, 0><<<dim3(fp32_group->nitems), dim3(64), 0, st>>>(ca);
        const int rc = static_cast<int>(hipGetLastError());
        if (rc != 0) return rc;
    }
    if (ph->nquant > 0) {
        finalize_plan_kernel<kFinalizeWaves><<<dim3(ph->nvars), dim3(64 * kFinalizeWaves), 0, st>>>(
            ca.plan, ph->var_off, ws, sb_table);
        return static_cast<int>(hipGetLastError());
    }
    return 0;
}

}  // namespace omc
