// omc_decompress / omc_decompress_set: packed codes + (s, b) -> fp32.
#include "omc_codec_impl.h"

namespace omc {

static int launch_full(uint32_t bits, uint32_t grid, const CodecArgs &ca, hipStream_t st) {
    switch (bits) {
#define X(BITS)                                                                       \
    case BITS:                                                                        \
        codec_kernel<BITS, kDecompress, 0><<<dim3(grid), dim3(64), 0, st>>>(ca);      \
        break;
        OMC_FOR_EACH_BITS(X)
#undef X
        default:
            return static_cast<int>(hipErrorInvalidValue);
    }
    return static_cast<int>(hipGetLastError());
}

int launch_decompress(const void *codes, const VarArgs &va, const float *sb, float *out, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t tiles = single_tiles_per_item(va.fp.bits, va.n);
    const uint32_t nchunks = static_cast<uint32_t>((va.n / kTileElems + tiles - 1) / tiles);
    const bool has_tail = (va.n % kTileElems) != 0;
    CodecArgs ca{};
    ca.arena = static_cast<uint8_t *>(const_cast<void *>(codes));   // never written in this mode
    ca.single.n = va.n;
    ca.single.total_dwords = va.total_dwords;
    ca.single.fp = va.fp;
    ca.single_tiles = tiles;
    ca.single_tail = has_tail ? 1u : 0u;
    ca.sb_in = sb;
    ca.vout = out;
    ca.nitems = nchunks + (has_tail ? 1u : 0u);            // the ragged tail is the launch's last workgroup
    return launch_full(va.fp.bits, ca.nitems, ca, st);
}

int launch_decompress_set(const void *arena, const PlanHeader *ph, const void *plan_dev, const float *sb_table,
                          float *out, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint8_t *ph_bytes = reinterpret_cast<const uint8_t *>(ph);
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(ph_bytes + ph->group_off);
    CodecArgs ca{};
    ca.arena = static_cast<uint8_t *>(const_cast<void *>(arena));
    ca.plan = static_cast<const uint8_t *>(plan_dev);
    ca.var_off = ph->var_off;
    ca.item_off = ph->item_off;
    ca.sb_in = sb_table;
    ca.vout = out;
    const PlanGroup *fp32_group = nullptr;
    for (uint32_t gi = 0; gi < ph->ngroups; ++gi)
        if (groups[gi].kind == kGroupFp32 && groups[gi].nitems > 0) fp32_group = &groups[gi];
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
            if (!fp32_done) {
                ca.fp32_first = fp32_group->first_item;
                ca.fp32_nitems = fp32_group->nitems;
                fp32_done = true;
            }
            rc = launch_full(g.bits, g.nitems + ca.fp32_nitems, ca, st);
        } else {
            codec_tail_kernel<kDecompress, false><<<dim3(g.nitems), dim3(64), 0, st>>>(ca);
            rc = static_cast<int>(hipGetLastError());
        }
        if (rc != 0) return rc;
    }
    if (!fp32_done) {
        ca.first_item = 0;
        ca.nitems = 0;
        ca.fp32_first = fp32_group->first_item;
        ca.fp32_nitems = fp32_group->nitems;
        codec_kernel<8, kDecompress, 0><<<dim3(fp32_group->nitems), dim3(64), 0, st>>>(ca);
        return static_cast<int>(hipGetLastError());
    }
    return 0;
}

}  // namespace omc
