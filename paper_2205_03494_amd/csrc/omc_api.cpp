// Host side of libomc: format constants, plan construction, argument validation, and the
// extern "C" entry points.  No device code here; launches live in the .hip files.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "omc_internal.h"

namespace omc {

static int resolved_bias(omc_format f) {
    return f.exp_bias == OMC_BIAS_DEFAULT ? (1 << (f.exp_bits - 1)) - 1 : f.exp_bias;
}

static bool format_ok(omc_format f) {
    if (f.exp_bits < 1 || f.exp_bits > 8) return false;
    if (f.man_bits > 23) return false;
    if (f.exp_bias != OMC_BIAS_DEFAULT && (f.exp_bias < 0 || f.exp_bias > 127)) return false;
    return true;
}

// largest exponent field whose binade lies inside finite fp32
static int top_field(omc_format f) {
    const int bias = resolved_bias(f);
    int top = (1 << f.exp_bits) - 1;
    if (top - bias > 127) top = 127 + bias;
    return top;
}

bool make_fmt_params(omc_format f, FmtParams *out) {
    if (!format_ok(f)) return false;
    const int E = f.exp_bits, M = f.man_bits, bias = resolved_bias(f);
    FmtParams p{};
    p.bits = 1 + E + M;
    p.exp_bits = E;
    p.man_bits = M;
    p.bias = bias;
    p.sh = 23 - M;
    p.asr = 8 - E;
    p.keep_mask = 0x80000000u | (((1u << (E + M)) - 1u) << p.sh);
    p.min_norm_bits = static_cast<uint32_t>(127 + 1 - bias) << 23;
    p.magic_off = static_cast<uint32_t>(23 - M) << 23;
    const int top_exp = top_field(f) - bias;
    p.wide = (M == 23 || top_exp + 23 - M > 127) ? 1u : 0u;
    p.variant = (E == 4 && M == 3 && bias == 7) ? 2u : (E == 2 && M == 3 && bias == 1) ? 3u : p.wide;
    if (M >= 16) p.variant += kVariantExact;   // the fit's sums carry their rounding errors along
    p.exp_adj = 127 + M;
    p.dec_scale = std::ldexp(1.0f, 127 - bias);
    p.enc_scale = std::ldexp(1.0f, bias - 127);
    p.maxval = static_cast<float>(std::ldexp(2.0 - std::ldexp(1.0, -M), top_exp));
    *out = p;
    return true;
}

static size_t packed_bytes_u(uint32_t bits, uint64_t n) {
    const uint64_t total_bits = n * bits;
    const uint64_t bytes = (total_bits + 7) / 8;
    return static_cast<size_t>((bytes + 15) / 16 * 16);
}

constexpr uint64_t kMaxElems = 1ull << 36;

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// 64-bit checksum of the plan body (everything after the header), eight bytes at a time in four
// independent lanes so that it runs at memory speed: every entry point verifies it.
static uint64_t body_checksum(const uint8_t *p, uint64_t nbytes) {
    uint64_t h[4] = {0x9e3779b97f4a7c15ull, 0xc2b2ae3d27d4eb4full, 0x165667b19e3779f9ull, 0x27d4eb2f165667c5ull};
    const uint64_t nwords = nbytes / 8;
    uint64_t i = 0;
    for (; i + 4 <= nwords; i += 4)
        for (int l = 0; l < 4; ++l) {
            uint64_t w;
            std::memcpy(&w, p + 8 * (i + l), 8);
            h[l] = (h[l] ^ w) * 0x100000001b3ull;
            h[l] = (h[l] << 29) | (h[l] >> 35);
        }
    for (; i < nwords; ++i) {
        uint64_t w;
        std::memcpy(&w, p + 8 * i, 8);
        h[0] = (h[0] ^ w) * 0x100000001b3ull;
        h[0] = (h[0] << 29) | (h[0] >> 35);
    }
    uint64_t tail = 0;
    std::memcpy(&tail, p + 8 * nwords, nbytes - 8 * nwords);
    uint64_t r = (h[0] ^ tail) * 0x100000001b3ull;
    for (int l = 1; l < 4; ++l) r = ((r << 31) | (r >> 33)) ^ (h[l] * 0x9e3779b97f4a7c15ull);
    return r ^ nbytes;
}

// Header consistency, checksum of the body, and bounds of everything the host reads from the body
// (the launch groups).  The item and variable tables are what the checksum vouches for: the builder
// wrote them from a validated variable table.
const PlanHeader *plan_check(const void *plan_host) {
    if (!plan_host) return nullptr;
    const PlanHeader *ph = static_cast<const PlanHeader *>(plan_host);
    if (ph->magic != kPlanMagic || ph->version != kPlanVersion) return nullptr;
    if (ph->nvars == 0 || ph->nitems > 0x7fffffffu || ph->ngroups > kVariants * 33u + 3u) return nullptr;
    if (ph->var_off != sizeof(PlanHeader)) return nullptr;
    if (ph->item_off != ph->var_off + static_cast<uint64_t>(ph->nvars) * sizeof(PlanVar)) return nullptr;
    if (ph->group_off != ph->item_off + static_cast<uint64_t>(ph->nitems) * sizeof(PlanItem)) return nullptr;
    if (ph->total_bytes != align_up(ph->group_off + static_cast<uint64_t>(ph->ngroups) * sizeof(PlanGroup), 16))
        return nullptr;
    if (ph->ws_bytes != std::max<uint64_t>(16, static_cast<uint64_t>(ph->nitems) * sizeof(Partial))) return nullptr;
    const uint8_t *base = static_cast<const uint8_t *>(plan_host);
    if (ph->checksum != body_checksum(base + sizeof(PlanHeader), ph->total_bytes - sizeof(PlanHeader))) return nullptr;
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(base + ph->group_off);
    for (uint32_t g = 0; g < ph->ngroups; ++g) {
        if (groups[g].kind > kGroupFp32) return nullptr;
        if (static_cast<uint64_t>(groups[g].first_item) + groups[g].nitems > ph->nitems) return nullptr;
        if (groups[g].kind == kGroupFull && (groups[g].bits < 2 || groups[g].bits > 32 || groups[g].wide >= kVariants))
            return nullptr;
    }
    return ph;
}

struct PlanLayout {
    uint64_t var_off, item_off, group_off, total;
    uint32_t nitems, ngroups, nquant;
    // launches in order: full-tile kernels by ascending 2*bits + wide, tail kernels (narrow, wide),
    // the fp32 kernel
    std::vector<PlanGroup> groups;
};

// Validates the table; returns OMC_OK and the layout, or the first error.
static omc_status plan_layout(const omc_var *vars, uint32_t nvars, PlanLayout *pl) {
    if (!vars) return OMC_ERR_NULL;
    if (nvars == 0) return OMC_ERR_SIZE;
    bool present[kVariants * 33] = {false};  // kVariants * bits + variant
    bool tails[2] = {false, false};
    bool any_fp32 = false;
    uint64_t nitems = 0;
    uint32_t nquant = 0;
    struct Span { uint64_t lo, hi; };
    std::vector<Span> data(nvars), aux(nvars);
    for (uint32_t i = 0; i < nvars; ++i) {
        const omc_var &v = vars[i];
        if (v.n == 0 || v.n > kMaxElems) return OMC_ERR_SIZE;
        if (v.data_offset % 16 != 0 || v.aux_offset % 4 != 0) return OMC_ERR_ALIGN;
        if (v.flags & ~(OMC_VAR_QUANTIZED | OMC_VAR_NO_PVT)) return OMC_ERR_SIZE;
        uint64_t bytes;
        if (v.flags & OMC_VAR_QUANTIZED) {
            if (!format_ok(v.fmt)) return OMC_ERR_FORMAT;
            const uint32_t bits = 1u + v.fmt.exp_bits + v.fmt.man_bits;
            FmtParams fp;
            make_fmt_params(v.fmt, &fp);
            if (v.n >= kTileElems) present[kVariants * bits + fp.variant] = true;
            if (v.n % kTileElems) tails[fp.wide] = true;
            bytes = packed_bytes_u(bits, v.n);
            ++nquant;
            nitems += (v.n / kTileElems + tiles_per_chunk(bits) - 1) / tiles_per_chunk(bits) + (v.n % kTileElems ? 1 : 0);
        } else {
            any_fp32 = true;
            bytes = 4 * v.n;
            nitems += (v.n + kChunkElems - 1) / kChunkElems;
        }
        data[i] = {v.data_offset, v.data_offset + bytes};
        aux[i] = {v.aux_offset, v.aux_offset + v.n};
    }
    if (nitems > 0x7fffffffull) return OMC_ERR_SIZE;
    auto overlaps = [](std::vector<Span> s) {
        std::sort(s.begin(), s.end(), [](const Span &a, const Span &b) { return a.lo < b.lo; });
        for (size_t i = 1; i < s.size(); ++i)
            if (s[i].lo < s[i - 1].hi) return true;
        return false;
    };
    if (overlaps(data) || overlaps(aux)) return OMC_ERR_SIZE;
    pl->groups.clear();
    for (uint32_t k = 2 * kVariants; k < kVariants * 33; ++k)
        if (present[k]) pl->groups.push_back(PlanGroup{kGroupFull, k / kVariants, k % kVariants, 0, 0, 0});
    for (uint32_t w = 0; w < 2; ++w)
        if (tails[w]) pl->groups.push_back(PlanGroup{kGroupTail, 0, w, 0, 0, 0});
    if (any_fp32) pl->groups.push_back(PlanGroup{kGroupFp32, 0, 0, 0, 0, 0});
    pl->nitems = static_cast<uint32_t>(nitems);
    pl->ngroups = static_cast<uint32_t>(pl->groups.size());
    pl->nquant = nquant;
    pl->var_off = sizeof(PlanHeader);
    pl->item_off = pl->var_off + static_cast<uint64_t>(nvars) * sizeof(PlanVar);
    pl->group_off = pl->item_off + nitems * sizeof(PlanItem);
    pl->total = align_up(pl->group_off + static_cast<uint64_t>(pl->ngroups) * sizeof(PlanGroup), 16);
    return OMC_OK;
}

// Validates the table and writes the plan blob.  sb_index: entry of the (s, b) table per variable, or
// nullptr for the identity (a plan built from a caller's table).
static omc_status build_plan(const omc_var *vars_host, const uint32_t *sb_index, uint32_t nvars, void *plan_host,
                             size_t plan_bytes) {
    if (!plan_host) return OMC_ERR_NULL;
    PlanLayout pl;
    const omc_status st = plan_layout(vars_host, nvars, &pl);
    if (st != OMC_OK) return st;
    if (plan_bytes < pl.total) return OMC_ERR_SIZE;
    uint8_t *base = static_cast<uint8_t *>(plan_host);
    std::memset(base, 0, pl.total);
    PlanHeader *ph = reinterpret_cast<PlanHeader *>(base);
    PlanVar *pv = reinterpret_cast<PlanVar *>(base + pl.var_off);
    PlanItem *items = reinterpret_cast<PlanItem *>(base + pl.item_off);
    PlanGroup *groups = reinterpret_cast<PlanGroup *>(base + pl.group_off);
    uint64_t arena_bytes = 0, aux_elems = 0;
    for (uint32_t i = 0; i < nvars; ++i) {
        const omc_var &v = vars_host[i];
        PlanVar &d = pv[i];
        d.data_offset = v.data_offset;
        d.aux_offset = v.aux_offset;
        d.n = v.n;
        d.flags = v.flags;
        uint64_t bytes;
        if (v.flags & OMC_VAR_QUANTIZED) {
            make_fmt_params(v.fmt, &d.fp);
            bytes = packed_bytes_u(d.fp.bits, v.n);
            d.total_dwords = bytes / 4;
        } else {
            bytes = 4 * v.n;
        }
        d.sb_index = sb_index ? sb_index[i] : i;
        d.first_item = kNoItem;
        d.nitems = 0;
        d.tail_item = kNoItem;
        arena_bytes = std::max(arena_bytes, v.data_offset + bytes);
        aux_elems = std::max(aux_elems, v.aux_offset + v.n);
    }
    uint32_t next = 0;
    for (uint32_t gi = 0; gi < pl.ngroups; ++gi) {
        PlanGroup g = pl.groups[gi];
        g.first_item = next;
        for (uint32_t i = 0; i < nvars; ++i) {
            const omc_var &v = vars_host[i];
            const bool q = (v.flags & OMC_VAR_QUANTIZED) != 0;
            if (g.kind == kGroupFull) {
                if (!q || pv[i].fp.bits != g.bits || pv[i].fp.variant != g.wide || v.n < kTileElems) continue;
                pv[i].first_item = next;
                pv[i].nitems = static_cast<uint32_t>((v.n / kTileElems + tiles_per_chunk(g.bits) - 1) / tiles_per_chunk(g.bits));
                for (uint32_t c = 0; c < pv[i].nitems; ++c) items[next++] = PlanItem{i, c};
            } else if (g.kind == kGroupTail) {
                if (!q || pv[i].fp.wide != g.wide || v.n % kTileElems == 0) continue;
                pv[i].tail_item = next;
                items[next++] = PlanItem{i, 0};
            } else {
                if (q) continue;
                pv[i].first_item = next;
                pv[i].nitems = static_cast<uint32_t>((v.n + kChunkElems - 1) / kChunkElems);
                for (uint32_t c = 0; c < pv[i].nitems; ++c) items[next++] = PlanItem{i, c};
            }
        }
        g.nitems = next - g.first_item;
        groups[gi] = g;
    }
    ph->magic = kPlanMagic;
    ph->version = kPlanVersion;
    ph->nvars = nvars;
    ph->nitems = pl.nitems;
    ph->ngroups = pl.ngroups;
    ph->nquant = pl.nquant;
    ph->total_bytes = pl.total;
    ph->var_off = pl.var_off;
    ph->item_off = pl.item_off;
    ph->group_off = pl.group_off;
    ph->arena_bytes = arena_bytes;
    ph->aux_elems = aux_elems;
    ph->ws_bytes = std::max<uint64_t>(16, static_cast<uint64_t>(pl.nitems) * sizeof(Partial));
    ph->checksum = body_checksum(base + sizeof(PlanHeader), pl.total - sizeof(PlanHeader));
    return OMC_OK;
}


static bool opt_flags_ok(uint32_t flags) {
    if (flags & ~(OMC_OPT_STREAM_CODES | OMC_OPT_KEEP_CODES)) return false;
    return flags != (OMC_OPT_STREAM_CODES | OMC_OPT_KEEP_CODES);   // the two policies exclude each other
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace omc

using namespace omc;

extern "C" {

const char *omc_status_string(omc_status s) {
    switch (s) {
        case OMC_OK: return "ok";
        case OMC_ERR_NULL: return "null pointer";
        case OMC_ERR_FORMAT: return "unsupported format";
        case OMC_ERR_SIZE: return "bad size or offsets";
        case OMC_ERR_ALIGN: return "misaligned pointer or offset";
        case OMC_ERR_WORKSPACE: return "workspace missing or too small";
        case OMC_ERR_OPT: return "bad optimizer or missing state";
        case OMC_ERR_DEVICE: return "HIP launch failed";
        case OMC_ERR_PLAN: return "corrupt or foreign plan";
    }
    return "unknown status";
}

omc_status omc_format_validate(omc_format f) { return format_ok(f) ? OMC_OK : OMC_ERR_FORMAT; }

uint32_t omc_format_bits(omc_format f) { return format_ok(f) ? 1u + f.exp_bits + f.man_bits : 0u; }

float omc_format_max(omc_format f) {
    FmtParams p;
    return make_fmt_params(f, &p) ? p.maxval : 0.0f;
}

size_t omc_packed_bytes(omc_format f, uint64_t n) {
    if (!format_ok(f) || n == 0 || n > kMaxElems) return 0;
    return packed_bytes_u(1u + f.exp_bits + f.man_bits, n);
}

size_t omc_compress_workspace_bytes(uint64_t n) {
    if (n == 0 || n > kMaxElems) return 0;
    return static_cast<size_t>((n / kTileElems + kMinTilesPerChunk - 1) / kMinTilesPerChunk + 1) * sizeof(Partial);
}

omc_status omc_compress(const float *v, uint64_t n, omc_format f, int use_pvt, void *codes, float *sb,
                        void *ws, size_t ws_bytes, void *stream) {
    if (!v || !codes || !sb) return OMC_ERR_NULL;
    FmtParams fp;
    if (!make_fmt_params(f, &fp)) return OMC_ERR_FORMAT;
    if (n == 0 || n > kMaxElems) return OMC_ERR_SIZE;
    if (!aligned16(v) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return OMC_ERR_ALIGN;
    const size_t need = omc_compress_workspace_bytes(n);
    if (!ws || ws_bytes < need) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    const size_t pb = packed_bytes_u(fp.bits, n);
    const uintptr_t v0 = reinterpret_cast<uintptr_t>(v), c0 = reinterpret_cast<uintptr_t>(codes);
    if (v0 < c0 + pb && c0 < v0 + 4 * n) return OMC_ERR_SIZE;  // input and output overlap
    VarArgs va{n, pb / 4, fp};
    const int rc = launch_compress(v, va, use_pvt, codes, sb, static_cast<Partial *>(ws), stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

uint64_t omc_compress_noalloc_max_elems(void) {
    // largest n whose partial sums fit the static array: one partial per kMinTilesPerChunk full tiles, one for the tail
    const uint64_t parts = kStaticScratchBytes / sizeof(Partial);
    return (parts - 1) * kMinTilesPerChunk * kTileElems;
}

omc_status omc_compress_noalloc(const float *v, uint64_t n, omc_format f, int use_pvt, void *codes, float *sb,
                                void *stream) {
    if (!v || !codes || !sb) return OMC_ERR_NULL;
    FmtParams fp;
    if (!make_fmt_params(f, &fp)) return OMC_ERR_FORMAT;
    if (n == 0 || n > omc_compress_noalloc_max_elems()) return OMC_ERR_SIZE;
    if (omc_compress_workspace_bytes(n) > kStaticScratchBytes) return OMC_ERR_SIZE;
    if (!aligned16(v) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return OMC_ERR_ALIGN;
    const size_t pb = packed_bytes_u(fp.bits, n);
    const uintptr_t v0 = reinterpret_cast<uintptr_t>(v), c0 = reinterpret_cast<uintptr_t>(codes);
    if (v0 < c0 + pb && c0 < v0 + 4 * n) return OMC_ERR_SIZE;  // input and output overlap
    void *ws = nullptr;
    if (static_scratch(&ws) != 0) return OMC_ERR_DEVICE;
    // every partial the finalize reads is written by this call's kernels first: nothing has to start at zero
    VarArgs va{n, pb / 4, fp};
    const int rc = launch_compress(v, va, use_pvt, codes, sb, static_cast<Partial *>(ws), stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

omc_status omc_decompress(const void *codes, uint64_t n, omc_format f, const float *sb, float *out,
                          void *stream) {
    if (!codes || !out) return OMC_ERR_NULL;
    FmtParams fp;
    if (!make_fmt_params(f, &fp)) return OMC_ERR_FORMAT;
    if (n == 0 || n > kMaxElems) return OMC_ERR_SIZE;
    if (!aligned16(codes) || !aligned16(out) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return OMC_ERR_ALIGN;
    const size_t pb = packed_bytes_u(fp.bits, n);
    const uintptr_t o0 = reinterpret_cast<uintptr_t>(out), c0 = reinterpret_cast<uintptr_t>(codes);
    if (o0 < c0 + pb && c0 < o0 + 4 * n) return OMC_ERR_SIZE;
    VarArgs va{n, pb / 4, fp};
    const int rc = launch_decompress(codes, va, sb, out, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

size_t omc_plan_bytes(const omc_var *vars_host, uint32_t nvars) {
    PlanLayout pl;
    if (plan_layout(vars_host, nvars, &pl) != OMC_OK) return 0;
    return static_cast<size_t>(pl.total);
}

omc_status omc_plan_build(const omc_var *vars_host, uint32_t nvars, void *plan_host, size_t plan_bytes) {
    return build_plan(vars_host, nullptr, nvars, plan_host, plan_bytes);
}

size_t omc_workspace_bytes(const omc_var *vars_host, uint32_t nvars) {
    PlanLayout pl;
    if (plan_layout(vars_host, nvars, &pl) != OMC_OK) return 0;
    return static_cast<size_t>(std::max<uint64_t>(16, static_cast<uint64_t>(pl.nitems) * sizeof(Partial)));
}

size_t omc_plan_workspace_bytes(const void *plan_host) {
    const PlanHeader *ph = plan_check(plan_host);
    return ph ? static_cast<size_t>(ph->ws_bytes) : 0;
}

size_t omc_plan_arena_bytes(const void *plan_host) {
    const PlanHeader *ph = plan_check(plan_host);
    return ph ? static_cast<size_t>(ph->arena_bytes) : 0;
}

uint64_t omc_plan_aux_elems(const void *plan_host) {
    const PlanHeader *ph = plan_check(plan_host);
    return ph ? ph->aux_elems : 0;
}

static uint32_t plan_launches(const PlanHeader *ph) {
    const uint8_t *b = reinterpret_cast<const uint8_t *>(ph);
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(b + ph->group_off);
    uint32_t k = ph->nquant > 0 ? 1u : 0u;
    bool full = false, fp32 = false;
    for (uint32_t g = 0; g < ph->ngroups; ++g) {
        if (groups[g].nitems == 0) continue;
        ++k;
        full = full || groups[g].kind == kGroupFull;
        fp32 = fp32 || groups[g].kind == kGroupFp32;
    }
    if (full && fp32) --k;   // the fp32 variables share the first full-tile launch
    return k;
}

uint32_t omc_plan_launches(const void *plan_host) {
    const PlanHeader *ph = plan_check(plan_host);
    return ph ? plan_launches(ph) : 0;
}

omc_status omc_step_update_recompress_events(void *arena, size_t arena_bytes, const void *plan_host,
                                             const void *plan_dev, float *sb_table, const float *grads,
                                             float *state0, float *state1, uint64_t aux_elems,
                                             const omc_opt *opt, void *ws, size_t ws_bytes, void *stream,
                                             void *const *events, uint32_t nevents) {
    if (!arena || !plan_host || !plan_dev || !sb_table || !grads || !opt) return OMC_ERR_NULL;
    const PlanHeader *ph = plan_check(plan_host);
    if (!ph) return OMC_ERR_PLAN;
    if (opt->kind != OMC_SGD && opt->kind != OMC_MOMENTUM && opt->kind != OMC_ADAM) return OMC_ERR_OPT;
    if (!opt_flags_ok(opt->flags)) return OMC_ERR_OPT;
    if (opt->kind >= OMC_MOMENTUM && !state0) return OMC_ERR_OPT;
    if (opt->kind == OMC_ADAM && !state1) return OMC_ERR_OPT;
    if (arena_bytes < ph->arena_bytes || aux_elems < ph->aux_elems) return OMC_ERR_SIZE;
    if (!aligned16(arena) || !aligned16(grads) || !aligned16(plan_dev) ||
        (reinterpret_cast<uintptr_t>(sb_table) & 7u))
        return OMC_ERR_ALIGN;
    if (opt->kind >= OMC_MOMENTUM && !aligned16(state0)) return OMC_ERR_ALIGN;
    if (opt->kind == OMC_ADAM && !aligned16(state1)) return OMC_ERR_ALIGN;
    if (!ws || ws_bytes < ph->ws_bytes) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    if (events) {
        const uint32_t need = 2 * plan_launches(ph);
        if (nevents < need) return OMC_ERR_SIZE;
        for (uint32_t i = 0; i < need; ++i)
            if (!events[i]) return OMC_ERR_NULL;
    }
    const int rc = launch_step(arena, ph, plan_dev, sb_table, grads, state0, state1, *opt,
                               static_cast<Partial *>(ws), stream, events);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

omc_status omc_step_update_recompress(void *arena, size_t arena_bytes, const void *plan_host,
                                      const void *plan_dev, float *sb_table, const float *grads,
                                      float *state0, float *state1, uint64_t aux_elems,
                                      const omc_opt *opt, void *ws, size_t ws_bytes, void *stream) {
    return omc_step_update_recompress_events(arena, arena_bytes, plan_host, plan_dev, sb_table, grads,
                                             state0, state1, aux_elems, opt, ws, ws_bytes, stream,
                                             nullptr, 0);
}

omc_status omc_compress_set(const float *values, uint64_t aux_elems, const void *plan_host, const void *plan_dev,
                            void *arena, size_t arena_bytes, float *sb_table, void *ws, size_t ws_bytes,
                            void *stream) {
    if (!values || !plan_host || !plan_dev || !arena || !sb_table) return OMC_ERR_NULL;
    const PlanHeader *ph = plan_check(plan_host);
    if (!ph) return OMC_ERR_PLAN;
    if (arena_bytes < ph->arena_bytes || aux_elems < ph->aux_elems) return OMC_ERR_SIZE;
    if (!aligned16(values) || !aligned16(arena) || !aligned16(plan_dev) ||
        (reinterpret_cast<uintptr_t>(sb_table) & 7u))
        return OMC_ERR_ALIGN;
    if (!ws || ws_bytes < ph->ws_bytes) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    const uintptr_t v0 = reinterpret_cast<uintptr_t>(values), a0 = reinterpret_cast<uintptr_t>(arena);
    if (v0 < a0 + ph->arena_bytes && a0 < v0 + 4 * ph->aux_elems) return OMC_ERR_SIZE;   // overlap
    const int rc = launch_compress_set(values, ph, plan_dev, arena, sb_table, static_cast<Partial *>(ws), stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

omc_status omc_decompress_set(const void *arena, size_t arena_bytes, const void *plan_host, const void *plan_dev,
                              const float *sb_table, float *out, uint64_t aux_elems, void *stream) {
    if (!arena || !plan_host || !plan_dev || !sb_table || !out) return OMC_ERR_NULL;
    const PlanHeader *ph = plan_check(plan_host);
    if (!ph) return OMC_ERR_PLAN;
    if (arena_bytes < ph->arena_bytes || aux_elems < ph->aux_elems) return OMC_ERR_SIZE;
    if (!aligned16(out) || !aligned16(arena) || !aligned16(plan_dev) ||
        (reinterpret_cast<uintptr_t>(sb_table) & 7u))
        return OMC_ERR_ALIGN;
    const uintptr_t o0 = reinterpret_cast<uintptr_t>(out), a0 = reinterpret_cast<uintptr_t>(arena);
    if (o0 < a0 + ph->arena_bytes && a0 < o0 + 4 * ph->aux_elems) return OMC_ERR_SIZE;   // overlap
    const int rc = launch_decompress_set(arena, ph, plan_dev, sb_table, out, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

uint64_t omc_plan_transport_bytes(const void *plan_host) {
    const PlanHeader *ph = plan_check(plan_host);
    if (!ph) return 0;
    const uint8_t *b = reinterpret_cast<const uint8_t *>(ph);
    const PlanVar *pv = reinterpret_cast<const PlanVar *>(b + ph->var_off);
    uint64_t total = 0;
    for (uint32_t i = 0; i < ph->nvars; ++i)
        total += (pv[i].flags & OMC_VAR_QUANTIZED) ? pv[i].total_dwords * 4 + 8 : 4 * pv[i].n;
    return total;
}

}  // extern "C"

// ---- server-side aggregation ---------------------------------------------------------------
namespace omc {
struct AggLayout {
    uint64_t var_off, src_off, item_off, group_off, total;
    uint32_t nitems;
    std::vector<PlanGroup> groups;
    std::vector<uint8_t> any_quant;          // per variable
};

static const AggHeader *agg_check(const void *agg_host) {
    if (!agg_host) return nullptr;
    const AggHeader *ah = static_cast<const AggHeader *>(agg_host);
    if (ah->magic != kAggMagic || ah->version != kAggVersion) return nullptr;
    if (ah->nreplicas == 0 || ah->nreplicas > kMaxReplicas) return nullptr;
    if (ah->var_off != sizeof(AggHeader)) return nullptr;
    if (ah->src_off != ah->var_off + static_cast<uint64_t>(ah->nvars) * sizeof(AggVar)) return nullptr;
    if (ah->item_off != ah->src_off + static_cast<uint64_t>(ah->nvars) * ah->nreplicas * sizeof(AggSrc)) return nullptr;
    if (ah->group_off != ah->item_off + static_cast<uint64_t>(ah->nitems) * sizeof(PlanItem)) return nullptr;
    if (ah->total_bytes != align_up(ah->group_off + static_cast<uint64_t>(ah->ngroups) * sizeof(PlanGroup), 16))
        return nullptr;
    if (ah->checksum != body_checksum(static_cast<const uint8_t *>(agg_host) + sizeof(AggHeader), ah->total_bytes - sizeof(AggHeader)))
        return nullptr;
    const PlanGroup *groups = reinterpret_cast<const PlanGroup *>(static_cast<const uint8_t *>(agg_host) + ah->group_off);
    for (uint32_t g = 0; g < ah->ngroups; ++g) {          // what the host reads from the body: the launch groups
        if (groups[g].kind > kGroupFp32) return nullptr;
        if (static_cast<uint64_t>(groups[g].first_item) + groups[g].nitems > ah->nitems) return nullptr;
        if (groups[g].kind == kGroupFull && (groups[g].bits < 2 || groups[g].bits > 32)) return nullptr;
    }
    return ah;
}

static bool same_format(const FmtParams &a, const FmtParams &b) {
    return a.exp_bits == b.exp_bits && a.man_bits == b.man_bits && a.bias == b.bias;
}

// The clients' plans must describe one variable list: same count, sizes and aux offsets, and one
// format per variable among the clients that quantize it.
static omc_status agg_layout(const void *const *plans_host, uint32_t R, AggLayout *al) {
    if (!plans_host) return OMC_ERR_NULL;
    if (R == 0 || R > kMaxReplicas) return OMC_ERR_SIZE;
    const PlanHeader *p0 = plan_check(plans_host[0]);
    if (!p0) return OMC_ERR_PLAN;
    const uint32_t nvars = p0->nvars;
    const PlanVar *v0 = reinterpret_cast<const PlanVar *>(static_cast<const uint8_t *>(plans_host[0]) + p0->var_off);
    al->any_quant.assign(nvars, 0);
    std::vector<FmtParams> fmt(nvars);
    for (uint32_t r = 0; r < R; ++r) {
        const PlanHeader *ph = plan_check(plans_host[r]);
        if (!ph) return OMC_ERR_PLAN;
        if (ph->nvars != nvars) return OMC_ERR_SIZE;
        const PlanVar *pv = reinterpret_cast<const PlanVar *>(static_cast<const uint8_t *>(plans_host[r]) + ph->var_off);
        for (uint32_t i = 0; i < nvars; ++i) {
            if (pv[i].n != v0[i].n || pv[i].aux_offset != v0[i].aux_offset) return OMC_ERR_SIZE;
            if (pv[i].flags & OMC_VAR_QUANTIZED) {
                if (al->any_quant[i] && !same_format(fmt[i], pv[i].fp)) return OMC_ERR_FORMAT;
                al->any_quant[i] = 1;
                fmt[i] = pv[i].fp;
            }
        }
    }
    bool present[33] = {false};
    bool tails = false, flat = false;
    uint64_t nitems = 0;
    for (uint32_t i = 0; i < nvars; ++i) {
        const uint64_t n = v0[i].n;
        if (al->any_quant[i]) {
            if (n >= kTileElems) present[fmt[i].bits] = true;
            if (n % kTileElems) tails = true;
            nitems += (n / kTileElems + tiles_per_chunk(fmt[i].bits) - 1) / tiles_per_chunk(fmt[i].bits) + (n % kTileElems ? 1 : 0);
        } else {
            flat = true;
            nitems += (n + kChunkElems - 1) / kChunkElems;
        }
    }
    if (nitems > 0x7fffffffull) return OMC_ERR_SIZE;
    al->groups.clear();
    for (uint32_t b = 2; b <= 32; ++b)
        if (present[b]) al->groups.push_back(PlanGroup{kGroupFull, b, 0, 0, 0, 0});
    if (tails) al->groups.push_back(PlanGroup{kGroupTail, 0, 0, 0, 0, 0});
    if (flat) al->groups.push_back(PlanGroup{kGroupFp32, 0, 0, 0, 0, 0});
    al->nitems = static_cast<uint32_t>(nitems);
    al->var_off = sizeof(AggHeader);
    al->src_off = al->var_off + static_cast<uint64_t>(nvars) * sizeof(AggVar);
    al->item_off = al->src_off + static_cast<uint64_t>(nvars) * R * sizeof(AggSrc);
    al->group_off = al->item_off + nitems * sizeof(PlanItem);
    al->total = align_up(al->group_off + al->groups.size() * sizeof(PlanGroup), 16);
    return OMC_OK;
}
}  // namespace omc

extern "C" {

size_t omc_aggregate_plan_bytes(const void *const *plans_host, uint32_t nreplicas) {
    AggLayout al;
    if (agg_layout(plans_host, nreplicas, &al) != OMC_OK) return 0;
    return static_cast<size_t>(al.total);
}

omc_status omc_aggregate_plan_build(const void *const *plans_host, uint32_t nreplicas, void *agg_host,
                                    size_t agg_bytes) {
    if (!agg_host) return OMC_ERR_NULL;
    AggLayout al;
    const omc_status st = agg_layout(plans_host, nreplicas, &al);
    if (st != OMC_OK) return st;
    if (agg_bytes < al.total) return OMC_ERR_SIZE;
    const uint32_t R = nreplicas;
    uint8_t *base = static_cast<uint8_t *>(agg_host);
    std::memset(base, 0, al.total);
    AggHeader *ah = reinterpret_cast<AggHeader *>(base);
    AggVar *av = reinterpret_cast<AggVar *>(base + al.var_off);
    AggSrc *src = reinterpret_cast<AggSrc *>(base + al.src_off);
    PlanItem *items = reinterpret_cast<PlanItem *>(base + al.item_off);
    PlanGroup *groups = reinterpret_cast<PlanGroup *>(base + al.group_off);
    const PlanHeader *p0 = plan_check(plans_host[0]);
    const uint32_t nvars = p0->nvars;
    for (uint32_t r = 0; r < R; ++r) {
        const PlanHeader *ph = plan_check(plans_host[r]);
        const PlanVar *pv = reinterpret_cast<const PlanVar *>(static_cast<const uint8_t *>(plans_host[r]) + ph->var_off);
        ah->arena_bytes[r] = ph->arena_bytes;
        for (uint32_t i = 0; i < nvars; ++i) {
            AggSrc &s = src[static_cast<uint64_t>(i) * R + r];
            s.data_offset = pv[i].data_offset;
            s.quantized = (pv[i].flags & OMC_VAR_QUANTIZED) ? 1u : 0u;
            if (r == 0) {
                av[i].aux_offset = pv[i].aux_offset;
                av[i].n = pv[i].n;
            }
            if (s.quantized) {
                av[i].fp = pv[i].fp;
                av[i].total_dwords = pv[i].total_dwords;
            }
        }
    }
    uint32_t next = 0;
    for (size_t gi = 0; gi < al.groups.size(); ++gi) {
        PlanGroup g = al.groups[gi];
        g.first_item = next;
        for (uint32_t i = 0; i < nvars; ++i) {
            const uint64_t n = av[i].n;
            const bool q = al.any_quant[i] != 0;
            if (g.kind == kGroupFull) {
                if (!q || av[i].fp.bits != g.bits || n < kTileElems) continue;
                const uint32_t c_end = static_cast<uint32_t>((n / kTileElems + tiles_per_chunk(g.bits) - 1) / tiles_per_chunk(g.bits));
                for (uint32_t c = 0; c < c_end; ++c) items[next++] = PlanItem{i, c};
            } else if (g.kind == kGroupTail) {
                if (!q || n % kTileElems == 0) continue;
                items[next++] = PlanItem{i, 0};
            } else {
                if (q) continue;
                const uint32_t c_end = static_cast<uint32_t>((n + kChunkElems - 1) / kChunkElems);
                for (uint32_t c = 0; c < c_end; ++c) items[next++] = PlanItem{i, c};
            }
        }
        g.nitems = next - g.first_item;
        groups[gi] = g;
    }
    ah->magic = kAggMagic;
    ah->version = kAggVersion;
    ah->nvars = nvars;
    ah->nitems = al.nitems;
    ah->ngroups = static_cast<uint32_t>(al.groups.size());
    ah->nreplicas = R;
    ah->total_bytes = al.total;
    ah->var_off = al.var_off;
    ah->src_off = al.src_off;
    ah->item_off = al.item_off;
    ah->group_off = al.group_off;
    ah->aux_elems = p0->aux_elems;
    ah->checksum = body_checksum(base + sizeof(AggHeader), al.total - sizeof(AggHeader));
    return OMC_OK;
}

omc_status omc_aggregate_mean(const void *agg_host, const void *agg_dev, const void *const *arenas,
                              const size_t *arena_bytes, const float *const *sb_tables, float *out,
                              uint64_t aux_elems, void *stream) {
    if (!agg_host || !agg_dev || !arenas || !arena_bytes || !sb_tables || !out) return OMC_ERR_NULL;
    const AggHeader *ah = agg_check(agg_host);
    if (!ah) return OMC_ERR_PLAN;
    if (aux_elems < ah->aux_elems) return OMC_ERR_SIZE;
    if (!aligned16(agg_dev) || !aligned16(out)) return OMC_ERR_ALIGN;
    AggPointers ptrs{};
    const uintptr_t o0 = reinterpret_cast<uintptr_t>(out), o1 = o0 + 4 * ah->aux_elems;
    for (uint32_t r = 0; r < ah->nreplicas; ++r) {
        if (!arenas[r] || !sb_tables[r]) return OMC_ERR_NULL;
        if (arena_bytes[r] < ah->arena_bytes[r]) return OMC_ERR_SIZE;
        if (!aligned16(arenas[r]) || (reinterpret_cast<uintptr_t>(sb_tables[r]) & 3u)) return OMC_ERR_ALIGN;
        const uintptr_t a0 = reinterpret_cast<uintptr_t>(arenas[r]);
        if (a0 < o1 && o0 < a0 + ah->arena_bytes[r]) return OMC_ERR_SIZE;     // output overlaps an input
        ptrs.arena[r] = static_cast<const uint8_t *>(arenas[r]);
        ptrs.sb[r] = sb_tables[r];
    }
    const int rc = launch_aggregate_mean(ah, agg_dev, ptrs, out, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

size_t omc_dequant_gemm_workspace_bytes(uint32_t M) {
    return M == 0 ? 0 : 256;   // the flag words of the top-code scan (independent of M)
}

omc_status omc_dequant_gemm(const uint16_t *A, const void *codes, omc_format f, const float *sb, float *C,
                            uint32_t M, uint32_t N, uint32_t K, void *ws, size_t ws_bytes, void *stream) {
    if (!A || !codes || !C) return OMC_ERR_NULL;
    FmtParams fp;
    if (!make_fmt_params(f, &fp)) return OMC_ERR_FORMAT;
    if (fp.man_bits > 7) return OMC_ERR_FORMAT;
    if (M == 0 || N == 0 || K == 0 || M % 256 != 0 || N % 128 != 0 || K % 32 != 0) return OMC_ERR_SIZE;
    if (!aligned16(A) || !aligned16(codes) || !aligned16(C) || (reinterpret_cast<uintptr_t>(sb) & 3u))
        return OMC_ERR_ALIGN;
    if (!ws || ws_bytes < omc_dequant_gemm_workspace_bytes(M)) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    const int rc = launch_dequant_gemm(A, codes, fp, sb, C, M, N, K, static_cast<float *>(ws), 0, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

size_t omc_dw_update_workspace_bytes(omc_format f, uint32_t M, uint32_t N, uint32_t K) {
    if (!format_ok(f)) return 0;
    if (M == 0 || N == 0 || K == 0 || M % 32 != 0 || K % 256 != 0 || N % 128 != 0) return 0;
    return dw_workspace_bytes(1u + f.exp_bits + f.man_bits, M, N, K);
}

omc_status omc_dw_update_recompress(const uint16_t *X, const uint16_t *dY, void *codes, omc_format f, float *sb,
                                    int use_pvt, float *state0, float *state1, const omc_opt *opt, float *dW_out,
                                    uint32_t M, uint32_t N, uint32_t K, void *ws, size_t ws_bytes, void *stream) {
    if (!X || !dY || !codes || !sb || !opt) return OMC_ERR_NULL;
    FmtParams fp;
    if (!make_fmt_params(f, &fp)) return OMC_ERR_FORMAT;
    if (M == 0 || N == 0 || K == 0 || M % 32 != 0 || K % 256 != 0 || N % 128 != 0) return OMC_ERR_SIZE;
    if (opt->kind != OMC_SGD && opt->kind != OMC_MOMENTUM && opt->kind != OMC_ADAM) return OMC_ERR_OPT;
    if (!opt_flags_ok(opt->flags)) return OMC_ERR_OPT;
    if (opt->kind >= OMC_MOMENTUM && !state0) return OMC_ERR_OPT;
    if (opt->kind == OMC_ADAM && !state1) return OMC_ERR_OPT;
    if (!aligned16(X) || !aligned16(dY) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return OMC_ERR_ALIGN;
    if ((state0 && !aligned16(state0)) || (state1 && !aligned16(state1)) || (dW_out && !aligned16(dW_out)))
        return OMC_ERR_ALIGN;
    const size_t need = omc_dw_update_workspace_bytes(f, M, N, K);
    if (!ws || ws_bytes < need) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    const int rc = launch_dw_update(X, dY, codes, fp, sb, use_pvt, state0, state1, *opt, dW_out, M, N, K,
                                    ws, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

omc_status omc_dequant_gemm_dx(const uint16_t *dY, const void *codes, omc_format f, const float *sb, float *dX,
                               uint32_t M, uint32_t N, uint32_t K, void *ws, size_t ws_bytes, void *stream) {
    if (!dY || !codes || !dX) return OMC_ERR_NULL;
    FmtParams fp;
    if (!make_fmt_params(f, &fp)) return OMC_ERR_FORMAT;
    if (fp.man_bits > 7) return OMC_ERR_FORMAT;
    if (M == 0 || N == 0 || K == 0 || M % 256 != 0 || K % 128 != 0 || N % 32 != 0) return OMC_ERR_SIZE;
    if (!aligned16(dY) || !aligned16(codes) || !aligned16(dX) || (reinterpret_cast<uintptr_t>(sb) & 3u))
        return OMC_ERR_ALIGN;
    if (!ws || ws_bytes < omc_dequant_gemm_workspace_bytes(M)) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    // output columns = K (the weights' rows), contraction over N
    const int rc = launch_dequant_gemm(dY, codes, fp, sb, dX, M, K, N, static_cast<float *>(ws), 1, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

}  // extern "C"

// ---- change of the quantized subset between rounds (Sec. 2.5) ---------------------------------------
namespace omc {
struct ReselectLayout {
    std::vector<uint32_t> actions;
    std::vector<omc_var> c_vars, d_vars;       // derived tables
    std::vector<uint32_t> c_index, d_index;    // their entries of the (s, b) table
    uint64_t action_off, plan_c_off, plan_c_bytes, plan_d_off, plan_d_bytes, total;
    uint64_t alg_bytes;
};

static omc_format format_of(const FmtParams &fp) {
    omc_format f;
    f.exp_bits = static_cast<uint8_t>(fp.exp_bits);
    f.man_bits = static_cast<uint8_t>(fp.man_bits);
    f.exp_bias = static_cast<int16_t>(fp.bias);
    return f;
}

static const PlanVar *plan_vars(const PlanHeader *ph) {
    return reinterpret_cast<const PlanVar *>(reinterpret_cast<const uint8_t *>(ph) + ph->var_off);
}

// Both plans must describe the same variable list (count, sizes); a variable that is quantized in both
// must keep its format.  Every variable gets one action; the two derived tables address the old arena
// as the "values" of a compress-set (offsets in floats) and the new arena as the output of a decompress-set.
static omc_status reselect_layout(const void *old_host, const void *new_host, ReselectLayout *rl) {
    const PlanHeader *po = plan_check(old_host), *pn = plan_check(new_host);
    if (!po || !pn) return OMC_ERR_PLAN;
    if (po->nvars != pn->nvars) return OMC_ERR_SIZE;
    const PlanVar *vo = plan_vars(po), *vn = plan_vars(pn);
    const uint32_t nvars = po->nvars;
    rl->actions.assign(nvars, 0);
    rl->c_vars.clear(); rl->d_vars.clear(); rl->c_index.clear(); rl->d_index.clear();
    rl->alg_bytes = 0;
    for (uint32_t i = 0; i < nvars; ++i) {
        if (vo[i].n != vn[i].n) return OMC_ERR_SIZE;
        const bool qo = (vo[i].flags & OMC_VAR_QUANTIZED) != 0, qn = (vn[i].flags & OMC_VAR_QUANTIZED) != 0;
        omc_var v{};
        if (qo == qn) {                                   // unchanged: its bytes move as a run of floats
            if (qo && !(vo[i].fp.exp_bits == vn[i].fp.exp_bits && vo[i].fp.man_bits == vn[i].fp.man_bits &&
                        vo[i].fp.bias == vn[i].fp.bias))
                return OMC_ERR_FORMAT;
            const uint64_t bytes = qo ? vo[i].total_dwords * 4 : 4 * vo[i].n;
            rl->actions[i] = qo ? kRsCopyQuantized : kRsCopyFp32;
            v.data_offset = vn[i].data_offset;
            v.aux_offset = vo[i].data_offset / 4;
            v.n = bytes / 4;
            v.flags = 0;
            rl->c_vars.push_back(v);
            rl->c_index.push_back(i);
            rl->alg_bytes += 2 * bytes;
        } else if (qn) {                                  // fp32 -> codes: compressed straight from the old arena
            rl->actions[i] = kRsToQuantized;
            v.data_offset = vn[i].data_offset;
            v.aux_offset = vo[i].data_offset / 4;
            v.n = vn[i].n;
            v.fmt = format_of(vn[i].fp);
            v.flags = vn[i].flags;
            rl->c_vars.push_back(v);
            rl->c_index.push_back(i);
            rl->alg_bytes += 4 * vn[i].n + vn[i].total_dwords * 4 + 8;
        } else {                                          // codes -> fp32: decompressed straight into the new arena
            rl->actions[i] = kRsToFp32;
            v.data_offset = vo[i].data_offset;
            v.aux_offset = vn[i].data_offset / 4;
            v.n = vo[i].n;
            v.fmt = format_of(vo[i].fp);
            v.flags = vo[i].flags;
            rl->d_vars.push_back(v);
            rl->d_index.push_back(i);
            rl->alg_bytes += 4 * vo[i].n + vo[i].total_dwords * 4 + 8;
        }
    }
    rl->action_off = sizeof(ReselectHeader);
    uint64_t off = align_up(rl->action_off + 4ull * nvars, 16);
    rl->plan_c_off = rl->plan_c_bytes = rl->plan_d_off = rl->plan_d_bytes = 0;
    if (!rl->c_vars.empty()) {
        PlanLayout pl;
        const omc_status st = plan_layout(rl->c_vars.data(), static_cast<uint32_t>(rl->c_vars.size()), &pl);
        if (st != OMC_OK) return st;
        rl->plan_c_off = off;
        rl->plan_c_bytes = pl.total;
        off = align_up(off + pl.total, 16);
    }
    if (!rl->d_vars.empty()) {
        PlanLayout pl;
        const omc_status st = plan_layout(rl->d_vars.data(), static_cast<uint32_t>(rl->d_vars.size()), &pl);
        if (st != OMC_OK) return st;
        rl->plan_d_off = off;
        rl->plan_d_bytes = pl.total;
        off = align_up(off + pl.total, 16);
    }
    rl->total = off;
    return OMC_OK;
}

static const ReselectHeader *reselect_check(const void *rs_host) {
    if (!rs_host) return nullptr;
    const ReselectHeader *rh = static_cast<const ReselectHeader *>(rs_host);
    if (rh->magic != kReselectMagic || rh->version != kReselectVersion || rh->nvars == 0) return nullptr;
    if (rh->action_off != sizeof(ReselectHeader) || rh->total_bytes < rh->action_off + 4ull * rh->nvars) return nullptr;
    const uint8_t *base = static_cast<const uint8_t *>(rs_host);
    if (rh->checksum != body_checksum(base + sizeof(ReselectHeader), rh->total_bytes - sizeof(ReselectHeader))) return nullptr;
    if (rh->plan_c_bytes && (rh->plan_c_off % 16 || rh->plan_c_off + rh->plan_c_bytes > rh->total_bytes)) return nullptr;
    if (rh->plan_d_bytes && (rh->plan_d_off % 16 || rh->plan_d_off + rh->plan_d_bytes > rh->total_bytes)) return nullptr;
    if (rh->plan_c_bytes && !plan_check(base + rh->plan_c_off)) return nullptr;
    if (rh->plan_d_bytes && !plan_check(base + rh->plan_d_off)) return nullptr;
    return rh;
}

static const TransportHeader *transport_check(const void *prefix, size_t prefix_bytes, uint64_t msg_bytes) {
    if (!prefix || prefix_bytes < sizeof(TransportHeader)) return nullptr;
    const TransportHeader *th = static_cast<const TransportHeader *>(prefix);
    if (th->magic != kTransportMagic || th->version != kTransportVersion || th->nvars == 0) return nullptr;
    if (th->nquant > th->nvars) return nullptr;
    const uint64_t meta = align_up(sizeof(TransportHeader) + static_cast<uint64_t>(th->nvars) * sizeof(TransportVar), kTransportAlign);
    if (th->sb_off != meta) return nullptr;
    if (th->payload_off != align_up(th->sb_off + 8ull * th->nvars, kTransportAlign)) return nullptr;
    if (th->total_bytes != th->payload_off + th->payload_bytes || th->payload_bytes % 16) return nullptr;
    if (msg_bytes < th->total_bytes) return nullptr;
    return th;
}
}  // namespace omc

extern "C" {

size_t omc_reselect_plan_bytes(const void *plan_old_host, const void *plan_new_host) {
    ReselectLayout rl;
    if (reselect_layout(plan_old_host, plan_new_host, &rl) != OMC_OK) return 0;
    return static_cast<size_t>(rl.total);
}

omc_status omc_reselect_plan_build(const void *plan_old_host, const void *plan_new_host, void *rs_host, size_t rs_bytes) {
    if (!rs_host) return OMC_ERR_NULL;
    ReselectLayout rl;
    const omc_status st = reselect_layout(plan_old_host, plan_new_host, &rl);
    if (st != OMC_OK) return st;
    if (rs_bytes < rl.total) return OMC_ERR_SIZE;
    uint8_t *base = static_cast<uint8_t *>(rs_host);
    std::memset(base, 0, rl.total);
    ReselectHeader *rh = reinterpret_cast<ReselectHeader *>(base);
    const PlanHeader *po = plan_check(plan_old_host), *pn = plan_check(plan_new_host);
    std::memcpy(base + rl.action_off, rl.actions.data(), 4ull * rl.actions.size());
    uint64_t ws = 16;
    if (rl.plan_c_bytes) {
        const omc_status sc = build_plan(rl.c_vars.data(), rl.c_index.data(), static_cast<uint32_t>(rl.c_vars.size()),
                                         base + rl.plan_c_off, rl.plan_c_bytes);
        if (sc != OMC_OK) return sc;
        ws = std::max<uint64_t>(ws, reinterpret_cast<const PlanHeader *>(base + rl.plan_c_off)->ws_bytes);
    }
    if (rl.plan_d_bytes) {
        const omc_status sd = build_plan(rl.d_vars.data(), rl.d_index.data(), static_cast<uint32_t>(rl.d_vars.size()),
                                         base + rl.plan_d_off, rl.plan_d_bytes);
        if (sd != OMC_OK) return sd;
    }
    rh->magic = kReselectMagic;
    rh->version = kReselectVersion;
    rh->nvars = po->nvars;
    rh->total_bytes = rl.total;
    rh->action_off = rl.action_off;
    rh->plan_c_off = rl.plan_c_off; rh->plan_c_bytes = rl.plan_c_bytes;
    rh->plan_d_off = rl.plan_d_off; rh->plan_d_bytes = rl.plan_d_bytes;
    rh->arena_old_bytes = po->arena_bytes;
    rh->arena_new_bytes = pn->arena_bytes;
    rh->ws_bytes = ws;
    rh->algorithmic_bytes = rl.alg_bytes;
    rh->checksum = body_checksum(base + sizeof(ReselectHeader), rl.total - sizeof(ReselectHeader));
    return OMC_OK;
}

size_t omc_reselect_workspace_bytes(const void *rs_host) {
    const ReselectHeader *rh = reselect_check(rs_host);
    return rh ? static_cast<size_t>(rh->ws_bytes) : 0;
}

uint64_t omc_reselect_algorithmic_bytes(const void *rs_host) {
    const ReselectHeader *rh = reselect_check(rs_host);
    return rh ? rh->algorithmic_bytes : 0;
}

omc_status omc_reselect(const void *rs_host, const void *rs_dev, const void *arena_old, size_t arena_old_bytes,
                        const float *sb_old, void *arena_new, size_t arena_new_bytes, float *sb_new, void *ws,
                        size_t ws_bytes, void *stream) {
    if (!rs_host || !rs_dev || !arena_old || !sb_old || !arena_new || !sb_new) return OMC_ERR_NULL;
    const ReselectHeader *rh = reselect_check(rs_host);
    if (!rh) return OMC_ERR_PLAN;
    if (arena_old_bytes < rh->arena_old_bytes || arena_new_bytes < rh->arena_new_bytes) return OMC_ERR_SIZE;
    if (!aligned16(rs_dev) || !aligned16(arena_old) || !aligned16(arena_new) ||
        (reinterpret_cast<uintptr_t>(sb_old) & 7u) || (reinterpret_cast<uintptr_t>(sb_new) & 7u))
        return OMC_ERR_ALIGN;
    if (!ws || ws_bytes < rh->ws_bytes) return OMC_ERR_WORKSPACE;
    if (!aligned16(ws)) return OMC_ERR_ALIGN;
    const uintptr_t o0 = reinterpret_cast<uintptr_t>(arena_old), n0 = reinterpret_cast<uintptr_t>(arena_new);
    if (o0 < n0 + rh->arena_new_bytes && n0 < o0 + rh->arena_old_bytes) return OMC_ERR_SIZE;   // the arenas overlap
    if (sb_old == sb_new) return OMC_ERR_SIZE;
    const uint8_t *hb = static_cast<const uint8_t *>(rs_host);
    const uint8_t *db = static_cast<const uint8_t *>(rs_dev);
    int rc = 0;
    if (rh->plan_c_bytes)
        rc = launch_compress_set(static_cast<const float *>(arena_old), reinterpret_cast<const PlanHeader *>(hb + rh->plan_c_off),
                                 db + rh->plan_c_off, arena_new, sb_new, static_cast<Partial *>(ws), stream);
    if (rc == 0 && rh->plan_d_bytes)
        rc = launch_decompress_set(arena_old, reinterpret_cast<const PlanHeader *>(hb + rh->plan_d_off), db + rh->plan_d_off,
                                   sb_old, static_cast<float *>(arena_new), stream);
    if (rc == 0)
        rc = launch_reselect_sb(reinterpret_cast<const uint32_t *>(db + rh->action_off), rh->nvars, sb_old, sb_new, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

// ---- transport / checkpoint message -------------------------------------------------------------------

size_t omc_transport_meta_bytes(uint32_t nvars) {
    if (nvars == 0) return 0;
    return static_cast<size_t>(align_up(sizeof(TransportHeader) + static_cast<uint64_t>(nvars) * sizeof(TransportVar), kTransportAlign));
}

static bool transport_header_for(const PlanHeader *ph, TransportHeader *th) {
    const PlanVar *pv = plan_vars(ph);
    uint64_t payload = 0;
    for (uint32_t i = 0; i < ph->nvars; ++i)
        payload += align_up((pv[i].flags & OMC_VAR_QUANTIZED) ? pv[i].total_dwords * 4 : 4 * pv[i].n, 16);
    std::memset(th, 0, sizeof *th);
    th->magic = kTransportMagic;
    th->version = kTransportVersion;
    th->nvars = ph->nvars;
    th->nquant = ph->nquant;
    th->sb_off = omc_transport_meta_bytes(ph->nvars);
    th->payload_off = align_up(th->sb_off + 8ull * ph->nvars, kTransportAlign);
    th->payload_bytes = payload;
    th->total_bytes = th->payload_off + payload;
    th->aux_elems = ph->aux_elems;
    return true;
}

uint64_t omc_transport_bytes(const void *plan_host) {
    const PlanHeader *ph = plan_check(plan_host);
    if (!ph) return 0;
    TransportHeader th;
    transport_header_for(ph, &th);
    return th.total_bytes;
}

omc_status omc_transport_pack(const void *plan_host, const void *plan_dev, const void *arena, size_t arena_bytes,
                              const float *sb_table, void *msg_dev, size_t msg_bytes, void *stream) {
    if (!plan_host || !plan_dev || !arena || !sb_table || !msg_dev) return OMC_ERR_NULL;
    const PlanHeader *ph = plan_check(plan_host);
    if (!ph) return OMC_ERR_PLAN;
    if (arena_bytes < ph->arena_bytes) return OMC_ERR_SIZE;
    TransportHeader th;
    transport_header_for(ph, &th);
    if (msg_bytes < th.total_bytes) return OMC_ERR_SIZE;
    if (!aligned16(plan_dev) || !aligned16(arena) || !aligned16(msg_dev) || (reinterpret_cast<uintptr_t>(sb_table) & 7u))
        return OMC_ERR_ALIGN;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(arena), m0 = reinterpret_cast<uintptr_t>(msg_dev);
    if (a0 < m0 + th.total_bytes && m0 < a0 + ph->arena_bytes) return OMC_ERR_SIZE;            // message overlaps the arena
    const int rc = launch_transport_pack(ph, plan_dev, arena, sb_table, msg_dev, th, stream);
    return rc == 0 ? OMC_OK : OMC_ERR_DEVICE;
}

omc_status omc_transport_open(const void *msg_prefix_host, size_t prefix_bytes, uint64_t msg_bytes, omc_var *vars_out,
                              uint32_t vars_cap, uint32_t *nvars_out, uint64_t *sb_offset, uint64_t *arena_offset,
                              uint64_t *arena_bytes, uint64_t *aux_elems) {
    if (!msg_prefix_host || !nvars_out) return OMC_ERR_NULL;
    const TransportHeader *th = transport_check(msg_prefix_host, prefix_bytes, msg_bytes);
    if (!th) return OMC_ERR_PLAN;
    *nvars_out = th->nvars;
    if (sb_offset) *sb_offset = th->sb_off;
    if (arena_offset) *arena_offset = th->payload_off;
    if (arena_bytes) *arena_bytes = th->payload_bytes;
    if (aux_elems) *aux_elems = th->aux_elems;
    if (!vars_out) return OMC_OK;                           // size query
    if (prefix_bytes < th->sb_off || vars_cap < th->nvars) return OMC_ERR_SIZE;
    const TransportVar *tv = reinterpret_cast<const TransportVar *>(static_cast<const uint8_t *>(msg_prefix_host) + sizeof(TransportHeader));
    uint64_t sum = 0, next = 0;
    uint32_t nq = 0;
    for (uint32_t i = 0; i < th->nvars; ++i) {
        sum += transport_var_hash(i, tv[i]);
        omc_var v{};
        v.data_offset = tv[i].payload_offset;
        v.aux_offset = tv[i].aux_offset;
        v.n = tv[i].n;
        v.fmt.exp_bits = tv[i].exp_bits;
        v.fmt.man_bits = tv[i].man_bits;
        v.fmt.exp_bias = tv[i].exp_bias;
        v.flags = tv[i].flags;
        if (v.flags & ~(OMC_VAR_QUANTIZED | OMC_VAR_NO_PVT)) return OMC_ERR_PLAN;
        uint64_t bytes;
        if (v.flags & OMC_VAR_QUANTIZED) {
            if (!format_ok(v.fmt)) return OMC_ERR_PLAN;
            ++nq;
            if (v.n == 0 || v.n > kMaxElems) return OMC_ERR_PLAN;
            bytes = packed_bytes_u(1u + v.fmt.exp_bits + v.fmt.man_bits, v.n);
        } else {
            if (v.n == 0 || v.n > kMaxElems) return OMC_ERR_PLAN;
            bytes = align_up(4 * v.n, 16);
        }
        if (v.data_offset != next) return OMC_ERR_PLAN;         // the payload is dense, in table order
        next += bytes;
        vars_out[i] = v;
    }
    if (next != th->payload_bytes || nq != th->nquant) return OMC_ERR_PLAN;
    if (transport_header_hash(*th, sum) != th->checksum) return OMC_ERR_PLAN;
    return OMC_OK;
}

}  // extern "C"
