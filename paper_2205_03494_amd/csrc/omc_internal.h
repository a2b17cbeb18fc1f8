// Shared host/device declarations of libomc (not part of the public ABI).
#pragma once
#include <stdint.h>
#include <stddef.h>
#include "omc.h"

namespace omc {

// Work decomposition of the streaming kernels.  One wavefront owns one tile at a time:
// 64 lanes x 32 consecutive elements.  32 elements of a B-bit format are exactly B dwords, so a
// lane's share of the packed stream is B whole dwords for every B and no dword is shared
// between lanes, tiles or variables.
constexpr int kLaneElems = 32;
constexpr int kTileElems = 64 * kLaneElems;           // 2048
#ifndef OMC_TUNE_TILES_PER_CHUNK
#define OMC_TUNE_TILES_PER_CHUNK 2
#endif
constexpr int kTilesPerChunk = OMC_TUNE_TILES_PER_CHUNK;   // tiles reduced into one partial
constexpr int kChunkElems = kTileElems * kTilesPerChunk;   // an fp32 variable's work item
// Tiles per work item of a quantized variable, by code width (measured: 6-bit kernels do better with
// four, all others with two).  Host and device agree on it through this one function.
__host__ __device__ constexpr uint32_t tiles_per_chunk(uint32_t bits) { return bits == 6 ? 2u * kTilesPerChunk : kTilesPerChunk; }
constexpr uint32_t kMinTilesPerChunk = kTilesPerChunk;
constexpr int kLdsDwords = kTileElems + kTileElems / 32;  // padded code tile for B = 32

// Constants derived from a format once on the host; uniform per variable (scalar registers).
struct FmtParams {
    uint32_t bits;           // B = 1 + E + M
    uint32_t exp_bits;       // E
    uint32_t man_bits;       // M
    uint32_t bias;
    uint32_t sh;             // 23 - M: fp32 mantissa bits below the format's mantissa
    uint32_t asr;            // 8 - E
    uint32_t keep_mask;      // fp32 bit positions that carry [sign | e | m] after alignment
    uint32_t min_norm_bits;  // fp32 bit pattern of 2^(1 - bias), the smallest normal
    uint32_t magic_off;      // (23 - M) << 23
    uint32_t wide;           // 1: round with ldexp/rint (top binade + 23 - M would overflow fp32, or M == 23)
    uint32_t variant;        // kernel variant: 0 add/subtract rounding, 1 = wide, 2 = the format is OCP FP8 E4M3
                             // except for its top code (S1E4M3, bias 7), 3 = the format is the OCP microscaling
                             // 6-bit E2M3 element (S1E2M3, bias 1): hardware conversions apply; 4 / 5 = 0 / 1
                             // with the fit's sums carried as (sum, error) pairs (16 or more mantissa bits)
    int32_t exp_adj;         // 127 + M
    float dec_scale;         // 2^(127 - bias)
    float enc_scale;         // 2^(bias - 127)
    float maxval;            // largest representable magnitude
};

// Kernel variants 4 and 5 (see FmtParams::variant).
constexpr uint32_t kVariantExact = 4;
__host__ __device__ constexpr bool variant_exact(uint32_t variant) { return variant >= kVariantExact; }
__host__ __device__ constexpr bool variant_wide(uint32_t variant) { return variant == 1 || variant == 5; }
constexpr uint32_t kVariants = 6;

// Per-chunk partial sums of the least-squares fit (paper Sec. 2.3).  The four sums are unevaluated
// pairs s + l: the kernels of formats with fewer than 16 mantissa bits leave l = 0, the others carry
// the rounding errors of their additions there (see FitAcc).
struct Partial {
    double sV, sT, sVT, sTT;
    double lV, lT, lVT, lTT;
    float tmin, tmax;
    uint32_t pad[2];
};
static_assert(sizeof(Partial) == 80, "Partial layout");

// ---- plan blob ---------------------------------------------------------------------------
constexpr uint32_t kPlanMagic = 0x434d4f50u;  // "POMC"
constexpr uint32_t kPlanVersion = 6;

struct PlanHeader {
    uint32_t magic, version;
    uint32_t nvars, nitems, ngroups, nquant;
    uint64_t total_bytes;
    uint64_t var_off, item_off, group_off;  // byte offsets of the three tables inside the blob
    uint64_t arena_bytes;                   // extent of the arena the plan addresses
    uint64_t aux_elems;                     // extent of grads / state
    uint64_t ws_bytes;
    uint64_t checksum;                      // over everything after the header
};

struct PlanVar {
    uint64_t data_offset, aux_offset, n;
    uint64_t total_dwords;   // packed buffer length in dwords (multiple of 4); 0 for fp32
    uint32_t flags;          // OMC_VAR_*
    uint32_t first_item;     // index of this variable's first full-tile work item / partial
    uint32_t nitems;         // number of those (0 when n < 2048)
    uint32_t tail_item;      // index of the ragged-tail item / partial, kNoItem if n % 2048 == 0
    FmtParams fp;
    uint32_t sb_index;       // entry of the (s, b) table that belongs to this variable (its own index in a plan
                             // built from a caller's table; the index in the original set for derived plans)
};
static_assert(sizeof(PlanVar) == 112, "PlanVar layout");

struct PlanItem {
    uint32_t var;
    uint32_t chunk;
};

constexpr uint32_t kNoItem = 0xffffffffu;

// One kernel launch: a run of work items that the same kernel instance serves.
enum GroupKind : uint32_t { kGroupFull = 0, kGroupTail = 1, kGroupFp32 = 2 };
struct PlanGroup {
    uint32_t kind;           // GroupKind
    uint32_t bits;           // kGroupFull: code width of the group's variables
    uint32_t wide;           // kGroupFull: FmtParams::variant, kGroupTail: FmtParams::wide of the group's variables
    uint32_t first_item;
    uint32_t nitems;
    uint32_t pad;
};

// ---- aggregation plan blob (server side: R clients' copies of one variable set) ---------------
constexpr uint32_t kAggMagic = 0x47414d4fu;  // "OMAG"
constexpr uint32_t kAggVersion = 2;
constexpr uint32_t kMaxReplicas = 16;

struct AggHeader {
    uint32_t magic, version;
    uint32_t nvars, nitems, ngroups, nreplicas;
    uint64_t total_bytes;
    uint64_t var_off, src_off, item_off, group_off;
    uint64_t aux_elems;
    uint64_t arena_bytes[kMaxReplicas];     // extent each client's arena must have
    uint64_t checksum;                      // over everything after the header
    uint64_t pad;
};

struct AggVar {
    uint64_t aux_offset, n;
    uint64_t total_dwords;   // packed length of the variable where it is quantized; 0: fp32 at every client
    FmtParams fp;            // the one format every quantizing client uses for this variable
};

struct AggSrc {              // one per (variable, client), variable-major
    uint64_t data_offset;    // into that client's arena
    uint32_t quantized;
    uint32_t pad;
};

// groups reuse PlanGroup: kGroupFull (bits) = full tiles of variables quantized somewhere,
// kGroupTail = their ragged tails, kGroupFp32 = variables that are fp32 at every client

// ---- reselection blob (Sec. 2.5: the set of quantized variables changes from round to round) ----
// Two derived plans over (old arena -> new arena): one whose "values" are the old arena (variables that
// become quantized are compressed from there, unchanged variables are copied as runs of floats), one
// whose "output" is the new arena (variables that become fp32 are decompressed into it).
constexpr uint32_t kReselectMagic = 0x53524d4fu;  // "OMRS"
constexpr uint32_t kReselectVersion = 1;
enum ReselectAction : uint32_t { kRsCopyQuantized = 0, kRsCopyFp32 = 1, kRsToQuantized = 2, kRsToFp32 = 3 };
struct ReselectHeader {
    uint32_t magic, version;
    uint32_t nvars, pad;
    uint64_t total_bytes;
    uint64_t action_off;                    // nvars x uint32 ReselectAction
    uint64_t plan_c_off, plan_c_bytes;      // derived plan run through the compress-set kernels (0: none)
    uint64_t plan_d_off, plan_d_bytes;      // derived plan run through the decompress-set kernels (0: none)
    uint64_t arena_old_bytes, arena_new_bytes;
    uint64_t ws_bytes;
    uint64_t algorithmic_bytes;             // bytes the conversion must move
    uint64_t checksum;                      // over everything after the header
};

// ---- transport message (Sec. 1: parameters are kept and transported in compressed form) ----------
// [TransportHeader | nvars x TransportVar | pad to 256 | (s, b) table: nvars x 2 floats | pad to 256 | payload]
// The payload holds every variable's packed stream or fp32 values back to back at 16-byte aligned
// offsets, so the message body is itself an arena + (s, b) table for the plan built from its table.
constexpr uint32_t kTransportMagic = 0x54584d4fu;  // "OMXT"
constexpr uint32_t kTransportVersion = 1;
struct TransportHeader {
    uint32_t magic, version;
    uint32_t nvars, nquant;
    uint64_t total_bytes;                   // whole message
    uint64_t sb_off, payload_off, payload_bytes;
    uint64_t aux_elems;
    uint64_t checksum;                      // over the header fields above and the variable table
};
static_assert(sizeof(TransportHeader) == 64, "TransportHeader layout");
struct TransportVar {
    uint64_t payload_offset;                // bytes from payload_off, multiple of 16
    uint64_t aux_offset;
    uint64_t n;
    uint8_t exp_bits, man_bits;
    int16_t exp_bias;                       // resolved bias
    uint32_t flags;                         // OMC_VAR_*
};
static_assert(sizeof(TransportVar) == 32, "TransportVar layout");
__host__ __device__ inline uint64_t transport_mix(uint64_t h, uint64_t w) {
    h = (h ^ w) * 0x100000001b3ull;
    return (h << 29) | (h >> 35);
}
// order-independent part of the checksum: one term per variable, summed (wrapping)
__host__ __device__ inline uint64_t transport_var_hash(uint32_t index, const TransportVar &v) {
    uint64_t h = 0x9e3779b97f4a7c15ull + index;
    h = transport_mix(h, v.payload_offset);
    h = transport_mix(h, v.aux_offset);
    h = transport_mix(h, v.n);
    h = transport_mix(h, static_cast<uint64_t>(v.exp_bits) | (static_cast<uint64_t>(v.man_bits) << 8) |
                             (static_cast<uint64_t>(static_cast<uint16_t>(v.exp_bias)) << 16) |
                             (static_cast<uint64_t>(v.flags) << 32));
    return h;
}
__host__ __device__ inline uint64_t transport_header_hash(const TransportHeader &h, uint64_t var_sum) {
    uint64_t x = 0xc2b2ae3d27d4eb4full;
    x = transport_mix(x, static_cast<uint64_t>(h.nvars) | (static_cast<uint64_t>(h.nquant) << 32));
    x = transport_mix(x, h.total_bytes);
    x = transport_mix(x, h.sb_off);
    x = transport_mix(x, h.payload_off);
    x = transport_mix(x, h.payload_bytes);
    x = transport_mix(x, h.aux_elems);
    return transport_mix(x, var_sum);
}
constexpr uint64_t kTransportAlign = 256;

// ---- host helpers (omc_host.cpp) -----------------------------------------------------------
bool make_fmt_params(omc_format f, FmtParams *out);
const PlanHeader *plan_check(const void *plan_host);

// ---- launchers, one translation unit each (device code) -----------------------------------
// Arguments already validated.  Return hipError_t as int.
struct VarArgs {
    uint64_t n;
    uint64_t total_dwords;
    FmtParams fp;
};

uint32_t single_tiles_per_item(uint32_t bits, uint64_t n);
int launch_compress(const float *v, const VarArgs &va, int use_pvt, void *codes, float *sb,
                    Partial *ws, void *stream);
// Size of the library's own device scratch array (omc_compress_noalloc) and the address of the current
// device's copy of it (looked up once per device); returns a hipError_t as int.
constexpr size_t kStaticScratchBytes = 2u << 20;
int static_scratch(void **ptr_out);
int launch_decompress(const void *codes, const VarArgs &va, const float *sb, float *out, void *stream);
int launch_compress_set(const float *values, const PlanHeader *ph, const void *plan_dev, void *arena,
                        float *sb_table, Partial *ws, void *stream);
int launch_decompress_set(const void *arena, const PlanHeader *ph, const void *plan_dev, const float *sb_table,
                          float *out, void *stream);
int launch_step(void *arena, const PlanHeader *ph, const void *plan_dev, float *sb_table,
                const float *grads, float *state0, float *state1, const omc_opt &opt, Partial *ws,
                void *stream, void *const *events);
int launch_reselect_sb(const uint32_t *actions_dev, uint32_t nvars, const float *sb_old, float *sb_new, void *stream);
int launch_transport_pack(const PlanHeader *ph, const void *plan_dev, const void *arena, const float *sb_table,
                          void *msg_dev, const TransportHeader &th, void *stream);
struct DwConfig {
    uint32_t rows;     // weight rows per tile: 256 or 128
    uint32_t nsplit;   // workgroups per tile along the contraction
    uint32_t ws;       // 1: the 16-wave kernel with separate multiplying and staging waves (rows = 256, always parks)
};
DwConfig dw_config(uint32_t M, uint32_t N, uint32_t K);
size_t dw_workspace_bytes(uint32_t bits, uint32_t M, uint32_t N, uint32_t K);
int launch_dw_update(const uint16_t *X, const uint16_t *dY, void *codes, const FmtParams &fp, float *sb, int use_pvt,
                     float *state0, float *state1, const omc_opt &opt, float *dW_out, uint32_t M, uint32_t N,
                     uint32_t K, void *ws, void *stream);
struct AggPointers {
    const uint8_t *arena[kMaxReplicas];
    const float *sb[kMaxReplicas];
};
int launch_aggregate_mean(const AggHeader *ah, const void *agg_dev, const AggPointers &ptrs, float *out, void *stream);
int launch_dequant_gemm(const uint16_t *A, const void *codes, const FmtParams &fp, const float *sb,
                        float *C, uint32_t M, uint32_t N, uint32_t K, float *ws, int trans, void *stream);

}  // namespace omc
