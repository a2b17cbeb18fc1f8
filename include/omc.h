/*
 * omc.h -- C ABI of libomc: the per-iteration hot path of Online Model Compression (OMC,
 * arxiv 2205.03494) on one AMD MI355X (gfx950).
 *
 * The method keeps model variables in a reduced-bitwidth floating-point format, decompresses
 * them when an operation needs them, and recompresses them after every training iteration
 * (paper Sec. 2.1).  This library is that cycle:
 *
 *   omc_compress                 fp32 variable -> packed codes + per-variable (s, b)   (Sec. 2.2, 2.3)
 *   omc_decompress               packed codes + (s, b) -> fp32                           (Sec. 2.1, 2.3)
 *   omc_step_update_recompress   one training iteration over a whole variable set:
 *                                decompress -> parameter update -> recompress, fused     (Sec. 2.1, backward path)
 *   omc_dequant_gemm             C = A * decompress(W), weights expanded on chip          (Sec. 2.1, forward path)
 *   omc_dequant_gemm_dx          dX = dY * decompress(W)^T                                (Sec. 2.1, backward path)
 *   omc_dw_update_recompress     dW = X^T dY consumed by the update in the GEMM's epilogue  (Sec. 2.1, backward path)
 *   omc_aggregate_mean           server: mean of R clients' mixed-precision copies        (Sec. 1, 2.5)
 *   omc_reselect                 a new round's quantized subset without a full-precision copy (Sec. 2.5)
 *   omc_transport_pack / _open   the packed set as one self-describing message / checkpoint  (Sec. 1)
 *
 * Conventions that hold for every entry point
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     process memory.  The library allocates nothing, frees nothing and keeps no pointer after
 *     a call returns.  There is no global state (with the one exception stated at
 *     omc_compress_noalloc); calls on different streams may overlap as long as their buffers do not.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     on it and the call returns without synchronising.
 *   - Arguments are validated on the host before anything is enqueued: every status other than
 *     OMC_OK and OMC_ERR_DEVICE means that no kernel was launched and no buffer was touched.
 *     OMC_ERR_DEVICE is the HIP runtime refusing a launch; a call that needs several launches may
 *     then already have enqueued the earlier ones, so the buffers it writes are undefined.
 *   - Device buffers of packed codes, fp32 values, gradients and optimizer state must be
 *     16-byte aligned (OMC_ERR_ALIGN otherwise).
 *
 * Format (Sec. 2.2; notation SxEyMz of Sec. 3.1, x = 1).  A code has B = 1 + E + M bits,
 * most significant first [sign | e : E bits | m : M bits].
 *     e == 0 :  value = (-1)^sign * 2^(1-bias)   * (m / 2^M)          zero and subnormals
 *     e >= 1 :  value = (-1)^sign * 2^(e-bias)   * (1 + m / 2^M)      every other exponent, the top one included
 * There are no Inf/NaN codes.  bias defaults to 2^(E-1)-1.  Conversion from fp32 rounds to the
 * nearest value, ties to the even integer significand, and saturates at the largest magnitude.
 * Codes whose value would exceed the largest finite fp32 (possible only when 2^E-1-bias > 127,
 * i.e. E = 8) are never produced and must not be fed to the decoder.  Non-finite inputs encode
 * to the saturated code of their sign and make the variable's (s, b) NaN.
 *
 * Packing.  A variable of n elements is a dense little-endian bit stream: element k occupies
 * stream bits [k*B, (k+1)*B), least significant code bit first; stream bit i is bit (i mod 32) of
 * the little-endian 32-bit word i/32.  The buffer is omc_packed_bytes(f, n) long: the stream padded
 * with zero bits to a multiple of 16 bytes.  This is also the transport form of a variable.
 *
 * Per-variable transformation (Sec. 2.3).  The decompressed value of element k is
 *     Vbar_k = fl32( fl32(s * Vtilde_k) + b )
 * with Vtilde_k the value of its code and (s, b) two fp32 numbers per variable.  At compression
 * (s, b) minimise || s*Vtilde + b*1 - V ||_2 over the n elements:
 *     s = (n SUM V Vt - SUM V SUM Vt) / (n SUM Vt^2 - (SUM Vt)^2),   b = (SUM V - s SUM Vt) / n,
 * evaluated in fp64 and stored as fp32; s = 1 when all Vtilde_k are equal (the degenerate case).
 * The four sums are accumulated in a fixed order, so results are bit-identical from run to run:
 * in fp64 for formats of fewer than 16 mantissa bits (every term is exact; the additions round, which
 * moves the fp32 result only if it lies within ~1e-16 of a rounding boundary), and in fp64 with the
 * rounding error of every addition carried along (about 106 bits) for man_bits >= 16, where b is a
 * difference of nearly equal sums and plain fp64 additions would show in its last bits.
 */
#ifndef OMC_H
#define OMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OMC_OK = 0,
    OMC_ERR_NULL = 1,      /* a required pointer is NULL */
    OMC_ERR_FORMAT = 2,    /* exp_bits / man_bits / bias outside the supported range */
    OMC_ERR_SIZE = 3,      /* n == 0, a dimension is 0 or not a supported multiple, offsets overlap or run past a buffer */
    OMC_ERR_ALIGN = 4,     /* a device pointer or an offset is not aligned as required */
    OMC_ERR_WORKSPACE = 5, /* workspace missing or smaller than the queried size */
    OMC_ERR_OPT = 6,       /* unknown optimizer kind, or a state buffer it needs is NULL */
    OMC_ERR_DEVICE = 7,    /* the HIP runtime refused a launch */
    OMC_ERR_PLAN = 8       /* the plan blob is corrupt or does not belong to this call */
} omc_status;

/* SxEyMz with x = 1 (Sec. 2.2).  1 <= exp_bits <= 8, 0 <= man_bits <= 23,
 * exp_bias in [0, 127] or OMC_BIAS_DEFAULT. */
#define OMC_BIAS_DEFAULT (-1)
typedef struct {
    uint8_t exp_bits;
    uint8_t man_bits;
    int16_t exp_bias;
} omc_format;

/* One variable of a set (Sec. 2.4, 2.5: weight matrices may be quantized, everything else and
 * the matrices not selected by partial parameter quantization stay fp32). */
#define OMC_VAR_QUANTIZED 1u /* packed codes at data_offset; otherwise n fp32 values */
#define OMC_VAR_NO_PVT 2u    /* keep (s, b) = (1, 0): quantization without the transformation */
typedef struct {
    uint64_t data_offset; /* bytes into the arena; multiple of 16 */
    uint64_t aux_offset;  /* fp32 elements into grads / state0 / state1; multiple of 4 */
    uint64_t n;           /* elements, >= 1 */
    omc_format fmt;       /* ignored unless OMC_VAR_QUANTIZED */
    uint32_t flags;       /* OMC_VAR_* */
} omc_var;

/* The parameter update applied to the decompressed values (Sec. 2.1, backward path; the paper does
 * not name the client optimizer).  Every fp32 operation is rounded
 * on its own, in the order written:
 *   OMC_SGD       V' = V - fl(lr*g)
 *   OMC_MOMENTUM  m' = fl(fl(momentum*m) + g);                       V' = V - fl(lr*m')         state0 = m
 *   OMC_ADAM      m' = fl(fl(beta1*m) + fl(one_minus_beta1*g))
 *                 v' = fl(fl(beta2*v) + fl(fl(one_minus_beta2*g)*g))
 *                 V' = V - fl( fl(lr*fl(m'/bias_corr1)) / fl(fl(sqrt(fl(v'/bias_corr2))) + eps) )
 *                                                                         state0 = m, state1 = v
 * one_minus_beta* = fp32(1 - beta*) and bias_corr* = fp32(1 - beta*^t) are computed by the caller
 * in fp64 and rounded once.
 * flags choose the cache policy of the packed codes, which every step reads and rewrites in place; they
 * change memory traffic only, never a value.
 *   default (0)           a training loop runs a forward and a backward pass between two update steps
 *                         (Sec. 2.1), so nothing of the codes is left in the GPU's 256 MB memory-side
 *                         cache when the next step starts: all code accesses carry the non-temporal hint
 *                         and stream past the caches, like gradients and optimizer state always do.
 *   OMC_OPT_STREAM_CODES  names the default explicitly (accepted, no effect).
 *   OMC_OPT_KEEP_CODES    for callers that run steps back to back with nothing in between (benchmarks,
 *                         several optimizer steps per gradient): the first 224 MiB of codes (all of them
 *                         up to 264 MiB) are accessed with ordinary cached loads and stores, so that they
 *                         come back from the memory-side cache at the next step
 *                         (see omc_step_update_recompress_events).
 * Both bits together, or unknown bits, are OMC_ERR_OPT. */
typedef enum { OMC_SGD = 0, OMC_MOMENTUM = 1, OMC_ADAM = 2 } omc_opt_kind;
#define OMC_OPT_STREAM_CODES 1u
#define OMC_OPT_KEEP_CODES 2u
typedef struct {
    int32_t kind; /* omc_opt_kind */
    float lr;
    float momentum;
    float beta1, beta2, eps;
    float one_minus_beta1, one_minus_beta2;
    float bias_corr1, bias_corr2;
    uint32_t flags; /* OMC_OPT_* */
} omc_opt;

/* ---- host-only helpers (no device work) ------------------------------------------------- */

const char *omc_status_string(omc_status s);

/* OMC_OK or OMC_ERR_FORMAT. */
omc_status omc_format_validate(omc_format f);

/* Bits per code, 1 + E + M; 0 for an invalid format. */
uint32_t omc_format_bits(omc_format f);

/* Largest representable magnitude (exact in fp32); 0 for an invalid format. */
float omc_format_max(omc_format f);

/* Bytes of the packed buffer of n elements: ceil(n*B/8) rounded up to a multiple of 16;
 * 0 for an invalid format or n == 0. */
size_t omc_packed_bytes(omc_format f, uint64_t n);

/* Workspace (device bytes) that omc_compress needs for n elements. */
size_t omc_compress_workspace_bytes(uint64_t n);

/* ---- single variable --------------------------------------------------------------------- */

/* Compress n fp32 values (Sec. 2.2 quantization, Sec. 2.3 fit).
 *   v        device, n floats, read only
 *   codes    device, omc_packed_bytes(f, n) bytes, written completely (padding bits zero)
 *   sb       device, 2 floats: receives s, b ((1, 0) when use_pvt == 0)
 *   ws       device workspace of at least omc_compress_workspace_bytes(n) bytes, 16-byte aligned;
 *            contents undefined afterwards
 * v and codes must not overlap. */
omc_status omc_compress(const float *v, uint64_t n, omc_format f, int use_pvt, void *codes,
                        float *sb, void *ws, size_t ws_bytes, void *stream);

/* omc_compress for callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc -- and so cannot bring a workspace: the partial sums of
 * the fit go to a 2 MiB device array that is part of the library image (each GPU the library runs on
 * holds its own copy until the process ends).  Same arguments, same results bit for bit as omc_compress;
 * v, codes and sb are still the caller's.  The call allocates and frees nothing (its first use on a
 * device looks the array's address up once).
 *   n        at most omc_compress_noalloc_max_elems() (107 368 448), OMC_ERR_SIZE beyond
 * This is the one piece of state the library keeps: all calls on one GPU share that GPU's array, so two
 * such calls must not overlap in time on the same GPU (different streams, different threads): they would
 * race on the partial sums.  Calls on one stream, one after the other, are fine; nothing is carried over
 * from one call to the next.  The array belongs to the device that is current when the call is made,
 * which must be the device of `stream` and of the buffers. */
uint64_t omc_compress_noalloc_max_elems(void);
omc_status omc_compress_noalloc(const float *v, uint64_t n, omc_format f, int use_pvt, void *codes,
                                float *sb, void *stream);

/* Decompress n elements: out_k = fl32(fl32(s*Vtilde_k) + b)  (Sec. 2.1, 2.3).
 *   codes    device, omc_packed_bytes(f, n) bytes, read only
 *   sb       device, 2 floats (s, b), or NULL for s = 1, b = 0 (then out_k = Vtilde_k exactly)
 *   out      device, n floats */
omc_status omc_decompress(const void *codes, uint64_t n, omc_format f, const float *sb, float *out,
                          void *stream);

/* ---- variable set: the per-iteration cycle ---------------------------------------------- */

/* A plan is a position-independent blob that describes a variable set to the kernels: the
 * validated variable table, derived format constants and the list of work items.  It is built on
 * the host once per variable set (and again whenever the set of quantized variables changes,
 * Sec. 2.5); the caller copies the same bytes to device memory and passes both copies to every
 * step.
 *
 * omc_plan_bytes: size of the blob, 0 if the table is invalid (see omc_plan_build for the reason).
 * omc_plan_build: validates the table (formats, n >= 1, alignment of offsets, no two variables
 *   overlapping in the arena or in the aux range) and fills plan_host[0 .. plan_bytes).
 * omc_plan_workspace_bytes / omc_plan_arena_bytes / omc_plan_aux_elems: device workspace a step
 *   needs, and the extent of arena / aux that the plan addresses (0 for a corrupt blob).
 * omc_workspace_bytes: the same workspace size straight from a variable table (0 if invalid). */
size_t omc_plan_bytes(const omc_var *vars_host, uint32_t nvars);
omc_status omc_plan_build(const omc_var *vars_host, uint32_t nvars, void *plan_host, size_t plan_bytes);
size_t omc_plan_workspace_bytes(const void *plan_host);
size_t omc_workspace_bytes(const omc_var *vars_host, uint32_t nvars);
size_t omc_plan_arena_bytes(const void *plan_host);
uint64_t omc_plan_aux_elems(const void *plan_host);

/* One training iteration over the whole set (Sec. 2.1 backward path, with Sec. 2.4 / 2.5 deciding
 * which variables are packed).  For every quantized variable: unpack, decode, apply (s, b), apply
 * the update with the variable's gradient and optimizer state, round to the format, refit (s, b)
 * against the updated full-precision values, pack.  The decompressed copy lives in registers only.
 * For every fp32 variable: the update alone.  Everything is in place.
 *   arena        device, arena_bytes bytes: packed codes and fp32 values at the plan's data offsets
 *   plan_host    host copy of the plan blob;  plan_dev: device copy of the same bytes
 *   sb_table     device, 2*nvars floats: (s, b) per variable, read and rewritten for quantized
 *                variables, untouched for the others
 *   grads        device, aux_elems floats, read only
 *   state0/1     device, aux_elems floats each; state0 needed for OMC_MOMENTUM and OMC_ADAM,
 *                state1 for OMC_ADAM; otherwise ignored (may be NULL)
 *   ws           device workspace, at least omc_plan_workspace_bytes(plan_host), 16-byte aligned
 * arena_bytes and aux_elems must be at least what the plan addresses (OMC_ERR_SIZE otherwise). */
omc_status omc_step_update_recompress(void *arena, size_t arena_bytes, const void *plan_host,
                                      const void *plan_dev, float *sb_table, const float *grads,
                                      float *state0, float *state1, uint64_t aux_elems,
                                      const omc_opt *opt, void *ws, size_t ws_bytes, void *stream);

/* Whole-set conversion between fp32 and the plan's storage (the start and the end of a round: a
 * client receives or returns a model; Sec. 2.5 lets the set of quantized variables change from
 * round to round, which is a decompress with the old plan followed by a compress with the new one).
 *   omc_compress_set     for every quantized variable of the plan: compress the n floats at
 *                        values[aux_offset ..] into the arena and write its (s, b); for every fp32
 *                        variable: copy its floats into the arena.  Bit-identical to calling
 *                        omc_compress per variable.
 *   omc_decompress_set   the reverse: out[aux_offset ..] = decompressed values (or the fp32 copy).
 * values / out: device, aux_elems floats (at least what the plan addresses), must not overlap the
 * arena.  ws as for the step.  sb_table: device, 2*nvars floats.
 *   omc_plan_transport_bytes   bytes that represent the variable set in storage or on the wire
 *                        (Sec. 1: communication cost equals parameter memory): packed buffer plus
 *                        8 bytes of (s, b) per quantized variable, 4n per fp32 variable. */
omc_status omc_compress_set(const float *values, uint64_t aux_elems, const void *plan_host, const void *plan_dev,
                            void *arena, size_t arena_bytes, float *sb_table, void *ws, size_t ws_bytes,
                            void *stream);
omc_status omc_decompress_set(const void *arena, size_t arena_bytes, const void *plan_host, const void *plan_dev,
                              const float *sb_table, float *out, uint64_t aux_elems, void *stream);
uint64_t omc_plan_transport_bytes(const void *plan_host);

/* ---- a new round with another quantized subset (Sec. 2.5) ----------------------------------------
 * Partial parameter quantization picks the variables to quantize anew for every round and every client.
 * omc_reselect converts a set from the old selection (plan_old, its arena and (s, b) table) to the new one
 * (plan_new, another arena and table) in one pass and without a full-precision copy of the model:
 *   - a variable that becomes quantized is compressed straight from its fp32 values in the old arena
 *     into the new arena (Sec. 2.2, 2.3: codes and a fresh (s, b));
 *   - a variable that becomes fp32 is decompressed straight from its codes into the new arena;
 *   - every other variable is moved as bytes (its codes and (s, b), or its fp32 values), untouched.
 * Results are bit-identical to omc_decompress / omc_compress applied to the switched variables alone.
 * The two plans must list the same variables (count and sizes); a variable quantized in both must keep
 * its format (OMC_ERR_FORMAT otherwise: changing the format of codes is a decompress + compress).
 *
 * omc_reselect_plan_bytes / _build: host only; derive the conversion's own blob from the two host plans
 *   (position independent; the caller copies it to the device, 16-byte aligned).
 * omc_reselect_workspace_bytes, omc_reselect_algorithmic_bytes: device workspace of the call, and the bytes
 *   the conversion has to move (2 x size of every moved variable, 4n + packed size of every converted one).
 * omc_reselect:
 *   arena_old, sb_old   device: the set under plan_old (read only)
 *   arena_new, sb_new   device: receive the set under plan_new; must not overlap the old ones
 *   ws                  device workspace of omc_reselect_workspace_bytes(rs_host) bytes */
size_t omc_reselect_plan_bytes(const void *plan_old_host, const void *plan_new_host);
omc_status omc_reselect_plan_build(const void *plan_old_host, const void *plan_new_host, void *rs_host,
                                   size_t rs_bytes);
size_t omc_reselect_workspace_bytes(const void *rs_host);
uint64_t omc_reselect_algorithmic_bytes(const void *rs_host);
omc_status omc_reselect(const void *rs_host, const void *rs_dev, const void *arena_old, size_t arena_old_bytes,
                        const float *sb_old, void *arena_new, size_t arena_new_bytes, float *sb_new, void *ws,
                        size_t ws_bytes, void *stream);

/* ---- transport / checkpoint message (Sec. 1) ------------------------------------------------------
 * The paper keeps and transports parameters in compressed form: what a client sends back, what the server
 * sends out and what a checkpoint holds is the packed set itself.  omc_transport_pack serialises a set into
 * one self-describing buffer
 *     [ header | variable table | (s, b) table, 2 floats per variable | payload ]
 * whose payload holds every variable's packed stream (or fp32 values) back to back at 16-byte aligned
 * offsets, in table order.  Its size, omc_transport_bytes(plan), is omc_plan_transport_bytes(plan) plus the
 * header and table, 8 bytes per fp32 variable (the (s, b) table has an entry for every variable) and
 * alignment padding.  The message needs no unpacking: omc_transport_open validates the header and table
 * (magic, version, sizes, dense payload, checksum; OMC_ERR_PLAN otherwise) and returns an omc_var table
 * whose data offsets are relative to the payload, so that the receiver builds a plan from it and uses the
 * message body in place as arena (msg + arena_offset) and (s, b) table (msg + sb_offset).
 *   omc_transport_meta_bytes   size of header + variable table: the prefix of the message that
 *                              omc_transport_open needs in host memory
 *   omc_transport_pack         device to device; msg_dev 16-byte aligned, at least omc_transport_bytes long,
 *                              not overlapping the arena
 *   omc_transport_open         host only.  vars_out == NULL: only *nvars_out and the offsets are returned
 *                              (prefix of at least 64 bytes); otherwise the prefix must hold the whole table and
 *                              vars_cap >= nvars (OMC_ERR_SIZE).  Optimizer state is not part of the message: it
 *                              is the caller's own fp32 arrays. */
size_t omc_transport_meta_bytes(uint32_t nvars);
uint64_t omc_transport_bytes(const void *plan_host);
omc_status omc_transport_pack(const void *plan_host, const void *plan_dev, const void *arena, size_t arena_bytes,
                              const float *sb_table, void *msg_dev, size_t msg_bytes, void *stream);
omc_status omc_transport_open(const void *msg_prefix_host, size_t prefix_bytes, uint64_t msg_bytes,
                              omc_var *vars_out, uint32_t vars_cap, uint32_t *nvars_out, uint64_t *sb_offset,
                              uint64_t *arena_offset, uint64_t *arena_bytes, uint64_t *aux_elems);

/* Measurement aid.  Same work as omc_step_update_recompress; additionally records caller-owned HIP
 * events (hipEvent_t passed as void*) on the stream around every kernel launch, so that a
 * benchmark can time each kernel by itself: events[2k] before and events[2k+1] after the k-th
 * launch.  Launch order: the full-tile kernels, one per distinct code width among the quantized
 * variables of at least 2048 elements, in ascending width (two for a width whose formats need
 * both rounding variants: formats with man_bits == 23 or a top binade of 2^(105+man_bits) or more
 * use the second), the first of them also serving the fp32 variables as extra workgroups; then
 * up to two kernels for the ragged tails (n % 2048 != 0) of quantized variables; then, only if no
 * full-tile kernel ran, one kernel for the fp32 variables; then the per-variable
 * finalize, if any variable is quantized.  omc_plan_launches gives the count; nevents must be at
 * least twice that (OMC_ERR_SIZE otherwise).  Results are identical to the plain call.
 * Under OMC_OPT_KEEP_CODES a full-tile kernel may be enqueued as two launches, one event pair around
 * both: packed codes are read and rewritten in place by every step, so when a set holds more than 264 MiB of them, the
 * work items holding the first 224 MiB (in launch order) access their codes with ordinary cached
 * loads and stores, which lets them come back from the GPU's 256 MB memory-side cache at the
 * next step, and the work items after that limit access theirs with the non-temporal hint so that
 * they do not push the first ones out.  Gradients and optimizer state always carry the hint; the
 * values of fp32 variables share what the codes leave of the 224 MiB under OMC_SGD and carry the
 * hint otherwise.  Values are the same either way. */
uint32_t omc_plan_launches(const void *plan_host);
omc_status omc_step_update_recompress_events(void *arena, size_t arena_bytes, const void *plan_host,
                                             const void *plan_dev, float *sb_table, const float *grads,
                                             float *state0, float *state1, uint64_t aux_elems,
                                             const omc_opt *opt, void *ws, size_t ws_bytes, void *stream,
                                             void *const *events, uint32_t nevents);

/* ---- server-side aggregation ------------------------------------------------------------- */

/* The server's end of a federated round (Sec. 1: the clients' trained models are transported back and
 * aggregated; Sec. 2.5: every client quantizes its own subset of the variables, so one variable
 * arrives as codes + (s, b) from some clients and in fp32 from others).  The paper leaves the
 * aggregation itself open; this is the plain federated average with equal weights,
 *     out[i] = ( ... ((v_0[i] + v_1[i]) + v_2[i]) ... + v_{R-1}[i] ) / R,
 * over the clients' decompressed values, clients in index order, fp32, each operation rounded once.
 *
 * Each client r hands over what omc_compress_set / the training steps produced: its plan, arena and
 * (s, b) table.  The plans must describe the same variable list (count, sizes, aux offsets) and
 * agree on the format of every variable among the clients that quantize it; data offsets and the
 * quantized subsets may differ freely.  At most OMC_MAX_REPLICAS clients per call.
 *
 * omc_aggregate_plan_bytes / _build: host only; merge the R host plans into an aggregation plan
 * (position independent; the caller copies it to the device).  0 / an error status for plans that do
 * not fit together (OMC_ERR_PLAN, OMC_ERR_SIZE, OMC_ERR_FORMAT).
 *
 * omc_aggregate_mean:
 *   agg_host, agg_dev   the aggregation plan in host memory and its device copy (16-byte aligned)
 *   arenas, sb_tables   host arrays of R device pointers: client r's arena (arena_bytes[r] bytes, at
 *                       least what its plan addresses) and (s, b) table (2 floats per variable)
 *   out                 device, aux_elems floats, variable v at its aux_offset; the server model in
 *                       full precision (omc_compress_set packs it for the next round)
 * Inputs are read once, in the form they arrived in; nothing is written but out.  The library
 * allocates nothing; launches go to `stream`. */
#define OMC_MAX_REPLICAS 16
size_t omc_aggregate_plan_bytes(const void *const *plans_host, uint32_t nreplicas);
omc_status omc_aggregate_plan_build(const void *const *plans_host, uint32_t nreplicas, void *agg_host,
                                    size_t agg_bytes);
omc_status omc_aggregate_mean(const void *agg_host, const void *agg_dev, const void *const *arenas,
                              const size_t *arena_bytes, const float *const *sb_tables, float *out,
                              uint64_t aux_elems, void *stream);

/* ---- forward path ------------------------------------------------------------------------ */

/* Workspace (device bytes) for omc_dequant_gemm / omc_dequant_gemm_dx with M activation rows (a few
 * flag words of a pre-pass over the codes; 0 for M == 0). */
size_t omc_dequant_gemm_workspace_bytes(uint32_t M);

/* C[M x N] = A[M x K] * Wbar[K x N], Wbar = decompress(codes, sb)  (Sec. 2.1 forward path: the
 * layer's parameters are decompressed on the fly and consumed at once; here they are expanded
 * inside the kernel and never reach memory as fp32).
 *   A        device, M*K bfloat16 bit patterns, row-major
 *   codes    device, packed K*N-element variable, element index k*N + j
 *   sb       device, 2 floats, or NULL for (1, 0)
 *   C        device, M*N floats, row-major; fp32 accumulation
 *   ws       device workspace of omc_dequant_gemm_workspace_bytes(M) bytes
 * Uses  A*(s*Vt + b*1) = s*(A*Vt) + b*rowsum(A)*1^T.  Requires man_bits <= 7 (every Vtilde is then
 * exactly a bfloat16), M % 256 == 0, N % 128 == 0, K % 32 == 0 (OMC_ERR_FORMAT / OMC_ERR_SIZE).
 * Values of the format below 2^-126 (possible only with a bias near 127) may be flushed to zero by
 * the matrix cores.  S1E4M3 with bias 7 is converted by the hardware's FP8 instructions unless a
 * pre-pass over the codes finds the one code (all exponent and mantissa bits set, value 480) that
 * they read differently; results are the same either way. */
omc_status omc_dequant_gemm(const uint16_t *A, const void *codes, omc_format f, const float *sb,
                            float *C, uint32_t M, uint32_t N, uint32_t K, void *ws, size_t ws_bytes,
                            void *stream);

/* ---- backward path: gradient with respect to the layer's input ----------------------------- */

/* dX[M x K] = dY[M x N] * Wbar^T for the same packed K*N-element variable that omc_dequant_gemm
 * multiplies by (Sec. 2.1, backward propagation: the parameters a layer needs are decompressed on the
 * fly there as well; they are expanded inside the kernel here).
 *   dY       device, M*N bfloat16 bit patterns, row-major
 *   codes    device, packed variable, element index k*N + j   (unchanged layout; read transposed)
 *   sb       device, 2 floats, or NULL for (1, 0)
 *   dX       device, M*K floats, row-major; fp32 accumulation
 *   ws       device workspace of omc_dequant_gemm_workspace_bytes(M) bytes
 * Uses dY*(s*Vt + b*1)^T = s*(dY*Vt^T) + b*rowsum(dY)*1^T.  Requires man_bits <= 7, M % 256 == 0,
 * K % 128 == 0, N % 32 == 0 (OMC_ERR_FORMAT / OMC_ERR_SIZE); otherwise as omc_dequant_gemm. */
omc_status omc_dequant_gemm_dx(const uint16_t *dY, const void *codes, omc_format f, const float *sb,
                               float *dX, uint32_t M, uint32_t N, uint32_t K, void *ws, size_t ws_bytes,
                               void *stream);

/* ---- backward path: weight gradient consumed by the update ---------------------------------- */

/* Workspace (device bytes) for omc_dw_update_recompress with M rows of X / dY on a K x N weight matrix
 * stored in format f; 0 for unsupported formats or sizes.  When the matrix alone gives too few tiles
 * to fill the chip, the M rows are split between workgroups and the workspace holds their partial
 * accumulators (up to 8 * 4*K*N bytes); for code widths other than 8 it always holds one such copy. */
size_t omc_dw_update_workspace_bytes(omc_format f, uint32_t M, uint32_t N, uint32_t K);

/* The whole backward step of a linear layer Y = X * Wbar on its compressed weights (Sec. 2.1, backward
 * propagation: decompress the parameters, apply the gradients, compress, discard): the weight
 * gradient dW[K x N] = X^T * dY is formed on the matrix cores (fp32 accumulation) and consumed at
 * once: every weight is decoded and transformed (Sec. 2.2, 2.3), updated with its gradient by the
 * optimizer of omc_step_update_recompress, rounded to the format and stored back, and new (s, b)
 * are fitted.  The gradient itself is not written to memory unless dW_out is given.
 *   X        device, M*K bfloat16 bit patterns, row-major (the layer's input)
 *   dY       device, M*N bfloat16 bit patterns, row-major (gradient of the layer's output)
 *   codes    device, packed K*N-element variable, element index k*N + j, updated in place
 *   sb       device, 2 floats, in: (s, b) of the variable, out: the new pair ((1, 0) when use_pvt == 0)
 *   state0/1 device, K*N floats each, as for omc_step_update_recompress (momentum / Adam moments)
 *   dW_out   device, K*N floats, or NULL; receives the gradient exactly as the update consumed it
 *   ws       device workspace of omc_dw_update_workspace_bytes(f, M, N, K) bytes
 * Requires K % 256 == 0, N % 128 == 0, M % 32 == 0 (OMC_ERR_SIZE).  With an 8-bit format and enough
 * tiles the update runs in the GEMM kernel's epilogue (a lane of the accumulator layout owns whole
 * dwords of codes) and the gradient never reaches memory; otherwise the accumulators pass through
 * the workspace once and a second kernel does the update.  Result: identical to
 * omc_step_update_recompress on this variable with dW_out as its gradient; the gradient's summation
 * order is fixed by the sizes alone, so repeated calls give identical bits. */
omc_status omc_dw_update_recompress(const uint16_t *X, const uint16_t *dY, void *codes, omc_format f,
                                    float *sb, int use_pvt, float *state0, float *state1,
                                    const omc_opt *opt, float *dW_out, uint32_t M, uint32_t N, uint32_t K,
                                    void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OMC_H */
