/*
 * omc_oracle.c -- plain, slow CPU oracle for Online Model Compression (OMC).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is held
 * against.  It shares no code, header, table or helper with the HIP library,
 * and nothing in the product path may call it.
 *
 * What it follows (paper sections):
 *   - Sec. 2.2  floating-point quantization SxEyMz (1 sign, E exponent, M mantissa bits);
 *   - Sec. 2.3  per-variable transformation  Vbar = s*Vtilde + b*1  with the
 *               closed-form least-squares (s, b), fp64 compute, fp32 store,
 *               s = 1 in the degenerate case;
 *   - Sec. 2.1  the per-iteration cycle: decompress -> apply the gradient ->
 *               compress -> discard (backward path), decompress -> consume (forward path);
 *   - Sec. 2.4 / 2.5  only some variables are quantized, the rest stay fp32.
 *
 * Readings taken where the paper is silent or garbled (they are listed with
 * reasons in the design document of this repository):
 *   - exponent bias defaults to 2^(E-1)-1; e == 0 encodes zero and subnormals;
 *     there are no Inf/NaN codes (the top exponent is an ordinary binade);
 *   - rounding is to nearest, ties to the even integer significand; overflow saturates;
 *   - a code whose value would exceed the largest finite fp32 is not a valid
 *     code (only possible for E = 8); the encoder saturates to the largest valid one;
 *   - packing is a dense little-endian bit stream, element k in stream bits
 *     [k*B, (k+1)*B), padded with zero bits to a multiple of 16 bytes;
 *   - the denominator of s printed in Sec. 2.3 mixes V and Vtilde and the
 *     printed b carries a stray factor n; the least-squares objective stated in
 *     the same section fixes   s = (n SUM V Vt - SUM V SUM Vt) / (n SUM Vt^2 - (SUM Vt)^2),
 *     b = (SUM V - s SUM Vt) / n,   which is what is computed here;
 *   - the degenerate case is "all Vtilde equal" (tested as min == max);
 *   - all fp32 expressions are evaluated one rounding per operation (no fused
 *     multiply-add); the four sums of the fit are exactly rounded;
 *   - a non-finite input value encodes to the saturated code of its sign and
 *     makes (s, b) NaN.                                   [parity unpinned]
 *
 * Style: value-domain arithmetic in double (frexp / ldexp / nearbyint), a
 * bit-by-bit packer, a big-integer accumulator for exact sums.  Nothing is
 * blocked, fused or reordered beyond the steps named above.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC omc_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Format SxEyMz (Sec. 2.2; notation of Sec. 3.1).  x is always 1.            */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t exp_bits; /* E: 1..8  */
    int32_t man_bits; /* M: 0..23 */
    int32_t bias;     /* >= 0; caller resolves the default 2^(E-1)-1 */
} orc_format;

static int fmt_bits(orc_format f) { return 1 + f.exp_bits + f.man_bits; }

/* largest exponent field whose binade still lies inside finite fp32 */
static int fmt_top_field(orc_format f)
{
    int top = (1 << f.exp_bits) - 1;
    if (top - f.bias > 127) top = 127 + f.bias;
    return top;
}

int orc_format_bits(orc_format f) { return fmt_bits(f); }

/* largest representable magnitude */
double orc_format_max(orc_format f)
{
    return ldexp(2.0 - ldexp(1.0, -f.man_bits), fmt_top_field(f) - f.bias);
}

/* value of a code, as a double (exact).  Sec. 2.2. */
double orc_decode_value(uint32_t code, orc_format f)
{
    int E = f.exp_bits, M = f.man_bits;
    uint32_t m = code & ((M == 0) ? 0u : ((1u << M) - 1u));
    uint32_t e = (code >> M) & ((1u << E) - 1u);
    uint32_t sign = (code >> (E + M)) & 1u;
    double mag;
    if (e == 0)
        mag = ldexp((double)m, 1 - f.bias - M);           /* zero and subnormals */
    else
        mag = ldexp((double)((1u << M) + m), (int)e - f.bias - M); /* normal   */
    return sign ? -mag : mag;
}

float orc_decode(uint32_t code, orc_format f)
{
    return (float)orc_decode_value(code, f); /* exact for every valid code */
}

/* nearest code to v: round to nearest, ties to even significand, saturate. */
uint32_t orc_encode(float v, orc_format f)
{
    int E = f.exp_bits, M = f.man_bits;
    int top = fmt_top_field(f);
    uint32_t sign = signbit(v) ? 1u : 0u;
    uint32_t sat = ((uint32_t)top << M) | ((M == 0) ? 0u : ((1u << M) - 1u));
    uint32_t mag;
    if (isnan(v) || isinf(v)) {
        mag = sat;
    } else {
        double a = fabs((double)v);
        if (a == 0.0) {
            mag = 0;
        } else {
            int e2;
            (void)frexp(a, &e2);       /* a = f * 2^e2, f in [0.5, 1) */
            int ex = e2 - 1;           /* floor(log2 a) */
            int emin = 1 - f.bias;
            if (ex < emin) ex = emin;  /* subnormal range shares the step of the first binade */
            double ulp = ldexp(1.0, ex - M);
            double k = nearbyint(a / ulp); /* exact scaling, then ties-to-even */
            double two_m = ldexp(1.0, M);
            if (k == 2.0 * two_m) { ex += 1; k = two_m; }
            if (ex > top - f.bias) {
                mag = sat;
            } else if (k >= two_m) {
                mag = ((uint32_t)(ex + f.bias) << M) | (uint32_t)(k - two_m);
            } else {
                mag = (uint32_t)k;     /* e = 0 */
            }
        }
    }
    return (sign << (E + M)) | mag;
}

void orc_encode_array(const float *v, uint64_t n, orc_format f, uint32_t *codes)
{
    for (uint64_t k = 0; k < n; ++k) codes[k] = orc_encode(v[k], f);
}

void orc_decode_array(const uint32_t *codes, uint64_t n, orc_format f, float *out)
{
    for (uint64_t k = 0; k < n; ++k) out[k] = orc_decode(codes[k], f);
}

/* ------------------------------------------------------------------------- */
/* Dense bit stream.  Element k occupies stream bits [k*B, (k+1)*B), least    */
/* significant code bit first; stream bit i is bit (i % 8) of byte i / 8.     */
/* ------------------------------------------------------------------------- */
uint64_t orc_packed_bytes(uint64_t n, int B)
{
    uint64_t bits = n * (uint64_t)B;
    uint64_t bytes = (bits + 7) / 8;
    return (bytes + 15) / 16 * 16;
}

void orc_pack(const uint32_t *codes, uint64_t n, int B, uint8_t *out)
{
    memset(out, 0, orc_packed_bytes(n, B));
    for (uint64_t k = 0; k < n; ++k)
        for (int j = 0; j < B; ++j) {
            uint64_t i = k * (uint64_t)B + (uint64_t)j;
            if ((codes[k] >> j) & 1u) out[i / 8] |= (uint8_t)(1u << (i % 8));
        }
}

void orc_unpack(const uint8_t *in, uint64_t n, int B, uint32_t *codes)
{
    for (uint64_t k = 0; k < n; ++k) {
        uint32_t c = 0;
        for (int j = 0; j < B; ++j) {
            uint64_t i = k * (uint64_t)B + (uint64_t)j;
            if ((in[i / 8] >> (i % 8)) & 1u) c |= (1u << j);
        }
        codes[k] = c;
    }
}

/* ------------------------------------------------------------------------- */
/* Exact summation: a wide fixed-point accumulator.                           */
/* value = SUM limb[i] * 2^(32 i - ACC_LOW).  Every term handed in is a       */
/* product of at most two fp32 numbers, so it is a multiple of 2^-298 and     */
/* below 2^257; 2^31 such terms fit with room to spare.                       */
/* ------------------------------------------------------------------------- */
#define ACC_LOW 320
#define ACC_LIMBS 22
typedef struct { int64_t limb[ACC_LIMBS]; } exact_acc;

static void acc_clear(exact_acc *a) { memset(a, 0, sizeof *a); }

static void acc_add(exact_acc *a, double x)
{
    if (x == 0.0) return;
    int e2;
    double fr = frexp(fabs(x), &e2);                 /* |x| = fr * 2^e2 */
    uint64_t m = (uint64_t)ldexp(fr, 53);            /* 53-bit integer, exact */
    int pos = e2 - 53 + ACC_LOW;                     /* |x| = m * 2^(pos - ACC_LOW) */
    if (pos < 0) { m >>= -pos; pos = 0; }            /* dropped bits are zero for our terms */
    int q = pos / 32, r = pos % 32;
    unsigned __int128 w = (unsigned __int128)m << r; /* up to 85 bits */
    int64_t sg = (x < 0) ? -1 : 1;
    for (int i = 0; i < 3; ++i) {
        int64_t piece = (int64_t)(uint32_t)(w >> (32 * i));
        a->limb[q + i] += sg * piece;
    }
}

/* nearest double to the accumulated value, ties to even */
static double acc_round(const exact_acc *a)
{
    int64_t d[ACC_LIMBS + 1];
    int64_t carry = 0;
    for (int i = 0; i < ACC_LIMBS; ++i) {            /* canonical digits in [0, 2^32) */
        int64_t t = a->limb[i] + carry;
        int64_t lo = t & 0xffffffffLL;
        carry = (t - lo) / 4294967296LL;
        d[i] = lo;
    }
    d[ACC_LIMBS] = carry;                            /* signed top */
    int neg = 0;
    if (d[ACC_LIMBS] < 0) {                          /* negate: two's complement over the digits */
        neg = 1;
        int64_t c = 1;
        for (int i = 0; i < ACC_LIMBS; ++i) {
            int64_t t = (0xffffffffLL - d[i]) + c;
            d[i] = t & 0xffffffffLL;
            c = t >> 32;
        }
        d[ACC_LIMBS] = -d[ACC_LIMBS] - 1 + c;        /* ~top + carry */
    }
    int nd = ACC_LIMBS + 1;
    int hi = -1;                                     /* index of the top set bit */
    for (int i = nd - 1; i >= 0 && hi < 0; --i)
        if (d[i] != 0)
            for (int bit = 62; bit >= 0; --bit)
                if ((d[i] >> bit) & 1) { hi = 32 * i + bit; break; }
    if (hi < 0) return 0.0;
    /* gather bits hi .. hi-52 into an integer, then look at the rest.  The signed top
       limb is zero here: the magnitudes handed in stay far below 2^(32*ACC_LIMBS-ACC_LOW). */
    uint64_t mant = 0;
    for (int p = hi; p > hi - 53; --p) {
        int b = (p < 0) ? 0 : (int)((d[p / 32] >> (p % 32)) & 1);
        mant = (mant << 1) | (uint64_t)b;
    }
    int rpos = hi - 53;                              /* first dropped bit */
    int round_bit = 0, sticky = 0;
    if (rpos >= 0) {
        round_bit = (int)((d[rpos / 32] >> (rpos % 32)) & 1);
        for (int p = rpos - 1; p >= 0 && !sticky; --p)
            if ((d[p / 32] >> (p % 32)) & 1) sticky = 1;
    }
    if (round_bit && (sticky || (mant & 1))) mant += 1;  /* may reach 2^53: still exact below */
    double r = ldexp((double)mant, hi - 52 - ACC_LOW);
    return neg ? -r : r;
}

/* exactly rounded SUM x[k] (exported so that tests can pin it) */
double orc_exact_sum(const double *x, uint64_t n)
{
    exact_acc a;
    acc_clear(&a);
    for (uint64_t k = 0; k < n; ++k) acc_add(&a, x[k]);
    return acc_round(&a);
}

/* ------------------------------------------------------------------------- */
/* Per-variable transformation, fit (Sec. 2.3).                               */
/* V: full-precision values before compression; Vt: decompressed values.      */
/* ------------------------------------------------------------------------- */
void orc_pvt_fit(const float *V, const float *Vt, uint64_t n, float *s_out, float *b_out)
{
    exact_acc aV, aT, aVT, aTT;
    acc_clear(&aV); acc_clear(&aT); acc_clear(&aVT); acc_clear(&aTT);
    int finite = 1;
    float tmin = Vt[0], tmax = Vt[0];
    for (uint64_t k = 0; k < n; ++k) {
        if (!isfinite(V[k])) { finite = 0; break; }
        double v = (double)V[k], t = (double)Vt[k];
        acc_add(&aV, v);
        acc_add(&aT, t);
        acc_add(&aVT, v * t);   /* 24 x 24 bit product: exact in double */
        acc_add(&aTT, t * t);
        if (Vt[k] < tmin) tmin = Vt[k];
        if (Vt[k] > tmax) tmax = Vt[k];
    }
    if (!finite) { *s_out = NAN; *b_out = NAN; return; }
    double SV = acc_round(&aV), ST = acc_round(&aT), SVT = acc_round(&aVT), STT = acc_round(&aTT);
    double dn = (double)n;
    double s, b;
    if (tmin == tmax) {          /* all Vtilde equal: the degenerate case, s = 1 */
        s = 1.0;
    } else {
        double num = dn * SVT - SV * ST;
        double den = dn * STT - ST * ST;
        s = num / den;
    }
    b = (SV - s * ST) / dn;
    *s_out = (float)s;
    *b_out = (float)b;
}

/* ------------------------------------------------------------------------- */
/* compress / decompress of one variable (Sec. 2.1 - 2.3)                     */
/* ------------------------------------------------------------------------- */
int orc_compress(const float *V, uint64_t n, orc_format f, int use_pvt,
                 uint8_t *packed, float *sb /* [2] */)
{
    if (n == 0) return 1;
    int B = fmt_bits(f);
    uint32_t *codes = (uint32_t *)malloc(n * sizeof(uint32_t));
    float *Vt = (float *)malloc(n * sizeof(float));
    if (!codes || !Vt) { free(codes); free(Vt); return 2; }
    for (uint64_t k = 0; k < n; ++k) {
        codes[k] = orc_encode(V[k], f);
        Vt[k] = orc_decode(codes[k], f);
    }
    if (use_pvt) orc_pvt_fit(V, Vt, n, &sb[0], &sb[1]);
    else { sb[0] = 1.0f; sb[1] = 0.0f; }
    orc_pack(codes, n, B, packed);
    free(codes); free(Vt);
    return 0;
}

/* Vbar_k = fl32(fl32(s * Vtilde_k) + b) */
int orc_decompress(const uint8_t *packed, uint64_t n, orc_format f, const float *sb, float *out)
{
    if (n == 0) return 1;
    int B = fmt_bits(f);
    uint32_t *codes = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!codes) return 2;
    orc_unpack(packed, n, B, codes);
    float s = sb ? sb[0] : 1.0f, b = sb ? sb[1] : 0.0f;
    for (uint64_t k = 0; k < n; ++k) {
        float t = orc_decode(codes[k], f);
        float st = s * t;
        out[k] = st + b;
    }
    free(codes);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Parameter update on the decompressed values (Sec. 2.1, backward path).     */
/* The optimizer is not named by the paper; the three below are the plain     */
/* textbook forms, every fp32 operation rounded on its own.                   */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t kind;      /* 0 SGD, 1 momentum, 2 Adam */
    float lr;
    float momentum;    /* kind 1 */
    float beta1, beta2, eps;           /* kind 2 */
    float one_minus_beta1, one_minus_beta2; /* fp32(1 - beta) computed in fp64 by the caller */
    float bias_corr1, bias_corr2;      /* fp32(1 - beta^t)  computed in fp64 by the caller */
} orc_opt;

/* fl(x): the fp32 number nearest to the double x.  Each operation below is carried out on the exact
 * double images of its fp32 operands and then rounded with fl().  For +, -, *, / and sqrt of fp32
 * operands this equals the correctly rounded fp32 operation (a double keeps more than 2*24+2 bits, so
 * the intermediate rounding to double cannot move the final one): "every operation rounded on its own". */
static float fl(double x) { return (float)x; }

/* plain SGD:  w <- w - lr g */
static float sgd_rule(float w, float g, const orc_opt *o)
{
    float scaled_g = fl((double)o->lr * (double)g);
    return fl((double)w - (double)scaled_g);
}

/* SGD with momentum (no dampening, no Nesterov):  m <- mu m + g;  w <- w - lr m */
static float momentum_rule(float w, float g, float *m, const orc_opt *o)
{
    float decayed = fl((double)o->momentum * (double)*m);
    *m = fl((double)decayed + (double)g);
    float stepv = fl((double)o->lr * (double)*m);
    return fl((double)w - (double)stepv);
}

/* Adam:  m <- b1 m + (1-b1) g;  v <- b2 v + ((1-b2) g) g;
 *        w <- w - (lr (m / c1)) / (sqrt(v / c2) + eps),  c1 = 1-b1^t, c2 = 1-b2^t */
static float adam_rule(float w, float g, float *m, float *v, const orc_opt *o)
{
    float first_old = fl((double)o->beta1 * (double)*m);
    float first_new = fl((double)o->one_minus_beta1 * (double)g);
    *m = fl((double)first_old + (double)first_new);

    float second_old = fl((double)o->beta2 * (double)*v);
    float g_weighted = fl((double)o->one_minus_beta2 * (double)g);
    float second_new = fl((double)g_weighted * (double)g);
    *v = fl((double)second_old + (double)second_new);

    float m_unbiased = fl((double)*m / (double)o->bias_corr1);
    float v_unbiased = fl((double)*v / (double)o->bias_corr2);
    float numerator = fl((double)o->lr * (double)m_unbiased);
    float root = fl(sqrt((double)v_unbiased));
    float denominator = fl((double)root + (double)o->eps);
    float stepv = fl((double)numerator / (double)denominator);
    return fl((double)w - (double)stepv);
}

static float update_one(float w, float g, float *m, float *v, const orc_opt *o)
{
    switch (o->kind) {
    case 0:  return sgd_rule(w, g, o);
    case 1:  return momentum_rule(w, g, m, o);
    default: return adam_rule(w, g, m, v, o);
    }
}

/* one iteration on one quantized variable: decompress -> update -> recompress */
int orc_step_quantized(uint8_t *packed, uint64_t n, orc_format f, int use_pvt, float *sb,
                       const float *g, float *st0, float *st1, const orc_opt *o)
{
    if (n == 0) return 1;
    float *W = (float *)malloc(n * sizeof(float));
    if (!W) return 2;
    int rc = orc_decompress(packed, n, f, sb, W);
    if (rc) { free(W); return rc; }
    for (uint64_t k = 0; k < n; ++k)
        W[k] = update_one(W[k], g[k], st0 ? &st0[k] : NULL, st1 ? &st1[k] : NULL, o);
    rc = orc_compress(W, n, f, use_pvt, packed, sb);
    free(W);
    return rc;
}

/* one iteration on one variable kept in fp32 */
int orc_step_fp32(float *W, uint64_t n, const float *g, float *st0, float *st1, const orc_opt *o)
{
    for (uint64_t k = 0; k < n; ++k)
        W[k] = update_one(W[k], g[k], st0 ? &st0[k] : NULL, st1 ? &st1[k] : NULL, o);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* A variable set in one arena (Sec. 2.4, 2.5: some variables packed, the     */
/* others plain fp32).  Variables are independent; the loop over them may     */
/* run on several threads without changing any result.                        */
/* ------------------------------------------------------------------------- */
typedef struct {
    uint64_t data_offset; /* bytes into the arena */
    uint64_t aux_offset;  /* elements into grads / state arrays */
    uint64_t n;
    orc_format fmt;
    int32_t quantized;
    int32_t use_pvt;
} orc_var;

int orc_step_varset(uint8_t *arena, const orc_var *vars, uint32_t nvars, float *sb_table,
                    const float *grads, float *state0, float *state1, const orc_opt *o,
                    int threads)
{
    int bad = 0;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (uint32_t i = 0; i < nvars; ++i) {
        const orc_var *v = &vars[i];
        const float *g = grads + v->aux_offset;
        float *s0 = state0 ? state0 + v->aux_offset : NULL;
        float *s1 = state1 ? state1 + v->aux_offset : NULL;
        int rc;
        if (v->quantized)
            rc = orc_step_quantized(arena + v->data_offset, v->n, v->fmt, v->use_pvt,
                                    sb_table + 2 * (uint64_t)i, g, s0, s1, o);
        else
            rc = orc_step_fp32((float *)(arena + v->data_offset), v->n, g, s0, s1, o);
        if (rc) {
#pragma omp atomic write
            bad = rc;
        }
    }
    return bad;
}

/* ------------------------------------------------------------------------- */
/* Forward path (Sec. 2.1): the layer's weights are decompressed and consumed */
/* by the matrix product at once.  C = A * Wbar, A given as bfloat16 bit      */
/* patterns [M x K] row-major, Wbar = decompress(codes) as [K x N] row-major. */
/* Products and sums in double.                                               */
/* ------------------------------------------------------------------------- */
static double bf16_value(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float x;
    memcpy(&x, &u, 4);
    return (double)x;
}

int orc_dequant_gemm(const uint16_t *A, const uint8_t *packed, orc_format f, const float *sb,
                     double *C, uint32_t M, uint32_t N, uint32_t K,
                     uint32_t row_begin, uint32_t row_end, int threads)
{
    uint64_t n = (uint64_t)K * N;
    float *W = (float *)malloc(n * sizeof(float));
    if (!W) return 2;
    int rc = orc_decompress(packed, n, f, sb, W);
    if (rc) { free(W); return rc; }
    if (row_end > M) row_end = M;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (uint32_t i = row_begin; i < row_end; ++i) {
        double *c = C + (uint64_t)(i - row_begin) * N;
        for (uint32_t j = 0; j < N; ++j) c[j] = 0.0;
        for (uint32_t k = 0; k < K; ++k) {
            double a = bf16_value(A[(uint64_t)i * K + k]);
            const float *w = W + (uint64_t)k * N;
            for (uint32_t j = 0; j < N; ++j) c[j] += a * (double)w[j];
        }
    }
    free(W);
    return 0;
}

/* ---- server-side aggregation -------------------------------------------------------------------
 * Sec. 1 (a federated round ends with the clients' models transported back and aggregated) and
 * Sec. 2.5 (each client quantizes its own subset of the variables, so the server sees a variable
 * in full precision from some clients and as codes + (s, b) from others).  The paper does not spell
 * the aggregation out; the reading taken here is the plain federated average with equal weights:
 *     out[i] = ( ... ((v_0[i] + v_1[i]) + v_2[i]) ... + v_{R-1}[i] ) / R
 * on the clients' decompressed values, every operation rounded once to fp32, clients in index
 * order.  The caller decompresses (orc_decompress) whatever arrived compressed. */
int orc_mean_f32(const float *const *v, int R, uint64_t n, float *out)
{
    if (R < 1) return 1;
    for (uint64_t i = 0; i < n; ++i) {
        float acc = v[0][i];
        for (int r = 1; r < R; ++r) acc = acc + v[r][i];
        out[i] = acc / (float)R;
    }
    return 0;
}

/* ---- backward path of a linear layer: gradient with respect to the input ------------------------
 * Sec. 2.1, backward propagation: the layer's parameters are decompressed on the fly here too.
 * For Y = X * Wbar with Wbar [K x N] the input gradient is dX = dY * Wbar^T:
 *     dX[i][k] = sum_j dY[i][j] * Wbar[k][j],
 * evaluated in double on the fp32 values of the decompressed weights and the bfloat16 values of dY. */
int orc_dequant_gemm_dx(const uint16_t *dY, const uint8_t *packed, orc_format f, const float *sb,
                        double *dX, uint32_t M, uint32_t N, uint32_t K,
                        uint32_t row_begin, uint32_t row_end, int threads)
{
    uint64_t n = (uint64_t)K * N;
    float *W = (float *)malloc(n * sizeof(float));
    if (!W) return 2;
    int rc = orc_decompress(packed, n, f, sb, W);
    if (rc) { free(W); return rc; }
    if (row_end > M) row_end = M;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (uint32_t i = row_begin; i < row_end; ++i) {
        double *d = dX + (uint64_t)(i - row_begin) * K;
        for (uint32_t k = 0; k < K; ++k) {
            const float *w = W + (uint64_t)k * N;
            double acc = 0.0;
            for (uint32_t j = 0; j < N; ++j) acc += bf16_value(dY[(uint64_t)i * N + j]) * (double)w[j];
            d[k] = acc;
        }
    }
    free(W);
    return 0;
}

/* ---- backward path of a linear layer: gradient with respect to the weights -----------------------
 * For Y = X * Wbar the weight gradient is dW = X^T * dY:
 *     dW[k][j] = sum_i X[i][k] * dY[i][j],
 * in double on the bfloat16 values of X [M x K] and dY [M x N].  The update that consumes it is
 * orc_step_quantized with this gradient (Sec. 2.1, backward propagation: decompress, apply the
 * gradient, compress, discard). */
int orc_gemm_dw(const uint16_t *X, const uint16_t *dY, double *dW, uint32_t M, uint32_t N, uint32_t K,
                uint32_t row_begin, uint32_t row_end, int threads)
{
    if (row_end > K) row_end = K;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (uint32_t k = row_begin; k < row_end; ++k) {
        double *d = dW + (uint64_t)(k - row_begin) * N;
        for (uint32_t j = 0; j < N; ++j) d[j] = 0.0;
        for (uint32_t i = 0; i < M; ++i) {
            double x = bf16_value(X[(uint64_t)i * K + k]);
            const uint16_t *g = dY + (uint64_t)i * N;
            for (uint32_t j = 0; j < N; ++j) d[j] += x * bf16_value(g[j]);
        }
    }
    return 0;
}
