/* Walks the CPU oracle through ragged sizes under AddressSanitizer + UBSan (built and run by
 * tests/test_oracle_sanitizers.py; CPU only).  Prints "ok" and returns 0 when nothing was reported. */
#include "../oracle/omc_oracle.c"
#include <stdio.h>

static float frand(uint32_t *s)
{
    *s = *s * 1664525u + 1013904223u;
    return ((float)(*s >> 8) / 8388608.0f - 1.0f) * 0.05f;
}

int main(void)
{
    uint32_t seed = 12345;
    const int EM[][2] = {{4, 3}, {3, 7}, {2, 3}, {5, 10}, {4, 14}, {8, 23}, {1, 0}, {8, 7}, {4, 20}};
    const uint64_t sizes[] = {1, 2, 31, 32, 33, 127, 2047, 2048, 2049, 5000};
    for (unsigned f = 0; f < sizeof EM / sizeof EM[0]; ++f) {
        orc_format fmt = {EM[f][0], EM[f][1], (1 << (EM[f][0] - 1)) - 1};
        int B = orc_format_bits(fmt);
        for (unsigned k = 0; k < sizeof sizes / sizeof sizes[0]; ++k) {
            uint64_t n = sizes[k];
            float *v = malloc(n * sizeof(float)), *g = malloc(n * sizeof(float)), *out = malloc(n * sizeof(float));
            float *m = calloc(n, sizeof(float)), *vv = calloc(n, sizeof(float));
            uint8_t *packed = malloc(orc_packed_bytes(n, B));
            uint32_t *codes = malloc(n * sizeof(uint32_t));
            float sb[2];
            for (uint64_t i = 0; i < n; ++i) { v[i] = frand(&seed); g[i] = frand(&seed); }
            if (n > 3) { v[0] = 0.0f; v[1] = -0.0f; v[2] = 1e30f; v[3] = -1e-40f; }
            if (orc_compress(v, n, fmt, 1, packed, sb)) return 2;
            if (orc_decompress(packed, n, fmt, sb, out)) return 3;
            orc_unpack(packed, n, B, codes);
            orc_pack(codes, n, B, packed);
            for (int kind = 0; kind < 3; ++kind) {
                orc_opt o = {kind, 0.05f, 0.9f, 0.9f, 0.999f, 1e-8f, 0.1f, 0.001f, 0.1f, 0.001f};
                if (orc_step_quantized(packed, n, fmt, 1, sb, g, m, vv, &o)) return 4;
                orc_step_fp32(out, n, g, m, vv, &o);
            }
            const float *reps[3] = {v, g, out};
            orc_mean_f32(reps, 3, n, out);
            free(v); free(g); free(out); free(m); free(vv); free(packed); free(codes);
        }
    }
    /* a variable set in one arena, two threads */
    {
        orc_format f1 = {3, 7, 3}, f2 = {4, 3, 7};
        orc_var vars[3] = {{0, 0, 3000, f1, 1, 1}, {4128, 3000, 100, f1, 0, 1}, {4528, 3100, 2049, f2, 1, 0}};
        uint64_t arena_bytes = 4528 + orc_packed_bytes(2049, 8), aux = 3100 + 2049 + 3;
        uint8_t *arena = calloc(arena_bytes, 1);
        float *g = calloc(aux, sizeof(float)), *m = calloc(aux, sizeof(float)), *v = calloc(aux, sizeof(float));
        float sbt[6] = {1, 0, 1, 0, 1, 0};
        for (uint64_t i = 0; i < aux; ++i) g[i] = frand(&seed);
        orc_opt o = {2, 1e-3f, 0.9f, 0.9f, 0.999f, 1e-8f, 0.1f, 0.001f, 0.1f, 0.001f};
        if (orc_step_varset(arena, vars, 3, sbt, g, m, v, &o, 2)) return 5;
        free(arena); free(g); free(m); free(v);
    }
    /* the three matrix products on a small layer */
    {
        enum { M = 8, N = 16, K = 32 };
        orc_format fmt = {4, 3, 7};
        float W[K * N], sb[2];
        uint16_t A[M * K], dY[M * N];
        uint8_t packed[K * N + 16];
        double C[M * N], dX[M * K], dW[K * N];
        for (int i = 0; i < K * N; ++i) W[i] = frand(&seed);
        for (int i = 0; i < M * K; ++i) A[i] = (uint16_t)(0x3c00 + (i & 0xff));
        for (int i = 0; i < M * N; ++i) dY[i] = (uint16_t)(0xbc00 + (i & 0x7f));
        if (orc_compress(W, K * N, fmt, 1, packed, sb)) return 6;
        if (orc_dequant_gemm(A, packed, fmt, sb, C, M, N, K, 0, M, 2)) return 7;
        if (orc_dequant_gemm_dx(dY, packed, fmt, sb, dX, M, N, K, 0, M, 2)) return 8;
        if (orc_gemm_dw(A, dY, dW, M, N, K, 0, K, 2)) return 9;
    }
    puts("ok");
    return 0;
}
