/* Runs every function of the CPU oracle on heap buffers of exactly the documented sizes, ragged shapes and empty
 * inputs included, for a build with -fsanitize=address,undefined: any access beyond a buffer, signed overflow or
 * misaligned access in the oracle aborts the program.  Values are not checked here (the pin tests do that). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/oracle.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}

static uint8_t *codes(int64_t n, int bits, int enc)
{
    uint8_t *b = malloc(n > 0 ? (size_t)n : 1);
    for (int64_t i = 0; i < n; ++i)
        b[i] = enc == ORC_PM1 ? (uint8_t)((rnd() & 1) ? 1 : 0xFF) : (uint8_t)(rnd() & ((1u << bits) - 1));
    return b;
}

#define CHECK(call) do { int rc_ = (call); if (rc_ != ORC_OK) { printf("%s -> %d\n", #call, rc_); return 1; } } while (0)

int main(void)
{
    static const int shapes[][3] = {{1, 1, 1}, {3, 5, 33}, {17, 9, 64}, {8, 8, 100}, {0, 4, 7}, {4, 0, 7}, {4, 4, 0}};
    for (unsigned c = 0; c < sizeof shapes / sizeof shapes[0]; ++c) {
        const int64_t M = shapes[c][0], N = shapes[c][1], K = shapes[c][2];
        for (int kind = 0; kind < 4; ++kind) {
            const int encW = kind & 1 ? ORC_PM1 : ORC_UNSIGNED, encX = kind & 2 ? ORC_PM1 : ORC_UNSIGNED;
            const int p = encW == ORC_PM1 ? 1 : 1 + (int)(rnd() % 8), q = encX == ORC_PM1 ? 1 : 1 + (int)(rnd() % 8);
            uint8_t *W = codes(M * K, p, encW), *X = codes(N * K, q, encX);
            int32_t *Y = malloc((size_t)(M * N > 0 ? M * N : 1) * sizeof *Y);
            int32_t *D = malloc((size_t)(M * K > 0 ? M * K : 1) * sizeof *D);
            CHECK(orc_decode(W, M * K, p, encW, D));
            CHECK(orc_gemm(W, encW, p, X, encX, q, M, N, K, Y));
            CHECK(orc_gemm_rows(W, encW, p, X, encX, q, M, N, K, M / 2, M, Y));
            CHECK(orc_apbit_gemm(W, encW, p, X, encX, q, M, N, K, Y));
            free(W); free(X); free(Y); free(D);
        }
    }
    static const int convs[][9] = {   /* BS Cin H W Cout R S stride pad */
        {1, 3, 5, 7, 4, 3, 3, 1, 1}, {2, 8, 6, 6, 5, 1, 1, 2, 0}, {1, 2, 9, 4, 3, 5, 3, 2, 2}, {1, 1, 1, 1, 1, 1, 1, 1, 0}};
    for (unsigned c = 0; c < sizeof convs / sizeof convs[0]; ++c) {
        const int *v = convs[c];
        const int64_t BS = v[0], Cin = v[1], H = v[2], Wd = v[3], Cout = v[4];
        const int R = v[5], S = v[6], stride = v[7], pad = v[8];
        const int64_t Ho = (H + 2 * pad - R) / stride + 1, Wo = (Wd + 2 * pad - S) / stride + 1;
        for (int pm = 0; pm < 2; ++pm) {
            const int enc = pm ? ORC_PM1 : ORC_UNSIGNED, bits = pm ? 1 : 2;
            uint8_t *W = codes(Cout * Cin * R * S, bits, enc), *X = codes(BS * Cin * H * Wd, bits, enc);
            int32_t *Y = malloc((size_t)(BS * Cout * Ho * Wo) * sizeof *Y);
            CHECK(orc_conv2d(W, enc, bits, X, enc, bits, BS, Cin, H, Wd, Cout, R, S, stride, pad, Y));
            float *scale = malloc((size_t)Cout * sizeof *scale), *bias = malloc((size_t)Cout * sizeof *bias);
            for (int64_t i = 0; i < Cout; ++i) { scale[i] = 0.1f; bias[i] = 1.0f; }
            uint8_t *res = codes(BS * Cout * Ho * Wo, 2, ORC_UNSIGNED), *out = malloc((size_t)(BS * Cout * Ho * Wo));
            float *t = malloc((size_t)(BS * Cout * Ho * Wo) * sizeof *t);
            CHECK(orc_epilogue(Y, BS, Cout, Ho * Wo, scale, bias, res, 0.5f, 2, t, out));
            CHECK(orc_epilogue(Y, BS, Cout, Ho * Wo, scale, bias, NULL, 0.0f, 8, NULL, out));
            if (Ho >= 2 && Wo >= 2) {
                int32_t *P = malloc((size_t)(BS * Cout * (Ho / 2) * (Wo / 2)) * sizeof *P);
                CHECK(orc_gridpool(Y, BS, Cout, Ho, Wo, 2, 1, P));
                CHECK(orc_gridpool(Y, BS, Cout, Ho, Wo, 2, 2, P));
                free(P);
            }
            const int64_t Hm = (Ho + 2 - 3) / 2 + 1, Wm = (Wo + 2 - 3) / 2 + 1;
            if (Ho >= 2 && Wo >= 2) {
                uint8_t *mp = malloc((size_t)(BS * Cout * Hm * Wm));
                CHECK(orc_maxpool(out, BS, Cout, Ho, Wo, 3, 2, 1, mp));
                free(mp);
            }
            for (int64_t i = 0; i < BS * Cout * Ho * Wo; ++i) out[i] &= 1;
            uint8_t *sp = malloc((size_t)(BS * Cout));
            if (Ho * Wo <= 255) CHECK(orc_sumpool(out, BS, Cout, Ho * Wo, sp));
            free(sp); free(W); free(X); free(Y); free(scale); free(bias); free(res); free(out); free(t);
        }
    }
    {
        const int64_t n = 1000;
        float *x = malloc((size_t)n * sizeof *x);
        uint8_t *cq = malloc((size_t)n);
        for (int64_t i = 0; i < n; ++i) x[i] = (float)((int)(rnd() % 2000) - 1000) * 0.01f;
        x[0] = 1e30f; x[1] = -1e30f; x[2] = 0.0f / 1.0f;
        for (int bits = 1; bits <= 8; ++bits) CHECK(orc_quantize(x, n, -0.3f, 0.07f, bits, cq));
        CHECK(orc_quantize(x, 0, 0.0f, 1.0f, 2, cq));
        double g[5] = {1, 2, 3, 4, 5}, bvec[5] = {0, 1, 0, 1, 0}, m[5] = {0.5, 0.5, 0.5, 0.5, 0.5}, var[5] = {1, 1, 2, 2, 3};
        float sc[5], bi[5];
        CHECK(orc_fold_bn(g, bvec, m, var, 1e-5, 0.1, 0.5, 5, sc, bi));
        free(x); free(cq);
    }
    /* error paths must report, not crash */
    {
        uint8_t bad[4] = {7, 0, 1, 2};
        int32_t y[4];
        if (orc_decode(bad, 4, 2, ORC_UNSIGNED, y) != ORC_ERR_VALUE) { puts("bad value not reported"); return 1; }
        if (orc_gemm(bad, ORC_UNSIGNED, 9, bad, ORC_UNSIGNED, 1, 1, 1, 1, y) == ORC_OK) { puts("9 bits accepted"); return 1; }
    }
    printf("oracle sanitizer run ok (%d threads)\n", orc_threads());
    return 0;
}
