/*
 * CPU oracle -- TEST INFRASTRUCTURE ONLY (see oracle.h).
 * Plain loops over decoded integers, int64 accumulation, no blocking, no
 * bit tricks (except in orc_apbit_gemm, whose whole point is to spell out
 * the bit-plane formulas of Sec. 3).  OpenMP only spreads the outermost
 * output loop over the host cores.
 */
#include "oracle.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sec. 3.2: a bit either counts as itself (0/1) or encodes -1/+1. */
int orc_decode(const uint8_t *stored, int64_t n, int bits, int enc, int32_t *out)
{
    if (!stored || !out || n < 0 || bits < 1 || bits > 8) return ORC_ERR_ARG;
    if (enc == ORC_PM1) {
        if (bits != 1) return ORC_ERR_ARG;
        for (int64_t i = 0; i < n; ++i) {
            int v = (int8_t)stored[i];
            if (v != 1 && v != -1) return ORC_ERR_VALUE;
            out[i] = v;
        }
        return ORC_OK;
    }
    if (enc != ORC_UNSIGNED) return ORC_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        int v = stored[i];
        if (v >= (1 << bits)) return ORC_ERR_VALUE;
        out[i] = v;
    }
    return ORC_OK;
}

int orc_gemm_rows(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
                  int64_t M, int64_t N, int64_t K, int64_t m0, int64_t m1, int32_t *Y)
{
    if (!Y || M < 0 || N < 0 || K < 0 || m0 < 0 || m1 > M || m0 > m1) return ORC_ERR_ARG;
    if (M == 0 || N == 0) return ORC_OK;
    int32_t *Wv = (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * K + 1));
    int32_t *Xv = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N * K + 1));
    if (!Wv || !Xv) { free(Wv); free(Xv); return ORC_ERR_NOMEM; }
    int rc = K ? orc_decode(W, M * K, p, encW, Wv) : ORC_OK;
    if (!rc && K) rc = orc_decode(X, N * K, q, encX, Xv);
    int overflow = 0;
    if (!rc) {
#pragma omp parallel for schedule(static) reduction(| : overflow)
        for (int64_t m = m0; m < m1; ++m)
            for (int64_t n = 0; n < N; ++n) {
                int64_t acc = 0;
                for (int64_t k = 0; k < K; ++k)
                    acc += (int64_t)Wv[m * K + k] * (int64_t)Xv[n * K + k];
                if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                Y[m * N + n] = (int32_t)acc;
            }
    }
    free(Wv); free(Xv);
    if (rc) return rc;
    return overflow ? ORC_ERR_OVERFLOW : ORC_OK;
}

int orc_gemm(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
             int64_t M, int64_t N, int64_t K, int32_t *Y)
{
    return orc_gemm_rows(W, encW, p, X, encX, q, M, N, K, 0, M, Y);
}

int orc_conv2d(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
               int64_t BS, int64_t Cin, int64_t H, int64_t Wd, int64_t Cout,
               int R, int S, int stride, int pad, int32_t *Y)
{
    if (!Y || BS < 0 || Cin < 1 || H < 1 || Wd < 1 || Cout < 1 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return ORC_ERR_ARG;
    if (H + 2 * pad < R || Wd + 2 * pad < S) return ORC_ERR_ARG;
    const int64_t Ho = (H + 2 * pad - R) / stride + 1, Wo = (Wd + 2 * pad - S) / stride + 1;
    const int64_t nW = Cout * Cin * R * S, nX = BS * Cin * H * Wd;
    int32_t *Wv = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nW + 1));
    int32_t *Xv = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nX + 1));
    if (!Wv || !Xv) { free(Wv); free(Xv); return ORC_ERR_NOMEM; }
    int rc = orc_decode(W, nW, p, encW, Wv);
    if (!rc && nX) rc = orc_decode(X, nX, q, encX, Xv);
    int overflow = 0;
    if (!rc) {
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
        for (int64_t b = 0; b < BS; ++b)
            for (int64_t co = 0; co < Cout; ++co)
                for (int64_t ho = 0; ho < Ho; ++ho)
                    for (int64_t wo = 0; wo < Wo; ++wo) {
                        int64_t acc = 0;
                        for (int64_t c = 0; c < Cin; ++c)
                            for (int r = 0; r < R; ++r)
                                for (int s = 0; s < S; ++s) {
                                    const int64_t h = ho * stride + r - pad, w = wo * stride + s - pad;
                                    if (h < 0 || h >= H || w < 0 || w >= Wd) continue; /* adds 0 */
                                    acc += (int64_t)Wv[((co * Cin + c) * R + r) * S + s] *
                                           (int64_t)Xv[((b * Cin + c) * H + h) * Wd + w];
                                }
                        if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                        Y[((b * Cout + co) * Ho + ho) * Wo + wo] = (int32_t)acc;
                    }
    }
    free(Wv); free(Xv);
    if (rc) return rc;
    return overflow ? ORC_ERR_OVERFLOW : ORC_OK;
}

/* ---- literal AP-Bit emulation (Sec. 3.1 template + Sec. 3.2 cases) ------ */

/* bit plane s of an operand, packed 64 k-positions per word; a +-1 operand
 * stores +1 as bit 1 and -1 as bit 0 ("map -1 to 0"). */
static uint64_t *apbit_planes(const uint8_t *A, int enc, int bits, int64_t rows, int64_t K, int64_t Kw)
{
    uint64_t *P = (uint64_t *)calloc((size_t)(rows * bits * Kw + 1), sizeof(uint64_t));
    if (!P) return NULL;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            unsigned v = (enc == ORC_PM1) ? ((int8_t)A[r * K + k] > 0 ? 1u : 0u) : A[r * K + k];
            for (int s = 0; s < bits; ++s)
                if ((v >> s) & 1u)                                   /* Eq. 2 */
                    P[(r * bits + s) * Kw + k / 64] |= (uint64_t)1 << (k % 64);
        }
    return P;
}

int orc_apbit_gemm(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
                   int64_t M, int64_t N, int64_t K, int32_t *Y)
{
    if (!Y || M < 0 || N < 0 || K < 0 || p < 1 || p > 8 || q < 1 || q > 8) return ORC_ERR_ARG;
    if ((encW == ORC_PM1 && p != 1) || (encX == ORC_PM1 && q != 1)) return ORC_ERR_ARG;
    const int64_t Kw = (K + 63) / 64;
    uint64_t *Wp = apbit_planes(W, encW, p, M, K, Kw);
    uint64_t *Xp = apbit_planes(X, encX, q, N, K, Kw);
    if (!Wp || !Xp) { free(Wp); free(Xp); return ORC_ERR_NOMEM; }
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t y;
            if (encW == ORC_PM1 && encX == ORC_PM1) {
                /* Case II: n - 2 popc(XOR); pad bits are 0 in both, XOR leaves 0 */
                int64_t c = 0;
                for (int64_t j = 0; j < Kw; ++j) c += __builtin_popcountll(Wp[m * Kw + j] ^ Xp[n * Kw + j]);
                y = K - 2 * c;
            } else {
                /* Case I: sum_{s,t} 2^(s+t) popc(AND) */
                int64_t a = 0;
                for (int s = 0; s < p; ++s)
                    for (int t = 0; t < q; ++t) {
                        int64_t c = 0;
                        for (int64_t j = 0; j < Kw; ++j)
                            c += __builtin_popcountll(Wp[(m * p + s) * Kw + j] & Xp[(n * q + t) * Kw + j]);
                        a += c << (s + t);
                    }
                y = a;
                if (encW == ORC_PM1 || encX == ORC_PM1) {
                    /* Case III: What = (W+J)/2, WX = 2 What X - J X, J X being the
                     * decoded row sum of the 0/1-encoded operand (either side). */
                    const uint64_t *U = (encW == ORC_PM1) ? Xp + n * q * Kw : Wp + m * p * Kw;
                    const int ub = (encW == ORC_PM1) ? q : p;
                    int64_t jx = 0;
                    for (int t = 0; t < ub; ++t) {
                        int64_t c = 0;
                        for (int64_t j = 0; j < Kw; ++j) c += __builtin_popcountll(U[t * Kw + j]);
                        jx += c << t;
                    }
                    y = 2 * a - jx;
                }
            }
            Y[m * N + n] = (int32_t)y;
        }
    free(Wp); free(Xp);
    return ORC_OK;
}

/* ---- element-wise layers (Sec. 5.2) ------------------------------------ */

int orc_quantize(const float *x, int64_t n, float zero, float step, int bits, uint8_t *codes)
{
    if (!x || !codes || n < 0 || bits < 1 || bits > 8 || !(step > 0.0f)) return ORC_ERR_ARG;
    const float hi = (float)((1 << bits) - 1);
    for (int64_t i = 0; i < n; ++i) {
        volatile float d = x[i] - zero;       /* one rounding per operation */
        volatile float v = d / step;
        float f = floorf(v);
        if (!(f >= 0.0f)) f = 0.0f;           /* also sends NaN to 0 */
        if (f > hi) f = hi;
        codes[i] = (uint8_t)f;
    }
    return ORC_OK;
}

int orc_fold_bn(const double *gamma, const double *beta, const double *mean, const double *var,
                double eps, double z, double s, int64_t C, float *scale, float *bias)
{
    if (!gamma || !beta || !mean || !var || !scale || !bias || C < 0 || !(s > 0.0)) return ORC_ERR_ARG;
    for (int64_t c = 0; c < C; ++c) {
        const double sd = sqrt(var[c] + eps);
        scale[c] = (float)(gamma[c] / (sd * s));
        bias[c] = (float)((beta[c] - mean[c] * gamma[c] / sd - z) / s);
    }
    return ORC_OK;
}

int orc_epilogue(const int32_t *Y, int64_t BS, int64_t C, int64_t HW,
                 const float *scale, const float *bias,
                 const uint8_t *res, float res_scale, int q_out,
                 float *t_out, uint8_t *codes)
{
    if (!Y || !scale || !bias || BS < 0 || C < 0 || HW < 0) return ORC_ERR_ARG;
    if (codes && (q_out < 1 || q_out > 8)) return ORC_ERR_ARG;
    const float hi = (float)((1 << (codes ? q_out : 1)) - 1);
    for (int64_t b = 0; b < BS; ++b)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t i = 0; i < HW; ++i) {
                const int64_t idx = (b * C + c) * HW + i;
                float t = fmaf(scale[c], (float)Y[idx], bias[c]);
                if (res) t = fmaf(res_scale, (float)res[idx], t);
                if (t_out) t_out[idx] = t;
                if (codes) {
                    float f = floorf(t);
                    if (!(f >= 0.0f)) f = 0.0f;
                    if (f > hi) f = hi;
                    codes[idx] = (uint8_t)f;
                }
            }
    return ORC_OK;
}

int orc_maxpool(const uint8_t *codes, int64_t BS, int64_t C, int64_t H, int64_t Wd,
                int k, int stride, int pad, uint8_t *out)
{
    if (!codes || !out || k < 1 || stride < 1 || pad < 0 || H + 2 * pad < k || Wd + 2 * pad < k) return ORC_ERR_ARG;
    const int64_t Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
    for (int64_t bc = 0; bc < BS * C; ++bc)
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo) {
                int best = 0;
                for (int r = 0; r < k; ++r)
                    for (int s = 0; s < k; ++s) {
                        const int64_t h = ho * stride + r - pad, w = wo * stride + s - pad;
                        if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                        const int v = codes[(bc * H + h) * Wd + w];
                        if (v > best) best = v;
                    }
                out[(bc * Ho + ho) * Wo + wo] = (uint8_t)best;
            }
    return ORC_OK;
}

int orc_sumpool(const uint8_t *codes, int64_t BS, int64_t C, int64_t HW, uint8_t *out)
{
    if (!codes || !out) return ORC_ERR_ARG;
    for (int64_t bc = 0; bc < BS * C; ++bc) {
        int64_t s = 0;
        for (int64_t i = 0; i < HW; ++i) s += codes[bc * HW + i];
        if (s > 255) return ORC_ERR_OVERFLOW;
        out[bc] = (uint8_t)s;
    }
    return ORC_OK;
}

/* k x k grid pooling of int32 convolution results (Sec. 5.2: the feature map is
 * split into k x k grids, one value per grid): mode 1 = maximum, mode 2 = sum
 * (the average times k*k; the caller folds 1/(k*k) into the scale that
 * follows).  Rows / columns that do not fill a grid are dropped. */
int orc_gridpool(const int32_t *Y, int64_t BS, int64_t C, int64_t H, int64_t Wd, int k, int mode, int32_t *out)
{
    if (!Y || !out || k < 1 || (mode != 1 && mode != 2)) return ORC_ERR_ARG;
    const int64_t Hp = H / k, Wp = Wd / k;
    for (int64_t bc = 0; bc < BS * C; ++bc)
        for (int64_t hp = 0; hp < Hp; ++hp)
            for (int64_t wp = 0; wp < Wp; ++wp) {
                int64_t acc = 0;
                for (int dy = 0; dy < k; ++dy)
                    for (int dx = 0; dx < k; ++dx) {
                        const int64_t v = Y[(bc * H + hp * k + dy) * Wd + wp * k + dx];
                        if (dy == 0 && dx == 0) acc = v;
                        else if (mode == 1) acc = v > acc ? v : acc;
                        else acc += v;
                    }
                if (acc > INT32_MAX || acc < INT32_MIN) return ORC_ERR_OVERFLOW;
                out[(bc * Hp + hp) * Wp + wp] = (int32_t)acc;
            }
    return ORC_OK;
}
