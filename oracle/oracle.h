/*
 * CPU oracle for arbitrary-precision (p-bit weight x q-bit activation)
 * GEMM / convolution and the layer epilogue.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition of what the
 * GPU library must compute; it shares no code with it.  Only the tests, the
 * smoke check and the CPU-baseline leg of the benchmark may call it.
 *
 * Operands arrive UNPACKED, one stored value per byte:
 *   encoding 0 (unsigned): byte is the integer v in [0, 2^bits)
 *   encoding 1 (+-1)     : byte is the int8 value -1 or +1, bits must be 1
 *                          (Sec. 3.2: bit 0 stands for -1, bit 1 for +1)
 * Tensors use the paper's logical orders (Sec. 4.1, 4.2):
 *   W  M x K, X  N x K  (both K-contiguous),  Y  M x N int32
 *   conv weights Cout x Cin x R x S, features BS x Cin x H x W,
 *   conv output BS x Cout x Ho x Wo.
 *
 * Every function returns 0 on success, ORC_ERR_* otherwise.
 *
 * Pin status: orc_gemm, orc_conv2d, orc_apbit_gemm, orc_quantize,
 * orc_epilogue, orc_fold_bn, orc_maxpool, orc_sumpool, orc_gridpool are pinned by the
 * non-GPU tests (printed examples of Sec. 3.2, closed forms, brute force,
 * float64 library cross-checks).  The chain built from them (network.py) is
 * pinned node by node against a layer table written out in its test and
 * against library pooling / float64 products; the residual wiring itself is
 * this build's reading, since the paper prints no layer list (Sec. 5.1).
 */
#ifndef APNN_ORACLE_H
#define APNN_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_OK = 0, ORC_ERR_ARG = 1, ORC_ERR_VALUE = 2, ORC_ERR_OVERFLOW = 3, ORC_ERR_NOMEM = 4 };
enum { ORC_UNSIGNED = 0, ORC_PM1 = 1 };

int orc_threads(void);

/* Stored byte -> the integer it stands for (Sec. 3.2). */
int orc_decode(const uint8_t *stored, int64_t n, int bits, int enc, int32_t *out);

/* Y[m][n] = sum_k dec(W[m][k]) * dec(X[n][k])      (Sec. 3.1: "Y = WX"). */
int orc_gemm(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
             int64_t M, int64_t N, int64_t K, int32_t *Y);

/* Same, but only rows m0 <= m < m1 of Y are produced (Y still holds M x N). */
int orc_gemm_rows(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
                  int64_t M, int64_t N, int64_t K, int64_t m0, int64_t m1, int32_t *Y);

/* Direct convolution on decoded integers; taps outside the frame add 0
 * (Sec. 4.2 (b): every padding strategy is built to reproduce this). */
int orc_conv2d(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
               int64_t BS, int64_t Cin, int64_t H, int64_t Wd, int64_t Cout,
               int R, int S, int stride, int pad, int32_t *Y);

/* Literal AP-Bit emulation of Sec. 3: split into 1-bit planes (Eq. 2), pack,
 * AND / XOR + popcount per plane pair, shift-add by 2^(s+t) (Eq. 1), with the
 * Case I / II / III recoveries.  Exists to check the identity "bit-plane sum
 * == decoded product" against orc_gemm; it is not used as the reference. */
int orc_apbit_gemm(const uint8_t *W, int encW, int p, const uint8_t *X, int encX, int q,
                   int64_t M, int64_t N, int64_t K, int32_t *Y);

/* y = clamp(floor((x - z) / s), 0, 2^bits - 1) in fp32          (Sec. 5.2). */
int orc_quantize(const float *x, int64_t n, float zero, float step, int bits, uint8_t *codes);

/* Fold BN (Eq. 5) + zero point + step into per-channel a', b' (double
 * arithmetic, rounded once to fp32):  a' = gamma / (sqrt(var+eps) * s),
 * b' = (beta - mean*gamma/sqrt(var+eps) - z) / s. */
int orc_fold_bn(const double *gamma, const double *beta, const double *mean, const double *var,
                double eps, double z, double s, int64_t C, float *scale, float *bias);

/* Fused epilogue on a BS x C x HW int32 tensor (Sec. 5.2):
 *   t = fmaf(scale[c], (float)Y, bias[c]);  if res: t = fmaf(res_scale, (float)res, t);
 *   code = clamp(floor(t), 0, 2^q_out - 1)        (the lower clamp is the ReLU)
 * t_out and codes may each be NULL. */
int orc_epilogue(const int32_t *Y, int64_t BS, int64_t C, int64_t HW,
                 const float *scale, const float *bias,
                 const uint8_t *res, float res_scale, int q_out,
                 float *t_out, uint8_t *codes);

/* k x k max pooling on integer codes, stride/pad given; padding never wins
 * (codes are >= 0 and padded positions are skipped). */
int orc_maxpool(const uint8_t *codes, int64_t BS, int64_t C, int64_t H, int64_t Wd,
                int k, int stride, int pad, uint8_t *out);

/* Global sum pooling of codes over H x W -> BS x C (must fit 8 bits). */
int orc_sumpool(const uint8_t *codes, int64_t BS, int64_t C, int64_t HW, uint8_t *out);

/* k x k grid pooling of int32 results BS x C x H x W -> BS x C x H/k x W/k
 * (Sec. 5.2); mode 1 maximum, mode 2 sum; incomplete grids are dropped. */
int orc_gridpool(const int32_t *Y, int64_t BS, int64_t C, int64_t H, int64_t Wd, int k, int mode, int32_t *out);

#ifdef __cplusplus
}
#endif
#endif
