/*
 * apnn.h -- C ABI of the MI355X (gfx950) arbitrary-precision bit-plane
 * GEMM / convolution library (libapnn.so).
 *
 * What is computed (APNN-TC, arxiv 2106.12169):
 *   a p-bit operand and a q-bit operand are split into 1-bit planes (Eq. 2),
 *   every plane pair is multiplied with AND (or XOR) + popcount (Sec. 3.2,
 *   Cases I-III) and the pq partial results are shift-added by 2^(s+t)
 *   (Sec. 3.1), which equals the plain integer product "Y = WX".
 *   The library holds two implementations of that product over the same
 *   packed planes, with identical (exact integer) results: the plane-pair
 *   AND/XOR + popcount form above, and a form that feeds two adjacent planes
 *   at a time, as 4-bit floating-point codes, to the matrix instruction and
 *   shift-adds base-4 digit pairs instead of bit pairs.  The second is used
 *   whenever every partial sum stays exactly representable in fp32; the
 *   choice is invisible at this interface.
 *
 * Conventions shared by every entry point
 *   - Pointers named *_dev are CALLER-OWNED DEVICE memory (e.g. a PyTorch
 *     tensor's data_ptr()).  The library never allocates, frees or keeps them.
 *   - `stream` is the caller's hipStream_t passed as void* (NULL = the null
 *     stream).  Calls validate their arguments on the host, enqueue their
 *     kernels on that stream and return without synchronising.
 *   - Every function returning int returns an apnn_status; on failure nothing
 *     has been enqueued and apnn_last_error() (thread local) says why.
 *   - Packed buffers must be 16-byte aligned (APNN_ERR_ALIGNMENT otherwise).
 *
 * Bit-plane layouts (part of the ABI)
 *   Element k of a row lives in bit (k mod 32), LSB first, of 32-bit word
 *   k/32 of its plane; pad bits and pad words are 0.
 *   "matrix" layout   uint32 [rows][bits][row_words], row_words =
 *                     apnn_row_words(K) = ceil(K/32) rounded up to 4 words,
 *                     so every plane row starts 16-byte aligned.  Both GEMM
 *                     operands are K-contiguous (Sec. 4.1: W is M x K, X is
 *                     N x K).
 *   "fmap" layout     uint32 [N][H][W][bits][Cw], Cw = ceil(C/32): the
 *                     channel-major organisation of Sec. 4.2 (a) with the
 *                     planes of one pixel adjacent.  C must be a multiple of
 *                     32 wherever a packed tensor feeds a convolution.
 *   conv weights      uint32 [Cout][bits][R][S][Cw].
 *   A +-1 tensor (1 bit only, Sec. 3.2) stores +1 as bit 1 and -1 as bit 0.
 */
#ifndef APNN_H
#define APNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    APNN_OK = 0,
    APNN_ERR_INVALID_ARG = 1, /* null pointer, negative size, inconsistent description */
    APNN_ERR_UNSUPPORTED = 2, /* bits outside 1..8, +-1 with more than 1 bit, ...       */
    APNN_ERR_OVERFLOW = 3,    /* K (2^p-1)(2^q-1) >= 2^31: the int32 result could wrap  */
    APNN_ERR_ALIGNMENT = 4,   /* a packed buffer is not 16-byte aligned                 */
    APNN_ERR_DEVICE = 5       /* a HIP call failed (text in apnn_last_error)            */
} apnn_status;

typedef enum {
    APNN_ENC_UNSIGNED = 0, /* a plane bit b counts as b: value = sum_s 2^s b_s     (Case I) */
    APNN_ENC_PM1 = 1       /* a bit b stands for 2b-1 in {-1,+1}; 1-bit only (Sec. 3.2)    */
} apnn_encoding;

typedef enum { APNN_LAYOUT_NHWC = 0, APNN_LAYOUT_NCHW = 1 } apnn_layout;

typedef enum { APNN_POOL_NONE = 0, APNN_POOL_MAX2 = 1, APNN_POOL_SUM2 = 2 } apnn_pool;

/* Text of the last failure on this thread ("" if none).  Never NULL. */
const char *apnn_last_error(void);

/* ---- sizes (host only, no GPU needed) ------------------------------------ */

/* Words per plane row of the matrix layout: ceil(K/32) rounded up to 4. */
int64_t apnn_row_words(int64_t K);
/* Total words of a packed rows x K matrix with `bits` planes. 0 on bad input. */
size_t apnn_packed_words(int64_t rows, int64_t K, int bits);
/* Total words of a packed feature map: pixels * bits * ceil(C/32). */
size_t apnn_fmap_words(int64_t pixels, int64_t C, int bits);

/* ---- bit decomposition and packing (Sec. 3.1 Eq. 2, Sec. 4.2 (a)) -------- */

/* src_dev: rows x K values, one per byte, row-major.  The encoding fixes how a
 * byte is read (no separate signedness argument): UNSIGNED: uint8 in
 * [0, 2^bits) (higher bits are ignored).  PM1: int8 -1/+1 (bit = value > 0).
 * dst_dev: matrix layout, apnn_packed_words(rows, K, bits) words, fully
 * written (pad words zeroed). */
int apnn_pack(const void *src_dev, int64_t rows, int64_t K, int bits, apnn_encoding enc,
              uint32_t *dst_dev, void *stream);

/* Feature map N x H x W x C (NHWC) or N x C x H x W (NCHW), one value per
 * byte, into the fmap layout [N][H][W][bits][ceil(C/32)]. */
int apnn_pack_fmap(const void *src_dev, apnn_layout layout, int64_t N, int64_t H, int64_t W, int64_t C,
                   int bits, apnn_encoding enc, uint32_t *dst_dev, void *stream);

/* Convolution weights in the paper's logical order Cout x Cin x R x S
 * (Sec. 4.2), one value per byte, into [Cout][bits][R][S][ceil(Cin/32)]. */
int apnn_pack_conv_weights(const void *src_dev, int64_t Cout, int64_t Cin, int R, int S,
                           int bits, apnn_encoding enc, uint32_t *dst_dev, void *stream);

/* Input-layer packing for few input channels (S*C <= 32): every output
 * pixel gets the bits of its R x S x C receptive field, one 32-bit word per
 * kernel row r holding bit (c*S + s), frame overhang as 0 bits.  Source is an
 * N x C x H x W image (one unsigned value per byte).  Result is a matrix
 * operand [N*Ho*Wo][bits][apnn_row_words(32*R)] that, multiplied with weights
 * packed by apnn_pack_patch_weights, equals the R x S convolution with
 * stride/pad (Sec. 4.2, Sec. 5.1 input layer). */
int apnn_pack_patches(const uint8_t *src_dev, int64_t N, int64_t C, int64_t H, int64_t W,
                      int R, int S, int stride, int pad, int bits, uint32_t *dst_dev, void *stream);
int apnn_pack_patch_weights(const void *src_dev, int64_t Cout, int64_t Cin, int R, int S,
                            int bits, apnn_encoding enc, uint32_t *dst_dev, void *stream);

/* Quantisation layer of Sec. 5.2 fused with the packer:
 * code = clamp(floor((x - zero) / step), 0, 2^bits - 1) in fp32, then planes
 * in the matrix layout.  step > 0. */
int apnn_quantize(const float *src_dev, int64_t rows, int64_t K, float zero, float step, int bits,
                  uint32_t *dst_dev, void *stream);

/* ---- arbitrary-precision GEMM (APMM, Sec. 4.1) ---------------------------- */

/* Y[m][n] = sum_k dec(W[m][k]) * dec(X[n][k]), int32, row-major M x N.
 * W_dev: matrix layout, M rows, p planes; X_dev: matrix layout, N rows, q
 * planes; both packed for the same K.  Encoding pairs: U x U (Case I, AND),
 * PM1 x PM1 (Case II, XOR), PM1 x U or U x PM1 (Case III, AND plus the row-sum
 * term).  M, N, K >= 0 (zero-sized problems succeed and write nothing; K = 0
 * writes zeros). */
int apnn_gemm(const uint32_t *W_dev, const uint32_t *X_dev, int32_t *Y_dev,
              int64_t M, int64_t N, int64_t K, int p, int q,
              apnn_encoding encW, apnn_encoding encX, void *stream);

/* ---- arbitrary-precision convolution (APConv, Sec. 4.2) ------------------- */

typedef struct {
    int64_t N, H, W, Cin, Cout; /* batch, input frame, channels (Cin multiple of 32)    */
    int R, S, stride, pad;      /* kernel, stride, zero-contribution padding            */
    int p, q;                   /* weight bits, activation bits                         */
    apnn_encoding encW, encX;   /* -1/+1 features: see apnn_conv2d                      */
} apnn_conv_desc;

/* Y[n][ho][wo][co] = sum_{r,s,c} dec(W[co][c][r][s]) * dec(X[n][ho*stride+r-pad][wo*stride+s-pad][c]),
 * taps outside the frame contributing 0 (Sec. 4.2 (b)).  W_dev: conv-weight
 * layout; X_dev: fmap layout; Y_dev: int32 [N][Ho][Wo][Cout].
 * -1/+1 features (Case II with -1/+1 weights, or the mirror of Case III with
 * unsigned weights): a 0 bit means -1, so frame overhang cannot be left to the
 * zero words of the loader.  Every form of the product gives the features a
 * made-up validity plane instead (1 inside the frame): the matrix-instruction
 * form ANDs its operand codes with it, the AND + popcount form counts it as a
 * second, negative plane (a = 2 bit - validity).  Nothing is refused. */
int apnn_conv2d(const apnn_conv_desc *desc, const uint32_t *W_dev, const uint32_t *X_dev,
                int32_t *Y_dev, void *stream);

/* ---- fused layer: conv or GEMM + scale/bias + residual + requantise + repack
 *      (Sec. 4.1 (b) element-wise routine, Sec. 5.2 semantic-aware fusion) --- */

typedef struct {
    apnn_conv_desc conv;   /* is_gemm: activations are a matrix operand with N rows
                              (conv.N), K = conv.Cin, weights a matrix operand with
                              conv.Cout rows; H = W = R = S = stride = 1, pad = 0.   */
    int is_gemm;
    int q_out;             /* 1..8: requantise and write packed planes; 0: none      */
    const float *scale_dev;/* per-Cout folded a' and b' (fp32), required unless only */
    const float *bias_dev; /* acc_out_dev is requested                               */
    const uint32_t *residual_dev; /* optional packed codes [pixel][q_res][Cout/32]   */
    int q_res;
    float res_scale;
    int32_t *acc_out_dev;  /* optional int32 [pixel][Cout] (raw accumulators)        */
    float *float_out_dev;  /* optional fp32  [pixel][Cout] (pre-floor values)        */
    int pool;              /* APNN_POOL_NONE, or 2 x 2 grid pooling of the int32
                              convolution results before scale/bias (Sec. 5.2):
                              APNN_POOL_MAX2 maximum, APNN_POOL_SUM2 sum (= 4 x the
                              average; fold 1/4 into scale).  "pixel" below then
                              runs over [N][Ho/2][Wo/2]; incomplete grids of an
                              odd Ho or Wo are dropped.  Convolutions only
                              (APNN_ERR_INVALID_ARG with is_gemm); a pooled sum
                              that may exceed int32: APNN_ERR_OVERFLOW.              */
} apnn_layer_desc;

/* For every output (pixel, co), Y being the convolution / GEMM result or, with
 * pooling, the maximum / sum of the four results of the pixel's 2 x 2 grid:
 *   t    = fmaf(scale[co], (float)Y, bias[co]);
 *   t    = fmaf(res_scale, (float)res_code, t)            if residual_dev
 *   code = clamp(floor(t), 0, 2^q_out - 1)                (lower clamp = ReLU)
 * and the q_out planes of the codes are written in the fmap layout
 * [pixel][q_out][Cout/32] (Cout multiple of 32 when q_out > 0), ready to be
 * the next layer's X_dev.  out_packed_dev may be NULL when q_out == 0. */
int apnn_layer(const apnn_layer_desc *desc, const uint32_t *W_dev, const uint32_t *X_dev,
               uint32_t *out_packed_dev, void *stream);

/* Device scratch memory apnn_layer / apnn_layer_pair / apnn_input_layer would
 * need for `desc`, for the caller to allocate: always 0.  Every reduction of the
 * kernels (K split over the waves of a block, the row-sum term of Sec. 3.2
 * Case III) happens in registers and LDS, so no entry point takes a workspace. */
size_t apnn_workspace_bytes(const apnn_layer_desc *desc);

/* Two layers that do not depend on each other (neither reads what the other
 * writes), e.g. the 3 x 3 convolution and the 1 x 1 shortcut convolution of a
 * down-sampling residual block (Sec. 5.1): same arguments, checks and results as
 * two apnn_layer calls.  Small convolution layers of the same operand kinds
 * share one kernel launch; any other pair is launched one after the other. */
int apnn_layer_pair(const apnn_layer_desc *descA, const uint32_t *WA_dev, const uint32_t *XA_dev,
                    uint32_t *outA_packed_dev, const apnn_layer_desc *descB, const uint32_t *WB_dev,
                    const uint32_t *XB_dev, uint32_t *outB_packed_dev, void *stream);

/* ---- input layer (Sec. 5.1): 8-bit image with few channels ----------------- */

/* The image's bytes go to the 8-bit integer matrix instruction as they are: one
 * pass where the 1-bit emulation needs 8 (Sec. 6 makes the same observation for
 * 8-bit operands on large shapes), no bit decomposition of the image, same
 * integer results.
 *
 * apnn_pack_input_weights: src_dev holds Cout x Cin x R x S values, one per byte
 * (-1/+1 as int8, or unsigned codes below 2^bits, bits <= 7; S <= 16).  dst_dev
 * receives apnn_input_weight_bytes(Cout, Cin, R, S) bytes: signed-byte rows in the
 * kernel's K order, then one int32 per output channel (128 x the row sum, the
 * constant that lets the image enter as signed bytes x - 128). */
size_t apnn_input_weight_bytes(int64_t Cout, int64_t Cin, int R, int S);
int apnn_pack_input_weights(const void *src_dev, int64_t Cout, int64_t Cin, int R, int S, int bits,
                            apnn_encoding enc, void *dst_dev, void *stream);

/* Y[n][ho][wo][co] as in apnn_conv2d for image_dev = N x Cin x H x W unsigned
 * bytes (any Cin >= 1; conv.q is the number of significant bits, higher bits of a
 * byte are ignored; conv.encX must be APNN_ENC_UNSIGNED), W_dev from apnn_pack_input_weights, then the epilogue and
 * the outputs of apnn_layer (acc_out_dev, float_out_dev, residual, q_out planes in
 * [pixel][q_out][Cout/32]).  desc->is_gemm and desc->pool must be 0.
 * APNN_ERR_UNSUPPORTED unless S <= 16, W >= 8, p <= 7, Cout <= 128 and
 * 255 K max|w| < 2^24. */
int apnn_input_layer(const apnn_layer_desc *desc, const void *W_dev, const uint8_t *image_dev,
                     uint32_t *out_packed_dev, void *stream);

/* Fold batch norm (Eq. 5), zero point and step into a', b' on the host
 * (double arithmetic, one rounding to fp32):
 *   a' = gamma / (sqrt(var + eps) * step),  b' = (beta - mean*gamma/sqrt(var+eps) - zero) / step.
 * All pointers are HOST memory of C entries. */
int apnn_fold_bn(const double *gamma, const double *beta, const double *mean, const double *var,
                 double eps, double zero, double step, int64_t C, float *scale, float *bias);

/* ---- pooling on packed codes (Sec. 5.2) ----------------------------------- */

/* k x k max pooling with stride/pad on a packed fmap [N][H][W][bits][Cw];
 * out-of-frame positions never win.  Output fmap [N][Ho][Wo][bits][Cw]. */
int apnn_maxpool(const uint32_t *X_dev, int64_t N, int64_t H, int64_t W, int64_t C, int bits,
                 int k, int stride, int pad, uint32_t *out_dev, void *stream);

/* Global sum pooling over H x W of `bits`-bit codes; the sums must fit
 * out_bits (H*W*(2^bits-1) < 2^out_bits, else APNN_ERR_OVERFLOW).  Output is
 * a matrix operand [N][out_bits][apnn_row_words(C)]. */
int apnn_sumpool(const uint32_t *X_dev, int64_t N, int64_t H, int64_t W, int64_t C, int bits,
                 int out_bits, uint32_t *out_dev, void *stream);

/* Global sum pooling followed by the fully connected layer that reads it
 * (the tail of a residual network, Sec. 5.1), in one launch:
 *   Y[n][co] = sum_c dec(W[co][c]) * sum_{h,w} code[n][h][w][c].
 * X_dev: packed fmap [N][H][W][bits][C/32] (C a multiple of 32, at most 8192;
 * N at most 65535);
 * the sums must fit 8 bits (H*W*(2^bits-1) < 256, else APNN_ERR_OVERFLOW).
 * W_dev: matrix layout, Cout rows of K = C, p planes, encW as in apnn_gemm.
 * Y_dev: int32 [N][Cout], no requantisation (the last layer keeps its
 * accumulators, Sec. 5.1).  Same result as apnn_sumpool to 8 bits followed by
 * apnn_layer(is_gemm) with acc_out_dev. */
int apnn_sumpool_fc(const uint32_t *X_dev, int64_t N, int64_t H, int64_t W, int64_t C, int bits,
                    const uint32_t *W_dev, int64_t Cout, int p, apnn_encoding encW, int32_t *Y_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* APNN_H */
