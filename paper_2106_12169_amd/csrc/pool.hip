// Pooling on packed codes (Sec. 5.2).
#include "common.h"

namespace apnn {

// Max pooling directly on bit planes: the running maximum and each candidate
// are compared bit-sliced from the most significant plane down, 32 channels at
// a time, so codes are never unpacked.
__global__ __launch_bounds__(256) void maxpool_kernel(const uint32_t *__restrict__ X, uint32_t *__restrict__ out,
                                                      int64_t npix_out, int H, int W, int Ho, int Wo, int Cw,
                                                      int bits, int k, int stride, int pad)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= npix_out * Cw) return;
    const int64_t pix = idx / Cw;
    const int cw = static_cast<int>(idx - pix * Cw);
    const int wo = static_cast<int>(pix % Wo), ho = static_cast<int>((pix / Wo) % Ho);
    const int64_t n = pix / (static_cast<int64_t>(Wo) * Ho);
    uint32_t m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int r = 0; r < k; ++r) {
        const int h = ho * stride + r - pad;
        if (h < 0 || h >= H) continue;
        for (int s = 0; s < k; ++s) {
            const int w = wo * stride + s - pad;
            if (w < 0 || w >= W) continue;
            const uint32_t *src = X + (((n * H + h) * W + w) * bits) * Cw + cw;
            uint32_t c[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) c[t] = (t < bits) ? src[static_cast<int64_t>(t) * Cw] : 0u;
            uint32_t gt = 0u, eq = ~0u;
#pragma unroll
            for (int t = 7; t >= 0; --t) {
                gt |= eq & c[t] & ~m[t];
                eq &= ~(c[t] ^ m[t]);
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) m[t] = (gt & c[t]) | (~gt & m[t]);
        }
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < bits) out[(pix * bits + t) * Cw + cw] = m[t];
}

// The same for windows up to 3 x 3 and up to BITS planes: all taps are loaded before the first comparison, so the
// kernel is one memory round trip long instead of one per tap.  A tap outside the frame reads as code 0, which
// never exceeds the running maximum.
template <int BITS>
__global__ __launch_bounds__(256) void maxpool3_kernel(const uint32_t *__restrict__ X, uint32_t *__restrict__ out,
                                                       int64_t npix_out, int H, int W, int Ho, int Wo, int Cw,
                                                       int bits, int k, int stride, int pad)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= npix_out * Cw) return;
    const int64_t pix = idx / Cw;
    const int cw = static_cast<int>(idx - pix * Cw);
    const int wo = static_cast<int>(pix % Wo), ho = static_cast<int>((pix / Wo) % Ho);
    const int64_t n = pix / (static_cast<int64_t>(Wo) * Ho);
    uint32_t c[9][BITS];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int h = ho * stride + r - pad, w = wo * stride + s - pad;
            const bool ok = r < k && s < k && h >= 0 && h < H && w >= 0 && w < W;
            const uint32_t *src = X + (((n * H + h) * W + w) * bits) * Cw + cw;
#pragma unroll
            for (int t = 0; t < BITS; ++t) c[3 * r + s][t] = (ok && t < bits) ? src[static_cast<int64_t>(t) * Cw] : 0u;
        }
    uint32_t m[BITS];
#pragma unroll
    for (int t = 0; t < BITS; ++t) m[t] = c[0][t];
#pragma unroll
    for (int i = 1; i < 9; ++i) {
        uint32_t gt = 0u, eq = ~0u;
#pragma unroll
        for (int t = BITS - 1; t >= 0; --t) {
            gt |= eq & c[i][t] & ~m[t];
            eq &= ~(c[i][t] ^ m[t]);
        }
#pragma unroll
        for (int t = 0; t < BITS; ++t) m[t] = (gt & c[i][t]) | (~gt & m[t]);
    }
#pragma unroll
    for (int t = 0; t < BITS; ++t)
        if (t < bits) out[(pix * bits + t) * Cw + cw] = m[t];
}

// Global sum pooling: one block of NWAVE waves per (image, group of 64 channels); lane = channel, wave w sums
// the pixels i = w (mod NWAVE), a handful each, with all their loads in flight together (the kernel is one
// memory round trip long); wave 0 adds the partial sums and packs the result planes by ballot.  Sixteen waves
// for a small batch (few blocks, latency bound), one wave when the batch alone fills the chip.
template <int NWAVE>
__global__ __launch_bounds__(64 * NWAVE) void sumpool_kernel(const uint32_t *__restrict__ X, uint32_t *__restrict__ out,
                                                             int HW, int C, int Cw, int bits, int out_bits, int ldw)
{
    __shared__ uint32_t part[NWAVE][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.y, c = blockIdx.x * 64 + lane;
    const int cw = c >> 5, cb = c & 31;
    uint32_t sum = 0;
    if (c < C) {
        const uint32_t *src = X + static_cast<int64_t>(n) * HW * bits * Cw + cw;
#pragma unroll 4
        for (int i = wave; i < HW; i += NWAVE)
            for (int t = 0; t < bits; ++t) sum += ((src[(static_cast<int64_t>(i) * bits + t) * Cw] >> cb) & 1u) << t;
    }
    if (NWAVE > 1) {
        part[wave][lane] = sum;
        __syncthreads();
        if (wave != 0) return;
        sum = 0;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) sum += part[w][lane];
    }
    for (int b = 0; b < out_bits; ++b) {
        const unsigned long long mask = __ballot((sum >> b) & 1u);
        uint32_t *dst = out + (static_cast<int64_t>(n) * out_bits + b) * ldw + 2 * blockIdx.x;
        if (lane == 0) dst[0] = static_cast<uint32_t>(mask);
        if (lane == 32 && 2 * static_cast<int>(blockIdx.x) + 1 < ldw) dst[1] = static_cast<uint32_t>(mask >> 32);
    }
}

}  // namespace apnn

using namespace apnn;

extern "C" int apnn_maxpool(const uint32_t *X_dev, int64_t N, int64_t H, int64_t W, int64_t C, int bits, int k,
                            int stride, int pad, uint32_t *out_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_maxpool", "code", bits, APNN_ENC_UNSIGNED)) return rc;
    if (N < 0 || H < 1 || W < 1 || C < 0 || k < 1 || stride < 1 || pad < 0 || H + 2 * pad < k || W + 2 * pad < k)
        return fail(APNN_ERR_INVALID_ARG, "apnn_maxpool: bad geometry");
    if (pad >= k) return fail(APNN_ERR_INVALID_ARG, "apnn_maxpool: pad must be smaller than the window");
    if (N == 0 || C == 0) return APNN_OK;
    if (!X_dev || !out_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_maxpool: null pointer");
    const int Ho = static_cast<int>((H + 2 * pad - k) / stride + 1), Wo = static_cast<int>((W + 2 * pad - k) / stride + 1);
    const int Cw = static_cast<int>(ceil_div(C, 32));
    const int64_t npix = N * Ho * Wo;
    const unsigned grid = static_cast<unsigned>(ceil_div(npix * Cw, 256));
    if (k <= 3 && bits <= 2)
        hipLaunchKernelGGL(maxpool3_kernel<2>, dim3(grid), dim3(256), 0, as_stream(stream), X_dev, out_dev, npix,
                           static_cast<int>(H), static_cast<int>(W), Ho, Wo, Cw, bits, k, stride, pad);
    else if (k <= 3 && bits <= 4)
        hipLaunchKernelGGL(maxpool3_kernel<4>, dim3(grid), dim3(256), 0, as_stream(stream), X_dev, out_dev, npix,
                           static_cast<int>(H), static_cast<int>(W), Ho, Wo, Cw, bits, k, stride, pad);
    else
        hipLaunchKernelGGL(maxpool_kernel, dim3(grid), dim3(256), 0, as_stream(stream), X_dev, out_dev, npix,
                           static_cast<int>(H), static_cast<int>(W), Ho, Wo, Cw, bits, k, stride, pad);
    return check_launch("apnn_maxpool");
}

extern "C" int apnn_sumpool(const uint32_t *X_dev, int64_t N, int64_t H, int64_t W, int64_t C, int bits, int out_bits,
                            uint32_t *out_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_sumpool", "code", bits, APNN_ENC_UNSIGNED)) return rc;
    if (int rc = check_bits_enc("apnn_sumpool", "sum", out_bits, APNN_ENC_UNSIGNED)) return rc;
    if (N < 0 || H < 1 || W < 1 || C < 0) return fail(APNN_ERR_INVALID_ARG, "apnn_sumpool: bad geometry");
    if (H * W * ((int64_t(1) << bits) - 1) >= (int64_t(1) << out_bits))
        return fail(APNN_ERR_OVERFLOW, "apnn_sumpool: sums of %lld %d-bit codes do not fit %d bits", (long long)(H * W), bits, out_bits);
    if (N == 0 || C == 0) return APNN_OK;
    if (N > 65535) return fail(APNN_ERR_INVALID_ARG, "apnn_sumpool: batch too large");
    if (!X_dev || !out_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_sumpool: null pointer");
    const int ldw = static_cast<int>(apnn_row_words(C));
    const int Cw = static_cast<int>(ceil_div(C, 32));
    const dim3 grid(ldw / 2, static_cast<unsigned>(N));
    if (N * (ldw / 2) >= 4096)      // (measured: 17.5 against 22 us at 4096 blocks; the sixteen-wave form wins below)
        hipLaunchKernelGGL(sumpool_kernel<1>, grid, dim3(64), 0, as_stream(stream), X_dev, out_dev, static_cast<int>(H * W),
                           static_cast<int>(C), Cw, bits, out_bits, ldw);
    else
        hipLaunchKernelGGL(sumpool_kernel<16>, grid, dim3(1024), 0, as_stream(stream), X_dev, out_dev,
                           static_cast<int>(H * W), static_cast<int>(C), Cw, bits, out_bits, ldw);
    return check_launch("apnn_sumpool");
}
