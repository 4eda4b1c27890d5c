// Pooling on packed codes (Sec. 5.2) and the measurement probes.
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

// Register-only AND + popcount-accumulate chain on an 8 x 8 accumulator tile.
__global__ __launch_bounds__(256) void probe_valu_kernel(uint32_t *__restrict__ out, int iters)
{
    uint32_t a[8], b[8], acc[8][8];
    const uint32_t seed = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = seed * 2654435761u + i * 40503u;
        b[i] = ~seed * 2246822519u + i * 9176u;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
            asm volatile(
                "v_and_b32 %0, %16, %17\n\tv_and_b32 %1, %16, %18\n\tv_and_b32 %2, %16, %19\n\tv_and_b32 %3, %16, %20\n\t"
                "v_and_b32 %4, %16, %21\n\tv_and_b32 %5, %16, %22\n\tv_and_b32 %6, %16, %23\n\tv_and_b32 %7, %16, %24\n\t"
                "v_bcnt_u32_b32 %8, %0, %8\n\tv_bcnt_u32_b32 %9, %1, %9\n\tv_bcnt_u32_b32 %10, %2, %10\n\t"
                "v_bcnt_u32_b32 %11, %3, %11\n\tv_bcnt_u32_b32 %12, %4, %12\n\tv_bcnt_u32_b32 %13, %5, %13\n\t"
                "v_bcnt_u32_b32 %14, %6, %14\n\tv_bcnt_u32_b32 %15, %7, %15"
                : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7),
                  "+v"(acc[i][0]), "+v"(acc[i][1]), "+v"(acc[i][2]), "+v"(acc[i][3]), "+v"(acc[i][4]),
                  "+v"(acc[i][5]), "+v"(acc[i][6]), "+v"(acc[i][7])
                : "v"(a[i]), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "v"(b[4]), "v"(b[5]), "v"(b[6]), "v"(b[7]));
        }
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * 256;
    for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
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

extern "C" int apnn_probe_valu(int blocks, int iters, uint32_t *out_dev, double *lane_ops, void *stream)
{
    clear_error();
    if (blocks < 1 || iters < 1 || !out_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_probe_valu: bad argument");
    hipLaunchKernelGGL(probe_valu_kernel, dim3(blocks), dim3(256), 0, as_stream(stream), out_dev, iters);
    if (lane_ops) *lane_ops = 128.0 * iters * 256.0 * blocks;   // 64 AND + 64 popcount-accumulate per iteration
    return check_launch("apnn_probe_valu");
}

extern "C" int apnn_probe_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream)
{
    clear_error();
    if (!src_dev || !dst_dev || bytes % 16 != 0) return fail(APNN_ERR_INVALID_ARG, "apnn_probe_copy: bad argument");
    if (!aligned16(src_dev) || !aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_probe_copy: buffers must be 16-byte aligned");
    if (bytes == 0) return APNN_OK;
    const size_t n = bytes / 16;
    const unsigned grid = static_cast<unsigned>(n / 256 + 1 < 8192 ? n / 256 + 1 : 8192);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, as_stream(stream),
                       static_cast<const uint4 *>(src_dev), static_cast<uint4 *>(dst_dev), n);
    return check_launch("apnn_probe_copy");
}
