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

// Global sum pooling and the fully connected layer that follows it, in one launch (the tail of a residual network,
// Sec. 5.1): Y[n][co] = sum_c dec(W[co][c]) * (sum over the H x W pixels of code[n][pixel][c]).
// A block of 256 threads owns one image and a tile of classes.  Phase 1 adds the pixels bit-sliced: a thread keeps an
// 8-plane counter for the 32 channels of a word and adds each pixel's planes with one full adder per plane (two
// three-input bit operations), so the sums come out as the bit planes phase 2 wants -- no unpacking, no ballots.  The
// pixels of a word are shared by up to 8 threads, each with the loads of 8 pixels in flight at once (otherwise the
// kernel is a chain of memory round trips), and their counters are added through LDS (laid out with lanes on adjacent
// words: a layout by thread made every access a 64-way bank conflict).  Phase 2: thread (class, eighth of K) runs the
// AP-Bit plane-pair sum of Sec. 3.1 over its weight words and the sum planes in LDS; the eight partial results meet
// in an LDS counter.  -1/+1 weights: Case III, 2 S - (sum of the sums), the latter from popcounts of the sum planes.
// Every block recomputes its image's sums (6 KB of reads): cheaper than a launch, while the blocks are few.
constexpr int kSumBits = 8;

__device__ __forceinline__ void bitsliced_add(uint32_t (&acc)[kSumBits], const uint32_t (&x)[kSumBits], int xbits)
{
    uint32_t carry = 0;
#pragma unroll
    for (int b = 0; b < kSumBits; ++b) {
        const uint32_t xb = b < xbits ? x[b] : 0u;
        const uint32_t s = acc[b] ^ xb ^ carry;
        carry = (acc[b] & xb) | (carry & (acc[b] ^ xb));
        acc[b] = s;
    }
}

template <int BITS>      // planes of a code, rounded up to 1, 2, 4 or 8
__global__ __launch_bounds__(256) void sumpool_fc_kernel(const uint32_t *__restrict__ X, const uint32_t *__restrict__ Wt,
                                                         int32_t *__restrict__ Y, int HW, int Cw, int bits, int Cout,
                                                         int class_tile, int p, int ldw, int pm1)
{
    constexpr int NT = 256, PIX = 8;                      // threads; pixels whose loads a thread keeps in flight together
    extern __shared__ uint32_t smem[];                    // sums [8 planes][Cw] | partial counters | total | results
    const int tid = threadIdx.x, n = blockIdx.y;
    const int PS = max(1, min(8, NT / Cw));               // threads that share the pixels of a word
    uint32_t *sums = smem;                                // [kSumBits][Cw]
    uint32_t *part = sums + kSumBits * Cw;                // [PS][kSumBits][Cw], PS Cw <= 256
    int *total = reinterpret_cast<int *>(part + kSumBits * NT);
    int *result = total + 1;                              // [class_tile]
    if (tid == 0) *total = 0;
    for (int c = tid; c < class_tile; c += NT) result[c] = 0;

    // phase 2 roles; the weight words of the first class group are fetched now and arrive during phase 1
    const int c32 = tid & 31, kq = tid >> 5;              // thread (class of a group of 32, words kq, kq + 8, ...)
    const int cls0 = blockIdx.x * class_tile;
    uint32_t w_first = 0;
    if (cls0 + c32 < Cout && kq < Cw) w_first = Wt[(static_cast<int64_t>(cls0 + c32) * p + (p - 1)) * ldw + kq];

    const uint32_t *img = X + static_cast<int64_t>(n) * HW * bits * Cw;
    for (int base = 0; base < Cw * PS; base += NT) {
        const int t = base + tid;
        if (t < Cw * PS) {
            const int part_id = t / Cw, cw = t - part_id * Cw;              // adjacent threads: adjacent channel words
            uint32_t acc[kSumBits];
#pragma unroll
            for (int b = 0; b < kSumBits; ++b) acc[b] = 0;
            for (int i0 = part_id; i0 < HW; i0 += PS * PIX) {
                uint32_t x[PIX][kSumBits];
#pragma unroll
                for (int j = 0; j < PIX; ++j) {           // all loads of the group first: one memory round trip
                    const int i = i0 + j * PS;
                    const uint32_t *px = img + static_cast<uint32_t>(min(i, HW - 1) * bits) * Cw + cw;
#pragma unroll
                    for (int b = 0; b < kSumBits; ++b) x[j][b] = (b < BITS && b < bits) ? px[static_cast<uint32_t>(b * Cw)] : 0u;
                    if (i >= HW) {
#pragma unroll
                        for (int b = 0; b < BITS; ++b) x[j][b] = 0u;
                    }
                }
#pragma unroll
                for (int j = 0; j < PIX; ++j) bitsliced_add(acc, x[j], BITS);
            }
#pragma unroll
            for (int b = 0; b < kSumBits; ++b) {
                if (PS > 1) part[(part_id * kSumBits + b) * Cw + cw] = acc[b];
                else sums[b * Cw + cw] = acc[b];
            }
        }
    }
    if (PS > 1) {
        __syncthreads();
        if (tid < Cw) {
            uint32_t acc[kSumBits];
#pragma unroll
            for (int b = 0; b < kSumBits; ++b) acc[b] = part[b * Cw + tid];
            for (int k = 1; k < PS; ++k) {
                uint32_t x[kSumBits];
#pragma unroll
                for (int b = 0; b < kSumBits; ++b) x[b] = part[(k * kSumBits + b) * Cw + tid];
                bitsliced_add(acc, x, kSumBits);
            }
#pragma unroll
            for (int b = 0; b < kSumBits; ++b) sums[b * Cw + tid] = acc[b];
        }
    }
    __syncthreads();
    if (pm1 && tid < 64) {                                // sum of the sums, for the Case III term: lane = (plane, eighth)
        const int b = tid & 7;
        int c = 0;
        for (int w = tid >> 3; w < Cw; w += 8) c += __popc(sums[b * Cw + w]);
        atomicAdd(total, c << b);
    }

    for (int g = 0; g < class_tile; g += 32) {
        const int cls = cls0 + g + c32;
        if (cls < Cout) {
            const uint32_t *wrow = Wt + static_cast<int64_t>(cls) * p * ldw;
            int y = 0;
            for (int s = p - 1; s >= 0; --s) {            // Horner over the weight planes, Eq. 1
                int acc = 0;
                for (int w = kq; w < Cw; w += 8) {
                    const uint32_t ww = (g == 0 && s == p - 1 && w == kq) ? w_first : wrow[s * ldw + w];
#pragma unroll
                    for (int b = 0; b < kSumBits; ++b) acc += __popc(ww & sums[b * Cw + w]) << b;
                }
                y = 2 * y + acc;
            }
            atomicAdd(&result[g + c32], y);
        }
    }
    __syncthreads();
    for (int c = tid; c < class_tile; c += NT) {
        if (cls0 + c < Cout) {
            int y = result[c];
            if (pm1) y = 2 * y - *total;
            Y[static_cast<int64_t>(n) * Cout + cls0 + c] = y;
        }
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

extern "C" int apnn_sumpool_fc(const uint32_t *X_dev, int64_t N, int64_t H, int64_t W, int64_t C, int bits,
                               const uint32_t *W_dev, int64_t Cout, int p, apnn_encoding encW, int32_t *Y_dev, void *stream)
{
    clear_error();
    const char *who = "apnn_sumpool_fc";
    if (int rc = check_bits_enc(who, "code", bits, APNN_ENC_UNSIGNED)) return rc;
    if (int rc = check_bits_enc(who, "weight", p, encW)) return rc;
    if (N < 0 || H < 1 || W < 1 || C < 0 || Cout < 0) return fail(APNN_ERR_INVALID_ARG, "%s: bad geometry", who);
    if (C % 32 != 0 || C == 0)
        return fail(APNN_ERR_INVALID_ARG, "%s: C = %lld must be a positive multiple of 32 (packed features)", who, (long long)C);
    if (H * W * ((int64_t(1) << bits) - 1) >= (int64_t(1) << kSumBits))
        return fail(APNN_ERR_OVERFLOW, "%s: sums of %lld %d-bit codes do not fit %d bits", who, (long long)(H * W), bits, kSumBits);
    if (int rc = check_int32_range(who, C, p, kSumBits)) return rc;
    if (N == 0 || Cout == 0) return APNN_OK;
    if (!Y_dev || !X_dev || !W_dev) return fail(APNN_ERR_INVALID_ARG, "%s: null pointer", who);
    if (!aligned16(W_dev)) return fail(APNN_ERR_ALIGNMENT, "%s: W_dev must be 16-byte aligned", who);
    if (C > 8192 || N > 65535 || H * W * bits * (C / 32) > 0x7FFFFFFF)
        return fail(APNN_ERR_UNSUPPORTED, "%s: at most 8192 channels, 65535 images and 2^31 words per image", who);
    const int Cw = static_cast<int>(C / 32), ldw = static_cast<int>(apnn_row_words(C));
    // A block per image and class tile; every block recomputes the image's sums, so the tiles widen with the batch.
    const int class_tile = N * ceil_div(Cout, 32) <= 2048 ? 32 : 256;
    // LDS: sum planes, the partial counters of up to 8 threads per word, the total, one result per class of the tile
    const size_t lds = (static_cast<size_t>(kSumBits) * Cw + kSumBits * 256 + 1 + class_tile) * sizeof(uint32_t);
    const dim3 grid(static_cast<unsigned>(ceil_div(Cout, class_tile)), static_cast<unsigned>(N));
    const int pm1 = encW == APNN_ENC_PM1 ? 1 : 0;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, dim3(256), lds, as_stream(stream), X_dev, W_dev, Y_dev, static_cast<int>(H * W), Cw,
                           bits, static_cast<int>(Cout), class_tile, p, ldw, pm1);
    };
    if (bits == 1) launch(sumpool_fc_kernel<1>);
    else if (bits == 2) launch(sumpool_fc_kernel<2>);
    else if (bits <= 4) launch(sumpool_fc_kernel<4>);
    else launch(sumpool_fc_kernel<8>);
    return check_launch(who);
}
