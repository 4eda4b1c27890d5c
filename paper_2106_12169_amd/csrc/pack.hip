// Bit decomposition and packing kernels (Sec. 3.1 Eq. 2; channel-major
// organisation of Sec. 4.2 (a); quantisation layer of Sec. 5.2).
//
// One thread produces the 32-bit word(s) of one (row, k-word) position for all
// planes: it reads 32 source values, takes bit t of each (Eq. 2) and gathers
// them LSB-first into the word of plane t.  The work is HBM-bound: rows*K bytes
// in, rows*K*bits/8 bytes out.
#include "common.h"
#include "lane_util.h"

namespace apnn {

// 4 bytes holding 0/1 each -> 4-bit number, byte 0 in bit 0.  The multiplier
// places byte i at bit 24+i; the stray partial products all land below bit 24
// in distinct positions, so nothing carries into the result.
__device__ __forceinline__ uint32_t gather4(uint32_t ones)
{
    return (ones * 0x01020408u) >> 24;
}

// Per-byte "value > 0" for int8 bytes: low seven bits non-zero and sign clear.
__device__ __forceinline__ uint32_t positive_bytes(uint32_t d)
{
    const uint32_t nz = (((d & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) >> 7) & 0x01010101u;
    return nz & ~(d >> 7);
}

struct PackGeom {
    int64_t rows;      // logical rows (matrix rows, pixels, or Cout*R*S)
    int64_t K;         // values per row
    int64_t row_stride;// source bytes between rows (within one outer block)
    int64_t k_stride;  // source bytes between consecutive k
    int64_t outer_div; // source: row -> (row / outer_div, row % outer_div)
    int64_t outer_stride; // source bytes per outer block
    int64_t inner_n;   // destination: row -> (row / inner_n, row % inner_n)
    int ldw;           // destination words per plane row
    int bits;
    int pm1;
};

// dst word index of (row, plane t, word kw)
__device__ __forceinline__ size_t dst_index(const PackGeom &g, int64_t row, int t, int kw)
{
    const int64_t outer = row / g.inner_n, inner = row - outer * g.inner_n;
    return (static_cast<size_t>(outer * g.bits + t) * g.inner_n + inner) * g.ldw + kw;
}

__global__ __launch_bounds__(256) void pack_generic_kernel(const uint8_t *__restrict__ src,
                                                           uint32_t *__restrict__ dst, PackGeom g)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t total = g.rows * g.ldw;
    if (idx >= total) return;
    const int64_t row = idx / g.ldw;
    const int kw = static_cast<int>(idx - row * g.ldw);
    const int64_t ro = row / g.outer_div, ri = row - ro * g.outer_div;
    const uint8_t *s = src + ro * g.outer_stride + ri * g.row_stride;
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t k0 = static_cast<int64_t>(kw) * 32;
    if (g.k_stride == 1 && k0 + 32 <= g.K && ((reinterpret_cast<uintptr_t>(s + k0) & 15u) == 0)) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(s + k0);
        const uint4 hi = *reinterpret_cast<const uint4 *>(s + k0 + 16);
        const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (g.pm1) {
                w[0] |= gather4(positive_bytes(d[i])) << (4 * i);
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < g.bits) w[t] |= gather4((d[i] >> t) & 0x01010101u) << (4 * i);
            }
        }
    } else {
        for (int b = 0; b < 32; ++b) {
            const int64_t k = k0 + b;
            if (k >= g.K) break;
            const uint8_t v = s[k * g.k_stride];
            if (g.pm1) {
                w[0] |= static_cast<uint32_t>(static_cast<int8_t>(v) > 0) << b;
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < g.bits) w[t] |= ((static_cast<uint32_t>(v) >> t) & 1u) << b;
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < g.bits) dst[dst_index(g, row, t, kw)] = w[t];
}

// Quantiser + packer, one wave per 256 consecutive values of a row: lane l converts values l, l + 64, l + 128,
// l + 192 of the segment (four coalesced 4-byte loads per wave), a ballot over bit t of the i-th code is words
// 2 i and 2 i + 1 of plane t, and the 8 words x bits planes of the segment are collected by lane writes (lane
// 8 t + w) and leave in one store.  The arithmetic per value is that of quantize_pack_kernel.
__global__ __launch_bounds__(256) void quantize_pack_wave_kernel(const float *__restrict__ src, uint32_t *__restrict__ dst,
                                                                 uint32_t nseg, int segs, int K, int ldw, int bits,
                                                                 float zero, float step)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (wave >= nseg) return;                           // wave-uniform
    const uint32_t row = wave / static_cast<uint32_t>(segs);
    const int seg = static_cast<int>(wave - row * segs);
    const float *s = src + static_cast<size_t>(row) * K;
    const float hi = static_cast<float>((1 << bits) - 1);
    uint32_t code[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int k = seg * 256 + 64 * i + lane;
        uint32_t c = 0;
        if (k < K) {
            // (x - z) / s with one rounding per operation, then floor and clamp
            const float d = __fsub_rn(s[k], zero);
            const float v = __fdiv_rn(d, step);
            float f = floorf(v);
            f = (f >= 0.0f) ? f : 0.0f;          // negatives and NaN -> 0
            f = (f > hi) ? hi : f;
            c = static_cast<uint32_t>(f);
        }
        code[i] = c;
    }
    int word = 0;
    static_for<8>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        if (t < bits) {
            static_for<4>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                write_lanes<8 * t + 2 * i, 8 * t + 2 * i + 1>(word, __ballot(code[i] & (1u << t)));
            });
        }
    });
    const int t = lane >> 3, kw = seg * 8 + (lane & 7);
    if (t < bits && kw < ldw) dst[(static_cast<size_t>(row) * bits + t) * ldw + kw] = static_cast<uint32_t>(word);
}

// Row-major source (matrix operand or NHWC feature map) whose rows start 16-byte aligned: the same work as
// pack_generic_kernel with 32-bit index arithmetic and one division; the generic kernel's four 64-bit divisions per
// thread cost more vector instructions than the bit gathering itself and kept a 16 MiB operand at 2.8 TB/s.
__global__ __launch_bounds__(256) void pack_rows_kernel(const uint8_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                        uint32_t total, int K, int ldw, int bits, int pm1)
{
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const uint32_t row = idx / static_cast<uint32_t>(ldw);
    const int kw = static_cast<int>(idx - row * ldw);
    const uint8_t *s = src + static_cast<size_t>(row) * K;
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int k0 = kw * 32;
    if (k0 + 32 <= K) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(s + k0);
        const uint4 hi = *reinterpret_cast<const uint4 *>(s + k0 + 16);
        const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (pm1) {
                w[0] |= gather4(positive_bytes(d[i])) << (4 * i);
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < bits) w[t] |= gather4((d[i] >> t) & 0x01010101u) << (4 * i);
            }
        }
    } else {
        for (int b = 0; b < 32 && k0 + b < K; ++b) {
            const uint8_t v = s[k0 + b];
            if (pm1) {
                w[0] |= static_cast<uint32_t>(static_cast<int8_t>(v) > 0) << b;
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < bits) w[t] |= ((static_cast<uint32_t>(v) >> t) & 1u) << b;
            }
        }
    }
    uint32_t *o = dst + static_cast<size_t>(row) * bits * ldw + kw;
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < bits) o[static_cast<size_t>(t) * ldw] = w[t];
}

// N x C x H x W source into the fmap layout.  A block owns 256 consecutive pixels of one image: wave w takes the
// channel words w, w + 4, ...; lane = four consecutive pixels, one dword load per channel, contiguous across the
// wave.  The plane words go to an LDS image of the block's output record ([pixel][plane][channel word], the pixel
// stride padded to an odd number of words) and leave as contiguous 4-byte-per-lane stores: both sides of the
// transposition are coalesced.  H W must be a multiple of 4 and the source 4-byte aligned (otherwise the generic
// kernel, one byte per load, takes over); dynamic LDS: 256 * (bits * Cw | 1) words.
__global__ __launch_bounds__(256) void pack_nchw_kernel(const uint8_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                        int C, int HW, int Cw, int bits, int pm1, int blocks_per_image)
{
    extern __shared__ uint32_t rec[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x / blocks_per_image, p0 = (blockIdx.x - n * blocks_per_image) * 256;   // first pixel of the block
    const int npix = min(256, HW - p0);                 // a multiple of 4
    const int RW = bits * Cw, PS = RW | 1;              // words per pixel record, padded stride in LDS
    const bool have = 4 * lane < npix;
    for (int cw = wave; cw < Cw; cw += 4) {
        const uint8_t *s = src + (static_cast<size_t>(n) * C + 32 * cw) * HW + p0 + 4 * lane;
        uint32_t d[32];
#pragma unroll
        for (int c = 0; c < 32; ++c) {
            d[c] = (have && 32 * cw + c < C) ? *reinterpret_cast<const uint32_t *>(s + static_cast<size_t>(c) * HW) : 0u;
            if (pm1) d[c] = positive_bytes(d[c]);       // bit 0 of every byte: value > 0
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (t < bits) {
                    uint32_t w = 0;
#pragma unroll
                    for (int c = 0; c < 32; ++c) w |= ((d[c] >> (8 * j + t)) & 1u) << c;
                    rec[(4 * lane + j) * PS + t * Cw + cw] = w;
                }
    }
    __syncthreads();
    uint32_t *o = dst + (static_cast<size_t>(n) * HW + p0) * RW;
    for (int i = threadIdx.x; i < npix * RW; i += 256) {
        const int px = i / RW;
        o[i] = rec[px * PS + (i - px * RW)];
    }
}

__global__ __launch_bounds__(256) void quantize_pack_kernel(const float *__restrict__ src,
                                                            uint32_t *__restrict__ dst, int64_t rows,
                                                            int64_t K, int ldw, int bits, float zero,
                                                            float step)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= rows * ldw) return;
    const int64_t row = idx / ldw;
    const int kw = static_cast<int>(idx - row * ldw);
    const float hi = static_cast<float>((1 << bits) - 1);
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int b = 0; b < 32; ++b) {
        const int64_t k = static_cast<int64_t>(kw) * 32 + b;
        if (k >= K) break;
        // (x - z) / s with one rounding per operation, then floor and clamp
        const float d = __fsub_rn(src[row * K + k], zero);
        const float v = __fdiv_rn(d, step);
        float f = floorf(v);
        f = (f >= 0.0f) ? f : 0.0f;          // negatives and NaN -> 0
        f = (f > hi) ? hi : f;
        const uint32_t code = static_cast<uint32_t>(f);
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (t < bits) w[t] |= ((code >> t) & 1u) << b;
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < bits) dst[(static_cast<size_t>(row) * bits + t) * ldw + kw] = w[t];
}

// Input-layer receptive-field packing: word r of an output pixel holds bit
// (c*S + s) = bit t of image[n][c][ho*stride+r-pad][wo*stride+s-pad].
//
// Row kernel (the usual case).  With the taps of one channel adjacent in the word,
// the S bits of (pixel, r, c, t) are S consecutive bits of the bit string "plane t of
// image row h, channel c".  A block owns one output row (n, ho): it first splits the
// R x C image rows it needs into plane bit strings in LDS (one thread per 32 pixels,
// the same byte gather as the matrix packer; two zero words in front and behind take
// the place of the frame overhang), then every thread assembles output words from
// S-bit fields cut out of those strings with a funnel shift and writes them as
// 16-byte vectors in destination order.  Per output word: C x (two LDS reads, one
// funnel shift, one mask-and-insert) instead of S*C byte loads and gathers.
__global__ __launch_bounds__(256) void pack_patches_rows_kernel(const uint8_t *__restrict__ img,
                                                                uint32_t *__restrict__ dst, int C, int H, int W,
                                                                int Ho, int Wo, int R, int S, int stride, int pad,
                                                                int bits, int LDW, int RW)
{
    extern __shared__ uint32_t rows[];                  // [R][C][bits][RW]; the string starts at word 1
    const int tid = threadIdx.x;
    const int ho = blockIdx.x % Ho;
    const int64_t n = blockIdx.x / Ho;
    const int Ww = (W + 31) / 32;
    for (int i = tid; i < R * C * bits * RW; i += 256) rows[i] = 0;
    __syncthreads();
    for (int item = tid; item < R * C * Ww; item += 256) {
        const int j = item % Ww, rc = item / Ww, c = rc % C, r = rc / C;
        const int h = ho * stride - pad + r;
        if (h < 0 || h >= H) continue;
        const uint8_t *src = img + ((n * C + c) * H + h) * static_cast<int64_t>(W) + 32 * j;
        uint32_t d[8];
        if (32 * j + 32 <= W && (reinterpret_cast<uintptr_t>(src) & 3u) == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) d[i] = reinterpret_cast<const uint32_t *>(src)[i];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                d[i] = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if (32 * j + 4 * i + b < W) d[i] |= static_cast<uint32_t>(src[4 * i + b]) << (8 * b);
            }
        }
        for (int t = 0; t < bits; ++t) {
            uint32_t w = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) w |= gather4((d[i] >> t) & 0x01010101u) << (4 * i);
            rows[((r * C + c) * bits + t) * RW + 1 + j] = w;
        }
    }
    __syncthreads();
    const uint32_t field = (1u << S) - 1u;
    const int Q = LDW / 4;                              // 16-byte vectors per (pixel, plane)
    uint32_t *out = dst + (static_cast<int64_t>(blockIdx.x) * Wo) * bits * LDW;
    for (int v = tid; v < Wo * bits * Q; v += 256) {
        const int q = v % Q, t = (v / Q) % bits, wo = v / (Q * bits);
        const int xb = wo * stride - pad + 32;          // bit position of tap s = 0 in the string (>= 0: pad <= 32)
        const int wi = xb >> 5, sh = xb & 31;
        uint32_t w4[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int r = 4 * q + k;
            uint32_t w = 0;
            if (r < R) {
                for (int c = 0; c < C; ++c) {
                    const uint32_t *str = &rows[((r * C + c) * bits + t) * RW + wi];
                    w |= (__funnelshift_r(str[0], str[1], sh) & field) << (c * S);
                }
            }
            w4[k] = w;
        }
        *reinterpret_cast<uint4 *>(out + static_cast<int64_t>(v) * 4) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
    }
}

// General kernel (any geometry that fits the word): a block handles 32 output
// pixels; thread (pixel, r) collects the S*C bytes of kernel row
// r four to a register, every plane takes one bit of each byte with the same
// gather as the row packer, and the 32 x bits x ldw words of the block, which are
// contiguous in the destination, leave through LDS as coalesced 16-byte stores.
__global__ __launch_bounds__(256) void pack_patches_kernel(const uint8_t *__restrict__ img,
                                                           uint32_t *__restrict__ dst, int64_t npix,
                                                           int C, int H, int W, int Ho, int Wo, int R, int S,
                                                           int stride, int pad, int bits, int LDW)
{
    // LDW = words per plane row, 4 or 8 (host checks R <= 8)
    __shared__ __attribute__((aligned(16))) uint32_t tile[32 * 8 * 8];
    const int tid = threadIdx.x;
    const int r = tid & 7, lp = tid >> 3;                // kernel row, pixel inside the block
    const int64_t pix = static_cast<int64_t>(blockIdx.x) * 32 + lp;
    uint32_t d[8] = {0, 0, 0, 0, 0, 0, 0, 0};            // byte (c*S + s) of the kernel row, 4 per register
    if (pix < npix) {
        const int wo = static_cast<int>(pix % Wo);
        const int ho = static_cast<int>((pix / Wo) % Ho);
        const int64_t n = pix / (static_cast<int64_t>(Wo) * Ho);
        const int h = ho * stride + r - pad;
        if (r < R && h >= 0 && h < H) {
            const int x0 = wo * stride - pad;
            int sc = 0, c = 0;                               // i = c*S + sc, stepped without dividing
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int x = x0 + sc;
                if (i < S * C && x >= 0 && x < W)
                    d[i >> 2] |= static_cast<uint32_t>(img[((n * C + c) * H + h) * W + x]) << (8 * (i & 3));
                if (++sc == S) { sc = 0; ++c; }
            }
        }
    }
    for (int t = 0; t < bits; ++t) {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) w |= gather4((d[i] >> t) & 0x01010101u) << (4 * i);
        if (r < LDW) tile[(lp * bits + t) * LDW + r] = w;
    }
    __syncthreads();
    const int64_t base = static_cast<int64_t>(blockIdx.x) * 32 * bits * LDW;      // words
    const int64_t limit = npix * bits * LDW;
    for (int v = tid; v < 32 * bits * LDW / 4; v += 256)
        if (base + 4 * v < limit)
            *reinterpret_cast<uint4 *>(dst + base + 4 * v) = *reinterpret_cast<const uint4 *>(&tile[4 * v]);
}

__global__ __launch_bounds__(256) void pack_patch_weights_kernel(const uint8_t *__restrict__ wsrc,
                                                                 uint32_t *__restrict__ dst, int Cout, int Cin,
                                                                 int R, int S, int bits, int pm1, int ldw)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Cout * ldw) return;
    const int co = idx / ldw, r = idx - co * ldw;
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (r < R) {
        for (int s = 0; s < S; ++s)
            for (int c = 0; c < Cin; ++c) {
                const uint8_t v = wsrc[((static_cast<size_t>(co) * Cin + c) * R + r) * S + s];
                if (pm1) {
                    w[0] |= static_cast<uint32_t>(static_cast<int8_t>(v) > 0) << (c * S + s);
                } else {
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        if (t < bits) w[t] |= ((static_cast<uint32_t>(v) >> t) & 1u) << (c * S + s);
                }
            }
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < bits) dst[(static_cast<size_t>(co) * bits + t) * ldw + r] = w[t];
}

static int launch_pack(const char *who, const void *src, uint32_t *dst, const PackGeom &g, void *stream)
{
    const int64_t total = g.rows * g.ldw;
    if (total == 0) return APNN_OK;
    if (total > (int64_t(1) << 38)) return fail(APNN_ERR_INVALID_ARG, "%s: tensor too large", who);
    const unsigned grid = static_cast<unsigned>(ceil_div(total, 256));
    // plain rows of K contiguous bytes, every row 16-byte aligned, destination planes of a row adjacent
    const bool rows_form = g.k_stride == 1 && g.row_stride == g.K && g.outer_div == g.rows && g.inner_n == 1 &&
                           g.K % 16 == 0 && aligned16(src) && total < (int64_t(1) << 32) - 256 && g.K <= INT32_MAX;
    if (rows_form)
        hipLaunchKernelGGL(pack_rows_kernel, dim3(grid), dim3(256), 0, as_stream(stream), static_cast<const uint8_t *>(src),
                           dst, static_cast<uint32_t>(total), static_cast<int>(g.K), g.ldw, g.bits, g.pm1);
    else
        hipLaunchKernelGGL(pack_generic_kernel, dim3(grid), dim3(256), 0, as_stream(stream),
                           static_cast<const uint8_t *>(src), dst, g);
    return check_launch(who);
}

}  // namespace apnn

using namespace apnn;

extern "C" int apnn_pack(const void *src_dev, int64_t rows, int64_t K, int bits, apnn_encoding enc,
                         uint32_t *dst_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_pack", "operand", bits, enc)) return rc;
    if (rows < 0 || K < 0) return fail(APNN_ERR_INVALID_ARG, "apnn_pack: negative size");
    if (rows == 0 || K == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_pack: null pointer");
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_pack: dst_dev not 16-byte aligned");
    PackGeom g{rows, K, K, 1, rows, 0, 1, static_cast<int>(apnn_row_words(K)), bits, enc == APNN_ENC_PM1};
    if (apnn_row_words(K) > INT32_MAX) return fail(APNN_ERR_INVALID_ARG, "apnn_pack: K too large");
    return launch_pack("apnn_pack", src_dev, dst_dev, g, stream);
}

extern "C" int apnn_pack_fmap(const void *src_dev, apnn_layout layout, int64_t N, int64_t H, int64_t W,
                              int64_t C, int bits, apnn_encoding enc, uint32_t *dst_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_pack_fmap", "feature", bits, enc)) return rc;
    if (N < 0 || H < 0 || W < 0 || C < 0) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_fmap: negative size");
    if (layout != APNN_LAYOUT_NHWC && layout != APNN_LAYOUT_NCHW)
        return fail(APNN_ERR_INVALID_ARG, "apnn_pack_fmap: unknown layout %d", static_cast<int>(layout));
    if (N * H * W * C == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_fmap: null pointer");
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_pack_fmap: dst_dev not 16-byte aligned");
    const int64_t HW = H * W;
    PackGeom g;
    g.rows = N * HW; g.K = C; g.inner_n = 1; g.ldw = static_cast<int>(ceil_div(C, 32));
    g.bits = bits; g.pm1 = enc == APNN_ENC_PM1;
    if (layout == APNN_LAYOUT_NHWC) {
        g.row_stride = C; g.k_stride = 1; g.outer_div = g.rows; g.outer_stride = 0;
    } else {
        g.row_stride = 1; g.k_stride = HW; g.outer_div = HW; g.outer_stride = C * HW;
        const int64_t bpi = ceil_div(HW, 256), lds = 4 * 256 * ((static_cast<int64_t>(bits) * g.ldw) | 1);
        if (HW % 4 == 0 && (reinterpret_cast<uintptr_t>(src_dev) & 3u) == 0 && N * bpi <= 0x7FFFFFFF && lds <= 48 * 1024 &&
            HW <= INT32_MAX - 256 && C <= INT32_MAX - 32) {
            hipLaunchKernelGGL(pack_nchw_kernel, dim3(static_cast<unsigned>(N * bpi)), dim3(256), static_cast<size_t>(lds),
                               as_stream(stream), static_cast<const uint8_t *>(src_dev), dst_dev, static_cast<int>(C),
                               static_cast<int>(HW), g.ldw, bits, g.pm1, static_cast<int>(bpi));
            return check_launch("apnn_pack_fmap");
        }
    }
    return launch_pack("apnn_pack_fmap", src_dev, dst_dev, g, stream);
}

extern "C" int apnn_pack_conv_weights(const void *src_dev, int64_t Cout, int64_t Cin, int R, int S, int bits,
                                      apnn_encoding enc, uint32_t *dst_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_pack_conv_weights", "weight", bits, enc)) return rc;
    if (Cout < 0 || Cin < 0 || R < 1 || S < 1) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_conv_weights: bad size");
    if (Cout * Cin == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_conv_weights: null pointer");
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_pack_conv_weights: dst_dev not 16-byte aligned");
    const int64_t RS = static_cast<int64_t>(R) * S;
    PackGeom g;
    g.rows = Cout * RS; g.K = Cin;           // a "row" is one (cout, r, s) tap, its values are the channels
    g.row_stride = 1; g.k_stride = RS;       // source Cout x Cin x R x S: tap index is contiguous, channels stride RS
    g.outer_div = RS; g.outer_stride = Cin * RS;
    g.inner_n = RS; g.ldw = static_cast<int>(ceil_div(Cin, 32));
    g.bits = bits; g.pm1 = enc == APNN_ENC_PM1;
    return launch_pack("apnn_pack_conv_weights", src_dev, dst_dev, g, stream);
}

extern "C" int apnn_pack_patches(const uint8_t *src_dev, int64_t N, int64_t C, int64_t H, int64_t W, int R, int S,
                                 int stride, int pad, int bits, uint32_t *dst_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_pack_patches", "image", bits, APNN_ENC_UNSIGNED)) return rc;
    if (N < 0 || C < 1 || H < 1 || W < 1 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return fail(APNN_ERR_INVALID_ARG, "apnn_pack_patches: bad geometry");
    if (static_cast<int64_t>(S) * C > 32)
        return fail(APNN_ERR_UNSUPPORTED, "apnn_pack_patches: S*C = %lld bits do not fit one word", (long long)(S * C));
    if (H + 2 * pad < R || W + 2 * pad < S) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_patches: kernel larger than padded frame");
    if (N == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_patches: null pointer");
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_pack_patches: dst_dev not 16-byte aligned");
    const int Ho = static_cast<int>((H + 2 * pad - R) / stride + 1), Wo = static_cast<int>((W + 2 * pad - S) / stride + 1);
    if (R > 8) return fail(APNN_ERR_UNSUPPORTED, "apnn_pack_patches: kernel height %d above 8", R);
    const int ldw = static_cast<int>(apnn_row_words(32 * static_cast<int64_t>(R)));
    const int64_t npix = N * Ho * Wo;
    // row kernel: needs pad <= 32 (non-negative string positions) and the plane strings of R x C rows in LDS
    const int rw = static_cast<int>((W + 31) / 32) + 4;
    const size_t lds = static_cast<size_t>(R) * C * bits * rw * sizeof(uint32_t);
    if (pad <= 32 && lds <= 48 * 1024 && N * Ho <= 0x7FFFFFFF && (N * C * H * W) < (int64_t(1) << 40)) {
        hipLaunchKernelGGL(pack_patches_rows_kernel, dim3(static_cast<unsigned>(N * Ho)), dim3(256), lds, as_stream(stream),
                           src_dev, dst_dev, static_cast<int>(C), static_cast<int>(H), static_cast<int>(W), Ho, Wo, R, S,
                           stride, pad, bits, ldw, rw);
        return check_launch("apnn_pack_patches");
    }
    const unsigned grid = static_cast<unsigned>(ceil_div(npix, 32));
    hipLaunchKernelGGL(pack_patches_kernel, dim3(grid), dim3(256), 0, as_stream(stream), src_dev, dst_dev, npix,
                       static_cast<int>(C), static_cast<int>(H), static_cast<int>(W), Ho, Wo, R, S, stride, pad, bits, ldw);
    return check_launch("apnn_pack_patches");
}

extern "C" int apnn_pack_patch_weights(const void *src_dev, int64_t Cout, int64_t Cin, int R, int S, int bits,
                                       apnn_encoding enc, uint32_t *dst_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_pack_patch_weights", "weight", bits, enc)) return rc;
    if (Cout < 0 || Cin < 1 || R < 1 || S < 1) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_patch_weights: bad size");
    if (static_cast<int64_t>(S) * Cin > 32)
        return fail(APNN_ERR_UNSUPPORTED, "apnn_pack_patch_weights: S*Cin = %lld bits do not fit one word", (long long)(S * Cin));
    if (Cout == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_pack_patch_weights: null pointer");
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_pack_patch_weights: dst_dev not 16-byte aligned");
    const int ldw = static_cast<int>(apnn_row_words(32 * static_cast<int64_t>(R)));
    const unsigned grid = static_cast<unsigned>(ceil_div(Cout * ldw, 256));
    hipLaunchKernelGGL(pack_patch_weights_kernel, dim3(grid), dim3(256), 0, as_stream(stream),
                       static_cast<const uint8_t *>(src_dev), dst_dev, static_cast<int>(Cout), static_cast<int>(Cin), R, S,
                       bits, enc == APNN_ENC_PM1 ? 1 : 0, ldw);
    return check_launch("apnn_pack_patch_weights");
}

extern "C" int apnn_quantize(const float *src_dev, int64_t rows, int64_t K, float zero, float step, int bits,
                             uint32_t *dst_dev, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_quantize", "output", bits, APNN_ENC_UNSIGNED)) return rc;
    if (rows < 0 || K < 0) return fail(APNN_ERR_INVALID_ARG, "apnn_quantize: negative size");
    if (!(step > 0.0f)) return fail(APNN_ERR_INVALID_ARG, "apnn_quantize: step must be > 0");
    if (rows == 0 || K == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_quantize: null pointer");
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "apnn_quantize: dst_dev not 16-byte aligned");
    const int ldw = static_cast<int>(apnn_row_words(K));
    const int64_t segs = ceil_div(K, 256), nseg = rows * segs;
    if (nseg < (int64_t(1) << 32) - 4 && K <= INT32_MAX) {
        hipLaunchKernelGGL(quantize_pack_wave_kernel, dim3(static_cast<unsigned>(ceil_div(nseg, 4))), dim3(256), 0,
                           as_stream(stream), src_dev, dst_dev, static_cast<uint32_t>(nseg), static_cast<int>(segs),
                           static_cast<int>(K), ldw, bits, zero, step);
    } else {
        const unsigned grid = static_cast<unsigned>(ceil_div(rows * ldw, 256));
        hipLaunchKernelGGL(quantize_pack_kernel, dim3(grid), dim3(256), 0, as_stream(stream), src_dev, dst_dev, rows, K,
                           ldw, bits, zero, step);
    }
    return check_launch("apnn_quantize");
}
