// Input layer (Sec. 5.1): convolution of an 8-bit image with few channels,
// followed by the fused epilogue that quantises to the network's activation
// bits.
//
// An operand of 8 bits would take eight plane passes in the AND+popcount form and
// four digit passes in the FP4 form; the built-in 8-bit integer matrix instruction
// takes one, reads the image bytes as they are and needs no bit decomposition, so
// for this layer it is the better primitive (the same observation as in the
// evaluation of APMM against int8 GEMM on large shapes, Sec. 6).  The results
// are the same integers.
//
// Implicit GEMM straight from the N x C x H x W image: row = output pixel,
// column = output channel, K position (c, r, s) at byte ((c R + r) SEG + s / 8) * 8
// + s % 8 of a K row, SEG = 1 for S <= 8 and 2 for S <= 16 (bytes s >= S carry
// weight 0).  One K segment of a pixel is thus 8 consecutive image bytes, one
// unaligned 8-byte load per lane.  The matrix
// instruction multiplies signed bytes: image bytes enter as x - 128 (one XOR) and
// the per-channel constant 128 * sum_k w[k], made by the weight packer, is added
// back in the epilogue; positions outside the frame are x = 0, i.e. -128, and are
// covered by the same constant (zero-contribution padding, Sec. 4.2 (b)).
#include "common.h"
#include "mfma_kernel.h"

namespace apnn {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

struct InputParams {
    const uint8_t *img;     // N x C x H x W bytes
    const int8_t *w;        // Cout x Kp signed bytes
    const int32_t *cterm;   // Cout: 128 * sum of the row's weights
    int C, Kp, KS, nseg;    // channels, bytes per weight row, steps of 32 bytes, K segments C * R * SEG
    float invR;
    uint32_t xmask;         // (2^q - 1) in every byte: image bits above the q significant ones are ignored
};

// One wave per 32-pixel row tile, all NT column tiles of 32 channels; steps of 32 K bytes:
// lane (half lh, row lr) supplies K bytes 16 lh .. 16 lh + 15 of a step, two segments.
// SEG: 8-byte segments per kernel row (1: S <= 8, 2: S <= 16); a lane's two segments of a step are then the two halves
// of one kernel row.
template <int NT, int SEG> __global__ __launch_bounds__(256, NT <= 2 ? 4 : 2) void input_conv_kernel(const MfmaParams p, const InputParams q)
{
    constexpr int GS = 6;                               // steps whose loads are in flight together
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 31, lh = lane >> 5;
    const int m0 = (blockIdx.x * 4 + wave) * 32;
    if (m0 >= p.M) return;                              // wave-uniform

    const int gm = m0 + lr;
    const bool a_ok = gm < p.M;
    int n, ho, wo;
    conv_row_to_pixel(p, a_ok ? gm : 0, n, ho, wo);
    const int h0 = ho * p.stride - p.pad, x0 = wo * p.stride - p.pad;
    // The 8 bytes are loaded from a start clamped into the image row and shifted into place;
    // the bytes shifted in are the zeros of the positions left and right of the frame.
    bool col_ok[SEG];
    int shl[SEG], shr[SEG], img_base[SEG];
#pragma unroll
    for (int g = 0; g < SEG; ++g) {
        const int xg = x0 + 8 * g, xs = min(max(xg, 0), p.W - 8), delta = xs - xg;
        col_ok[g] = a_ok && delta > -8 && delta < 8;
        shl[g] = delta > 0 ? 8 * delta : 0;
        shr[g] = delta < 0 ? -8 * delta : 0;
        img_base[g] = n * q.C * p.H * p.W + xs;
    }

    // per-channel parameters of the epilogue: fetched now, their latency hides behind the main loop
    bool cok[NT];
    float sc[NT], bi[NT];
    int ct[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int gn = 32 * j + lr;
        cok[j] = gn < p.N;
        sc[j] = 0.0f; bi[j] = 0.0f; ct[j] = 0;
        if (cok[j]) {
            ct[j] = q.cterm[gn];
            if (p.scale) { sc[j] = p.scale[gn]; bi[j] = p.bias[gn]; }
        }
    }

    v16i_t acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0;

    for (int s0 = 0; s0 < q.KS; s0 += GS) {
        uint64_t xa[GS][2];
        v4i_t wb[GS][NT];
#pragma unroll
        for (int g = 0; g < GS; ++g) {
            const int s = s0 + g;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int seg = 4 * s + 2 * lh + e;
                const int sg = SEG == 2 ? e : 0;                   // (4 s + 2 lh is even: segment e of the lane is half e of a kernel row)
                const int krow = SEG == 2 ? 2 * s + lh : seg;      // kernel row (c, r)
                const int c = static_cast<int>((static_cast<float>(krow) + 0.5f) * q.invR);
                const int h = h0 + (krow - c * p.R);
                uint64_t v = 0;
                if (col_ok[sg] && seg < q.nseg && h >= 0 && h < p.H)
                    __builtin_memcpy(&v, q.img + img_base[sg] + (c * p.H + h) * p.W, 8);
                xa[g][e] = v;
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int gn = 32 * j + lr;
                v4i_t b = {0, 0, 0, 0};
                if (s < q.KS && gn < p.N) b = *reinterpret_cast<const v4i_t *>(q.w + gn * q.Kp + 32 * s + 16 * lh);
                wb[g][j] = b;
            }
        }
#pragma unroll
        for (int g = 0; g < GS; ++g) {
            if (s0 + g < q.KS) {
                // (x & mask) ^ 0x80 per byte as one three-input bit operation (truth table a:0xF0, b:0xCC, c:0xAA)
                constexpr int AND_XOR = (0xF0 & 0xCC) ^ 0xAA;
                const uint64_t v0 = (xa[g][0] << shl[0]) >> shr[0], v1 = (xa[g][1] << shl[SEG - 1]) >> shr[SEG - 1];
                auto signed_bytes = [&](uint32_t x) {
                    return static_cast<int>(__builtin_amdgcn_bitop3_b32(x, q.xmask, 0x80808080u, AND_XOR));
                };
                const v4i_t a = {signed_bytes(static_cast<uint32_t>(v0)), signed_bytes(static_cast<uint32_t>(v0 >> 32)),
                                 signed_bytes(static_cast<uint32_t>(v1)), signed_bytes(static_cast<uint32_t>(v1 >> 32))};
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wb[g][j], acc[j], 0, 0, 0);
            }
        }
    }

    // Epilogue: the arithmetic of finish_value, written for few vector instructions per output value.  A wave
    // has 2048 output values and a SIMD about three such waves; the first version spent 50 - 90 instructions
    // per value and took longer than the rest of the kernel.  Row validity and addresses are lane constants made
    // once, and the words of a plane are collected by lane writes, one per lane, and leave in whole-wave stores:
    // word (row, tile j) of the 32 x NT words of a plane sits in lane (row NT + j) mod 64 of register
    // (row NT + j) / 64.
    // The optional outputs are separate passes over the accumulator registers, each behind one uniform branch.
    constexpr int WR = (32 * NT + 63) / 64;
    const int rows_left = p.M - m0 - 4 * lh;            // accumulator register r is a real row iff row_lo(r) < rows_left
    const int64_t first = static_cast<int64_t>(m0 + 4 * lh);
    auto row_lo = [](int r) { return 8 * (r >> 2) + (r & 3); };     // lane half 0; half 1 has row_lo + 4
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] += ct[j];
    if (p.Y) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            int32_t *yp = p.Y + first * p.N + 32 * j + lr;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (cok[j] && row_lo(r) < rows_left) yp[static_cast<int64_t>(row_lo(r)) * p.N] = acc[j][r];
        }
    }
    if (!p.scale) return;
    float t[NT][16];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) t[j][r] = __fmaf_rn(sc[j], static_cast<float>(acc[j][r]), bi[j]);
    if (p.res) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t *rp = p.res + first * p.q_res * p.NW + j;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                uint32_t code = 0;
                if (cok[j] && row_lo(r) < rows_left)
                    for (int b = 0; b < p.q_res; ++b) code |= ((rp[(row_lo(r) * p.q_res + b) * p.NW] >> lr) & 1u) << b;
                t[j][r] = __fmaf_rn(p.res_scale, static_cast<float>(code), t[j][r]);
            }
        }
    }
    if (p.T) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            float *tp = p.T + first * p.N + 32 * j + lr;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (cok[j] && row_lo(r) < rows_left) tp[static_cast<int64_t>(row_lo(r)) * p.N] = t[j][r];
        }
    }
    if (!p.out) return;
    // (N is a multiple of 32 from here on: every lane has a channel)
    const int64_t out_row = static_cast<int64_t>(p.q_out) * p.NW;
    auto store_plane = [&](int b, const int (&words)[WR]) {
#pragma unroll
        for (int w = 0; w < WR; ++w) {
            const int slot = 64 * w + lane, row = slot / NT, j = slot - row * NT;
            if (row < 32 && m0 + row < p.M) p.out[(m0 + row) * out_row + b * p.NW + j] = static_cast<uint32_t>(words[w]);
        }
    };
    // both rows of a ballot into the plane's word registers
    auto gather = [&](auto jc, auto rc, int (&words)[WR], unsigned long long bal) {
        constexpr int j = decltype(jc)::value, r = decltype(rc)::value;
        constexpr int s_lo = (8 * (r >> 2) + (r & 3)) * NT + j, s_hi = s_lo + 4 * NT;
        if constexpr ((s_lo >> 6) == (s_hi >> 6)) {
            write_lanes<(s_lo & 63), (s_hi & 63)>(words[s_lo >> 6], bal);
        } else {                                        // (three column tiles: a row pair can straddle two registers)
            write_lanes<(s_lo & 63), (s_lo & 63)>(words[s_lo >> 6], (bal & 0xFFFFFFFFull) | (bal << 32));
            write_lanes<(s_hi & 63), (s_hi & 63)>(words[s_hi >> 6], (bal >> 32) | (bal & 0xFFFFFFFF00000000ull));
        }
    };
    if (p.q_out <= 2) {
        // one or two planes straight from compares of t (as in finish_rows8): bit 1 = t >= 2,
        // bit 0 = (1 <= t < 2) or t >= 3; one plane: bit 0 = t >= 1
        int w0[WR], w1[WR];
#pragma unroll
        for (int w = 0; w < WR; ++w) { w0[w] = 0; w1[w] = 0; }
        static_for<NT>([&](auto jc) {
            static_for<16>([&](auto rc) {
                const float tv = t[decltype(jc)::value][decltype(rc)::value];
                const unsigned long long c1 = __ballot(tv >= 1.0f);
                if (p.q_out == 1) {
                    gather(jc, rc, w0, c1);
                } else {
                    const unsigned long long c2 = __ballot(tv >= 2.0f), c3 = __ballot(tv >= 3.0f);
                    gather(jc, rc, w0, (c1 & ~c2) | c3);
                    gather(jc, rc, w1, c2);
                }
            });
        });
        store_plane(0, w0);
        if (p.q_out == 2) store_plane(1, w1);
        return;
    }
    const float qmax = static_cast<float>((1 << p.q_out) - 1);
    uint32_t code[NT][16];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float f = floorf(t[j][r]);
            f = (f >= 0.0f) ? f : 0.0f;
            f = (f > qmax) ? qmax : f;
            code[j][r] = static_cast<uint32_t>(f);
        }
#pragma unroll 1
    for (int b = 0; b < p.q_out; ++b) {
        int words[WR];
#pragma unroll
        for (int w = 0; w < WR; ++w) words[w] = 0;
        static_for<NT>([&](auto jc) {
            static_for<16>([&](auto rc) {
                gather(jc, rc, words, __ballot(code[decltype(jc)::value][decltype(rc)::value] & (1u << b)));
            });
        });
        store_plane(b, words);
    }
}

// Signed-byte weight rows in the kernel's K order; values -1/+1, or unsigned codes below 2^bits.
__global__ __launch_bounds__(256) void input_weights_kernel(const uint8_t *__restrict__ src, int8_t *__restrict__ dst,
                                                            int Cout, int C, int R, int S, int Kp, int bits, int pm1)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Cout * Kp) return;
    const int co = idx / Kp, k = idx - co * Kp;
    const int nsg = S > 8 ? 2 : 1;                      // 8-byte segments per kernel row
    const int seg = k >> 3, krow = seg / nsg, s = (seg - krow * nsg) * 8 + (k & 7);
    const int c = krow / R, r = krow - c * R;
    int v = 0;
    if (c < C && s < S) {
        const uint8_t b = src[((static_cast<size_t>(co) * C + c) * R + r) * S + s];
        v = pm1 ? (static_cast<int8_t>(b) > 0 ? 1 : -1) : (b & ((1 << bits) - 1));
    }
    dst[idx] = static_cast<int8_t>(v);
}

__global__ __launch_bounds__(256) void input_cterm_kernel(const int8_t *__restrict__ w, int32_t *__restrict__ cterm, int Cout,
                                                          int Kp)
{
    const int co = blockIdx.x * 256 + threadIdx.x;
    if (co >= Cout) return;
    int sum = 0;
    for (int k = 0; k < Kp; ++k) sum += w[static_cast<size_t>(co) * Kp + k];
    cterm[co] = 128 * sum;
}

static int64_t input_row_bytes(int64_t Cin, int R, int S) { return round_up(Cin * R * (S > 8 ? 2 : 1) * 8, 32); }

}  // namespace apnn

using namespace apnn;

extern "C" size_t apnn_input_weight_bytes(int64_t Cout, int64_t Cin, int R, int S)
{
    if (Cout < 0 || Cin < 1 || R < 1 || S < 1 || S > 16) return 0;
    return static_cast<size_t>(round_up(Cout * input_row_bytes(Cin, R, S), 16) + 4 * Cout);
}

extern "C" int apnn_pack_input_weights(const void *src_dev, int64_t Cout, int64_t Cin, int R, int S, int bits,
                                       apnn_encoding enc, void *dst_dev, void *stream)
{
    clear_error();
    const char *who = "apnn_pack_input_weights";
    if (int rc = check_bits_enc(who, "weight", bits, enc)) return rc;
    if (Cout < 0 || Cin < 1 || R < 1 || S < 1) return fail(APNN_ERR_INVALID_ARG, "%s: bad size", who);
    if (S > 16) return fail(APNN_ERR_UNSUPPORTED, "%s: S = %d, supported up to 16 (two 8-byte K segments per kernel row)", who, S);
    if (bits > 7) return fail(APNN_ERR_UNSUPPORTED, "%s: %d-bit weights do not fit a signed byte", who, bits);
    const int64_t Kp = input_row_bytes(Cin, R, S);
    if (Cout * Kp > 0x7FFFFFFF) return fail(APNN_ERR_INVALID_ARG, "%s: tensor too large", who);
    if (Cout == 0) return APNN_OK;
    if (!src_dev || !dst_dev) return fail(APNN_ERR_INVALID_ARG, "%s: null pointer", who);
    if (!aligned16(dst_dev)) return fail(APNN_ERR_ALIGNMENT, "%s: dst_dev not 16-byte aligned", who);
    int8_t *w = static_cast<int8_t *>(dst_dev);
    int32_t *cterm = reinterpret_cast<int32_t *>(w + round_up(Cout * Kp, 16));
    hipLaunchKernelGGL(input_weights_kernel, dim3(static_cast<unsigned>(ceil_div(Cout * Kp, 256))), dim3(256), 0,
                       as_stream(stream), static_cast<const uint8_t *>(src_dev), w, static_cast<int>(Cout),
                       static_cast<int>(Cin), R, S, static_cast<int>(Kp), bits, enc == APNN_ENC_PM1 ? 1 : 0);
    if (int rc = check_launch(who)) return rc;
    hipLaunchKernelGGL(input_cterm_kernel, dim3(static_cast<unsigned>(ceil_div(Cout, 256))), dim3(256), 0, as_stream(stream),
                       w, cterm, static_cast<int>(Cout), static_cast<int>(Kp));
    return check_launch(who);
}

extern "C" int apnn_input_layer(const apnn_layer_desc *desc, const void *W_dev, const uint8_t *image_dev,
                                uint32_t *out_packed_dev, void *stream)
{
    clear_error();
    const char *who = "apnn_input_layer";
    if (!desc) return fail(APNN_ERR_INVALID_ARG, "%s: desc is null", who);
    const apnn_layer_desc &L = *desc;
    const apnn_conv_desc &d = L.conv;
    if (int rc = check_bits_enc(who, "weight", d.p, d.encW)) return rc;
    if (int rc = check_bits_enc(who, "activation", d.q, d.encX)) return rc;
    if (d.encX != APNN_ENC_UNSIGNED) return fail(APNN_ERR_INVALID_ARG, "%s: the image holds unsigned codes", who);
    if (L.is_gemm) return fail(APNN_ERR_INVALID_ARG, "%s: is_gemm does not apply", who);
    if (L.pool != APNN_POOL_NONE) return fail(APNN_ERR_UNSUPPORTED, "%s: no fused pooling in the input layer", who);
    if (d.N < 0 || d.Cin < 1 || d.Cout < 0) return fail(APNN_ERR_INVALID_ARG, "%s: bad size", who);
    if (d.H < 1 || d.W < 1 || d.R < 1 || d.S < 1 || d.stride < 1 || d.pad < 0)
        return fail(APNN_ERR_INVALID_ARG, "%s: bad convolution geometry", who);
    if (d.H + 2 * d.pad < d.R || d.W + 2 * d.pad < d.S)
        return fail(APNN_ERR_INVALID_ARG, "%s: kernel larger than the padded frame", who);
    if (d.S > 16 || d.W < 8) return fail(APNN_ERR_UNSUPPORTED, "%s: needs S <= 16 and W >= 8 (8-byte K segments)", who);
    if (d.p > 7) return fail(APNN_ERR_UNSUPPORTED, "%s: %d-bit weights do not fit a signed byte", who, d.p);
    if (d.Cout > 128) return fail(APNN_ERR_UNSUPPORTED, "%s: Cout = %lld, supported up to 128", who, (long long)d.Cout);
    if (L.q_out < 0 || L.q_out > 8) return fail(APNN_ERR_UNSUPPORTED, "%s: q_out = %d, supported 0..8", who, L.q_out);
    const bool want_float = L.q_out > 0 || L.float_out_dev != nullptr;
    if (want_float && (!L.scale_dev || !L.bias_dev)) return fail(APNN_ERR_INVALID_ARG, "%s: scale_dev/bias_dev required", who);
    if (L.q_out > 0 && !out_packed_dev) return fail(APNN_ERR_INVALID_ARG, "%s: out_packed_dev is null but q_out > 0", who);
    if (L.q_out > 0 && d.Cout % 32 != 0)
        return fail(APNN_ERR_INVALID_ARG, "%s: Cout = %lld must be a multiple of 32 for packed output", who, (long long)d.Cout);
    if (L.q_out == 0 && !L.acc_out_dev && !L.float_out_dev) return fail(APNN_ERR_INVALID_ARG, "%s: no output requested", who);
    if (L.residual_dev) {
        if (!want_float) return fail(APNN_ERR_INVALID_ARG, "%s: residual needs the scale/bias epilogue", who);
        if (L.q_res < 1 || L.q_res > 8) return fail(APNN_ERR_UNSUPPORTED, "%s: q_res = %d, supported 1..8", who, L.q_res);
        if (d.Cout % 32 != 0) return fail(APNN_ERR_INVALID_ARG, "%s: residual needs Cout multiple of 32", who);
    }
    // every sum of products (and the sum of the shifted ones) must be an exact fp32 integer for the epilogue
    const int64_t K = d.Cin * d.R * d.S, wmax = d.encW == APNN_ENC_PM1 ? 1 : (int64_t(1) << d.p) - 1;
    if (K * 255 * wmax >= (int64_t(1) << 24))
        return fail(APNN_ERR_UNSUPPORTED, "%s: K = %lld with %d-bit weights exceeds the exact range 2^24", who, (long long)K, d.p);
    const int64_t Ho = (d.H + 2 * d.pad - d.R) / d.stride + 1, Wo = (d.W + 2 * d.pad - d.S) / d.stride + 1;
    const int64_t M = d.N * Ho * Wo, N = d.Cout;
    if (M + 128 > 0x7FFFFFFF || d.N * d.Cin * d.H * d.W > 0x7FFFFFFF)
        return fail(APNN_ERR_INVALID_ARG, "%s: dimension exceeds 2^31", who);
    if (M == 0 || N == 0) return APNN_OK;
    if (!W_dev || !image_dev) return fail(APNN_ERR_INVALID_ARG, "%s: null operand", who);
    if (!aligned16(W_dev)) return fail(APNN_ERR_ALIGNMENT, "%s: W_dev not 16-byte aligned", who);
    if ((out_packed_dev && !aligned16(out_packed_dev)) || (L.acc_out_dev && !aligned16(L.acc_out_dev)))
        return fail(APNN_ERR_ALIGNMENT, "%s: outputs must be 16-byte aligned", who);

    MfmaParams p{};
    p.M = static_cast<int>(M); p.N = static_cast<int>(N);
    p.out_scale = 1.0f; p.c0 = 0;
    p.H = static_cast<int>(d.H); p.W = static_cast<int>(d.W); p.R = d.R; p.S = d.S;
    p.stride = d.stride; p.pad = d.pad; p.Ho = static_cast<int>(Ho); p.Wo = static_cast<int>(Wo);
    p.invWo = 1.0f / static_cast<float>(Wo);
    p.invHoWo = 1.0f / (static_cast<float>(Ho) * static_cast<float>(Wo));
    p.fastdiv = (M + 128 < (int64_t(1) << 21)) ? 1 : 0;
    p.Y = L.acc_out_dev;
    if (want_float) {
        p.scale = L.scale_dev; p.bias = L.bias_dev; p.T = L.float_out_dev;
        p.res = L.residual_dev; p.q_res = L.q_res; p.res_scale = L.res_scale;
        p.out = L.q_out > 0 ? out_packed_dev : nullptr; p.q_out = L.q_out;
    }
    p.NW = static_cast<int>(N / 32);
    InputParams q{};
    q.img = image_dev;
    q.C = static_cast<int>(d.Cin);
    q.Kp = static_cast<int>(input_row_bytes(d.Cin, d.R, d.S));
    q.KS = q.Kp / 32;
    q.nseg = static_cast<int>(d.Cin) * d.R * (d.S > 8 ? 2 : 1);
    q.invR = 1.0f / static_cast<float>(d.R);
    q.xmask = 0x01010101u * ((1u << d.q) - 1u);
    q.w = static_cast<const int8_t *>(W_dev);
    q.cterm = reinterpret_cast<const int32_t *>(q.w + round_up(N * q.Kp, 16));
    const unsigned grid = static_cast<unsigned>(ceil_div(M, 128));
    const int nt = static_cast<int>(ceil_div(N, 32));
    const bool two = d.S > 8;                           // two 8-byte segments per kernel row
    if (nt == 1) hipLaunchKernelGGL((two ? input_conv_kernel<1, 2> : input_conv_kernel<1, 1>), dim3(grid), dim3(256), 0, as_stream(stream), p, q);
    else if (nt == 2) hipLaunchKernelGGL((two ? input_conv_kernel<2, 2> : input_conv_kernel<2, 1>), dim3(grid), dim3(256), 0, as_stream(stream), p, q);
    else if (nt == 3) hipLaunchKernelGGL((two ? input_conv_kernel<3, 2> : input_conv_kernel<3, 1>), dim3(grid), dim3(256), 0, as_stream(stream), p, q);
    else hipLaunchKernelGGL((two ? input_conv_kernel<4, 2> : input_conv_kernel<4, 1>), dim3(grid), dim3(256), 0, as_stream(stream), p, q);
    return check_launch(who);
}
