// Matrix-core variant of the arbitrary-precision product: one template serves
// apnn_gemm, apnn_conv2d and apnn_layer whenever the result is exactly
// representable in fp32 (K * max|a| * max|b| < 2^24, checked by the host, which
// otherwise uses the AND+popcount kernel).
//
// CDNA4 has no 1-bit matrix instruction, but its FP4 (E2M1) matrix instruction
// represents exactly what one or two bit planes of an operand can encode:
// {0,1,2,3} (as the halves 0, 0.5, 1, 1.5, whose codes are the two plane bits
// themselves) and {-1,+1}.  The operands stay in the packed bit-plane layouts of
// the ABI in HBM and in LDS (Sec. 4.2 (a) data organisation, Sec. 4.1 (a)
// shared-memory caching).  An operand of more than two bits is cut into base-4
// digits of two adjacent planes (a last single plane counts as a digit with a
// zero upper plane); every digit pair (da, db) is one pass over K, and the passes
// are combined as in Eq. 1 with weights 4^(da+db), evaluated by Horner's rule
// directly in the accumulators (acc *= 4 whenever the digit diagonal da + db
// drops by one).  This is the AP-Bit template of Sec. 3.1 with a 2-bit instead of
// a 1-bit primitive.  Per lane and in registers, the planes of 32 consecutive K
// positions are re-composed into 32 FP4 codes (Eq. 2 read backwards) and one
// v_mfma_scale_f32_32x32x64_f8f6f4 performs 32 x 32 x 64 multiply-adds.  All
// products and partial sums are small integers, hence exact in fp32.  Because
// -1/+1 is encoded directly, Cases II and III of Sec. 3.2 need no XOR and no
// J-term here; the only correction is for K pad positions when both operands are
// -1/+1 (0 pad bits read as (-1)(-1) = +1).
//
// Geometry: NWM x NWN waves share a (NWM*FM*32) x (NWN*FN*32) block tile, each
// wave owning FM x FN matrix-instruction tiles of 32 x 32 (16 fp32 accumulators
// per lane each).  For small layers a block instead owns a single wave tile and
// its NSPLIT waves split the K steps of every chunk between them (partial tiles
// are added through LDS), which shortens the serial instruction stream per wave.  A K chunk is KC words (8 or 32) = KC/2 instruction steps; the summation order over K is free, so lane-half h of a step takes word
// (h*KC/2 + step) of the chunk, which lets every lane fetch its steps of one
// (row, plane) with 16-byte LDS reads.  Small problems use the longer chunk so
// that the exposed memory latency per chunk is paid fewer times.  Global loads of the next chunk
// fly while the current one is computed (LDS double buffer, one barrier per
// chunk).  In convolution mode the A rows are output pixels and the K index runs
// over (kernel row, kernel column, channel word) with zero words for taps outside
// the frame (Sec. 4.2 (b)).
//
// Epilogue (Sec. 4.1 (b), Sec. 5.2): accumulator register r of lane (half lh,
// column lr) of a 32 x 32 tile is row 8*(r/4) + 4*lh + r%4, column lr.  Lanes are
// output channels, so the requantised codes of 32 channels are packed with one
// wave ballot per plane: the low half of the ballot is the word of row(lh=0), the
// high half that of row(lh=1).
#pragma once
#include "lane_util.h"
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "vec_util.h"

namespace apnn {

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));

// digit kinds: one 0/1 plane, two 0/1 planes, one -1/+1 plane, and (convolution features only) one -1/+1
// plane accompanied by a validity word that the loader makes up: all ones for a tap inside the frame, zero
// outside, so that taps outside the frame contribute 0 instead of -1 (zero-contribution padding of Sec. 4.2 (b)
// for Case II and the mirrored Case III)
enum { OPK_U1 = 0, OPK_U2 = 1, OPK_PM1 = 2, OPK_PM1Z = 3 };

struct MfmaParams {
    const uint32_t *A, *B;   // row / column operand planes
    int M, N;
    int PA, PB;              // planes in memory
    int DA, DB;              // base-4 digits (ceil(planes / 2); 1 for single-plane kinds)
    int ldwA, ldwB;          // words per plane row (A: matrix mode only)
    int Kw;                  // words per plane along K
    int nk;                  // K chunks of KC words
    int c0;                  // additive correction (pad positions of a -1/+1 x -1/+1 product)
    float out_scale;         // 2^(number of two-plane operands): those enter the matrix unit as value / 2
    // convolution geometry of the A operand (conv mode only)
    int H, W, Cw, R, S, stride, pad, Ho, Wo;
    float invCw;
    // Fused 2 x 2 grid pooling (Sec. 5.2; convolution mode only): 0 none, 1 maximum, 2 sum.  Rows are then
    // enumerated as 4 * (pooled pixel over N x Hp x Wp) + 2 dy + dx, so the four results of a grid are four
    // consecutive accumulator registers of one lane; M counts these rows, the outputs have M / 4 rows.
    int pool, Hp, Wp;
    // Reciprocals for the index arithmetic of the convolution loader: floor(n / d) = int((n + 0.5f) * (1 / d)) is
    // exact for n < 2^21, which the host checks (fastdiv); larger problems divide integers.
    float invS, invWo, invHoWo, invWp, invHpWp;
    int fastdiv;
    int xcd_regions;         // pipelined large-tile kernel: tile grid walked as 2 x 4 regions, one per XCD (host: grid divides)
    // outputs, as in the AND+popcount kernel
    int32_t *Y;
    float *T;
    const float *scale, *bias;
    const uint32_t *res;
    int q_res;
    float res_scale;
    uint32_t *out;
    int q_out;
    int NW;
    // 8-bit integer matrix form only (mfma_i8_kernel): Y = accmul acc + mulA RA[row] + mulB RB[column] + c0, RA / RB
    // the decoded row sums of the operands; flipA / flipB invert the top plane of an 8-plane operand (value - 128)
    uint32_t flipA, flipB;
    int accmul, mulA, mulB;
};

// A 32-bit constant the optimiser cannot fold: it then lives in a register, so
// that (x & mask) | other compiles to one three-operand instruction instead of
// two instructions with one literal each.
__device__ __forceinline__ uint32_t reg_const(uint32_t k)
{
    asm volatile("" : "+v"(k));
    return k;
}

struct Fp4Masks { uint32_t m1, m2, m4, m8; };

// 32 K positions of one operand row -> 4 dwords of 8 FP4 codes; nibble i of
// dword r holds the element at bit (r + 4 i) of the plane words x0 (x1).
template <int KIND> __device__ __forceinline__ void expand_fp4(uint32_t x0, uint32_t x1, const Fp4Masks &k, v8i_t &out)
{
    if (KIND == OPK_U1) {                       // 0 -> 0000 (0.0), 1 -> 0010 (1.0)
        out[0] = (x0 << 1) & k.m2;
        out[1] = x0 & k.m2;
        out[2] = (x0 >> 1) & k.m2;
        out[3] = (x0 >> 2) & k.m2;
    } else if (KIND == OPK_PM1) {               // 1 -> 0010 (+1.0), 0 -> 1010 (-1.0)
        out[0] = (~(x0 << 3) & k.m8) | k.m2;
        out[1] = (~(x0 << 2) & k.m8) | k.m2;
        out[2] = (~(x0 << 1) & k.m8) | k.m2;
        out[3] = (~x0 & k.m8) | k.m2;
    } else if (KIND == OPK_PM1Z) {              // as PM1 where x1 (all ones or zero) says the tap exists, else 0000 (0.0)
        out[0] = ((~(x0 << 3) & k.m8) | k.m2) & x1;
        out[1] = ((~(x0 << 2) & k.m8) | k.m2) & x1;
        out[2] = ((~(x0 << 1) & k.m8) | k.m2) & x1;
        out[3] = ((~x0 & k.m8) | k.m2) & x1;
    } else {                                    // v = 2 x1 + x0 -> code x1 x0 = v / 2 (0, 0.5, 1, 1.5):
        // the two planes ARE the FP4 code of half the value, so no recoding is needed;
        // the host-set out_scale (2 per two-plane operand) restores the factor exactly
        out[0] = ((x1 << 1) & k.m2) | (x0 & k.m1);
        out[1] = (x1 & k.m2) | ((x0 >> 1) & k.m1);
        out[2] = ((x1 >> 1) & k.m2) | ((x0 >> 2) & k.m1);
        out[3] = ((x1 >> 2) & k.m2) | ((x0 >> 3) & k.m1);
    }
    out[4] = out[5] = out[6] = out[7] = 0;
}

// Epilogue on one output value: optional int32 store, fused scale/bias, residual,
// floor/clamp and the ballot-packed planes.  Every lane of the wave must call it
// (gm differs only between the two lane halves, gn = tile column base + lr).
__device__ __forceinline__ void finish_value(const MfmaParams &p, float v, int gm, int gn, float sc, float bi,
                                             bool have_res, uint32_t res_code, int lr, int lh)
{
    const bool rok = gm < p.M, cok = gn < p.N;
    const int wcol = gn >> 5;                   // word column of this lane's channel (the 32-wide tile shares it)
    const int y = static_cast<int>(v * p.out_scale) + p.c0;      // exact: v is a multiple of 1 / out_scale
    if (p.Y && rok && cok) p.Y[static_cast<int64_t>(gm) * p.N + gn] = y;
    if (p.scale) {
        float t = __fmaf_rn(sc, static_cast<float>(y), bi);
        if (p.res) {
            uint32_t code = res_code;
            if (!have_res && rok && cok) {
                const uint32_t *rp = p.res + static_cast<int64_t>(gm) * p.q_res * p.NW + wcol;
                for (int b = 0; b < p.q_res; ++b) code |= ((rp[b * p.NW] >> lr) & 1u) << b;
            }
            t = __fmaf_rn(p.res_scale, static_cast<float>(code), t);
        }
        if (p.T && rok && cok) p.T[static_cast<int64_t>(gm) * p.N + gn] = t;
        if (p.out) {
            const float qmax = static_cast<float>((1 << p.q_out) - 1);
            float f = floorf(t);
            f = (f >= 0.0f) ? f : 0.0f;
            f = (f > qmax) ? qmax : f;
            const uint32_t code = cok ? static_cast<uint32_t>(f) : 0u;
            uint32_t *op = p.out + static_cast<int64_t>(gm) * p.q_out * p.NW + wcol;
            for (int b = 0; b < p.q_out; ++b) {
                const unsigned long long bal = __ballot((code >> b) & 1u);
                const uint32_t word = lh ? static_cast<uint32_t>(bal >> 32) : static_cast<uint32_t>(bal);
                if (lr == 0 && rok && cok) op[b * p.NW] = word;
            }
        }
    }
}

// Residual words of the eight output rows row0 .. row0 + 7 of word column wcol: lane l of the wave returns the
// word of row row0 + (l & 7), plane l >> 3 (zero where there is none).  One load per wave.
__device__ __forceinline__ uint32_t load_res_rows8(const MfmaParams &p, int row0, int wcol, int lane)
{
    const int b = lane >> 3, row = row0 + (lane & 7);
    uint32_t w = 0;
    if (p.res && b < p.q_res && row < p.M && wcol < p.NW)
        w = p.res[(static_cast<int64_t>(row) * p.q_res + b) * p.NW + wcol];
    return w;
}

// finish_value for the four accumulator registers 4 k .. 4 k + 3 of a 32 x 32 tile at once: lane (lr, lh) holds
// v[i] for output row row0 + 4 lh + i and channel gn (row0 = tile row base + 8 k; gn = tile column base + lr).
// Same arithmetic and outputs as finish_value, written for few vector instructions per value, which is what
// bounds a layer that runs a few waves per SIMD: row validity is needed only where something is stored, the
// residual words arrive by one load per wave (res_words from load_res_rows8, fetched early) and are handed out
// by lane permutes, and the 8 x q_out plane words are collected by lane writes into one register (lane
// 8 b + row) and leave in one store.  Every lane of the wave must call it.
__device__ __forceinline__ void finish_rows8(const MfmaParams &p, const float (&v)[4], int row0, int gn, float sc, float bi,
                                             uint32_t res_words, int lane, int lr, int lh)
{
    const int rows_left = p.M - row0 - 4 * lh;          // v[i] is a real row iff i < rows_left
    const bool cok = gn < p.N;
    const int64_t first = static_cast<int64_t>(row0 + 4 * lh) * p.N + gn;
    const float c0 = static_cast<float>(p.c0);
    float y[4];                                         // exact integers below 2^24, as the int32 results are
#pragma unroll
    for (int i = 0; i < 4; ++i) y[i] = v[i] * p.out_scale + c0;
    if (p.Y) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (cok && i < rows_left) p.Y[first + static_cast<int64_t>(i) * p.N] = static_cast<int>(y[i]);
    }
    if (!p.scale) return;
    float t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = __fmaf_rn(sc, y[i], bi);
    if (p.res) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t code = 0;
            for (int b = 0; b < p.q_res; ++b) {
                const uint32_t w = static_cast<uint32_t>(
                    __builtin_amdgcn_ds_bpermute(4 * (8 * b + 4 * lh + i), static_cast<int>(res_words)));
                code |= ((w >> lr) & 1u) << b;
            }
            t[i] = __fmaf_rn(p.res_scale, static_cast<float>(code), t[i]);
        }
    }
    if (p.T) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (cok && i < rows_left) p.T[first + static_cast<int64_t>(i) * p.N] = t[i];
    }
    if (!p.out) return;
    // (N is a multiple of 32 whenever planes are written: a 32-column tile has all its channels or none)
    int word = 0;
    if (p.q_out <= 2) {
        // One or two planes: floor(t) >= k is t >= k for an integer k, so the planes of clamp(floor(t), 0, 3) are
        // compares of t itself (NaN compares false everywhere: code 0, as the clamp gives): bit 1 = t >= 2,
        // bit 0 = (1 <= t < 2) or t >= 3; with one plane, bit 0 = t >= 1.  No floor, clamp or conversion: a third
        // fewer vector instructions, which is what a large layer's duration consists of.
        static_for<4>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const unsigned long long c1 = __ballot(t[i] >= 1.0f);
            if (p.q_out == 1) {
                write_lanes<i, i + 4>(word, c1);
            } else {
                const unsigned long long c2 = __ballot(t[i] >= 2.0f), c3 = __ballot(t[i] >= 3.0f);
                write_lanes<i, i + 4>(word, (c1 & ~c2) | c3);
                write_lanes<8 + i, 8 + i + 4>(word, c2);
            }
        });
    } else {
        const float qmax = static_cast<float>((1 << p.q_out) - 1);
        uint32_t code[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float f = floorf(t[i]);
            f = (f >= 0.0f) ? f : 0.0f;
            f = (f > qmax) ? qmax : f;
            code[i] = static_cast<uint32_t>(f);
        }
        static_for<8>([&](auto bc) {
            constexpr int b = decltype(bc)::value;
            if (b < p.q_out) {
                static_for<4>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    write_lanes<8 * b + i, 8 * b + i + 4>(word, __ballot(code[i] & (1u << b)));
                });
            }
        });
    }
    const int b = lane >> 3, row = row0 + (lane & 7);
    const int wcol = gn >> 5;                           // (a block tile can reach beyond N: whole 32-column tiles then)
    if (b < p.q_out && row < p.M && wcol < p.NW)
        p.out[(static_cast<int64_t>(row) * p.q_out + b) * p.NW + wcol] = static_cast<uint32_t>(word);
}

__device__ __forceinline__ int div_by_reciprocal(int n, float inv)
{
    return static_cast<int>((static_cast<float>(n) + 0.5f) * inv);
}

// Row index of the convolution's implicit GEMM -> (image, output row, output column).
__device__ __forceinline__ void conv_row_to_pixel(const MfmaParams &p, int gm, int &n, int &ho, int &wo)
{
    const int P = p.pool ? gm >> 2 : gm;                // (pooled) pixel in raster order over N x Hq x Wq
    const int Wq = p.pool ? p.Wp : p.Wo, Hq = p.pool ? p.Hp : p.Ho;
    int row, col;                                       // P = (n * Hq + row) * Wq + col
    if (p.fastdiv) {
        const int q = div_by_reciprocal(P, p.pool ? p.invWp : p.invWo);
        col = P - q * Wq;
        n = div_by_reciprocal(P, p.pool ? p.invHpWp : p.invHoWo);
        row = q - n * Hq;
    } else {
        col = P % Wq;
        row = (P / Wq) % Hq;
        n = P / (Wq * Hq);
    }
    if (p.pool) {
        ho = 2 * row + ((gm >> 1) & 1);
        wo = 2 * col + (gm & 1);
    } else {
        ho = row;
        wo = col;
    }
}

// Tap index -> (kernel row, kernel column).
__device__ __forceinline__ void tap_to_rs(const MfmaParams &p, int tap, int &r, int &sc)
{
    r = div_by_reciprocal(tap, p.invS);                 // tap < R S, far below the exactness limit
    sc = tap - r * p.S;
}

// The four results of a pooling grid (exact integers in fp32): maximum or sum.
__device__ __forceinline__ float pool4(int mode, float a, float b, float c, float d)
{
    return mode == 1 ? fmaxf(fmaxf(a, b), fmaxf(c, d)) : (a + b) + (c + d);
}

template <int KIND> struct DigitPlanes { static constexpr int value = (KIND == OPK_U2 || KIND == OPK_PM1Z) ? 2 : 1; };

template <int KA, int KB, int NWM, int NWN, int NSPLIT, int FM, int FN, int KC, int VW, bool CONV>
__global__ __launch_bounds__(64 * NWM * NWN * NSPLIT, (NWM * NWN * FM * FN >= 64 && FM * FN >= 16) ? 1 : 2)
void mfma_fp4_kernel(const MfmaParams p)
{
    static_assert(NSPLIT == 1 || (NWM == 1 && NWN == 1), "K is split across the waves of a single-tile block only");
    constexpr int NT = 64 * NWM * NWN * NSPLIT;         // threads
    constexpr int NS = KC / 2;                          // matrix-instruction steps per chunk
    constexpr int NSW = NS / NSPLIT;                    // ... of which each wave of a K-split block takes NSW
    static_assert(NSW % 4 == 0, "a wave reads its steps with 16-byte LDS loads");
    constexpr int LA = DigitPlanes<KA>::value, LB = DigitPlanes<KB>::value;   // planes of one digit
    constexpr int BM = NWM * FM * 32, BN = NWN * FN * 32;
    constexpr int RSA = LA * KC + 4, RSB = LB * KC + 4; // padded LDS row strides (words)
    constexpr int CH = KC / VW;                         // loader vectors per (row, plane) and chunk
    constexpr int A_VECS = BM * LA * CH, B_VECS = BN * LB * (KC / 4);
    constexpr int A_SLOTS = (A_VECS + NT - 1) / NT, B_SLOTS = (B_VECS + NT - 1) / NT;
    using VecA = typename VecT<VW>::type;

    // one LDS arena: the double-buffered operand tiles; in a K-split block the
    // reduction buffer reuses it once the main loop is over
    constexpr int TILE_WORDS = 2 * BM * RSA + 2 * BN * RSB;
    constexpr int RED_WORDS = NSPLIT > 1 ? NSPLIT * FM * FN * 16 * 64 : 0;
    __shared__ __attribute__((aligned(16))) uint32_t smem[TILE_WORDS > RED_WORDS ? TILE_WORDS : RED_WORDS];
    uint32_t (*sA)[BM * RSA] = reinterpret_cast<uint32_t (*)[BM * RSA]>(smem);
    uint32_t (*sB)[BN * RSB] = reinterpret_cast<uint32_t (*)[BN * RSB]>(smem + 2 * BM * RSA);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ks = wave / (NWM * NWN);                  // K-split index of this wave
    const int wm = (wave % (NWM * NWN)) / NWN, wn = wave % NWN;   // wave position in the NWM x NWN arrangement
    const int lr = lane & 31, lh = lane >> 5;           // row / column inside a 32-wide tile, K half

    const int tilesN = (p.N + BN - 1) / BN;
    const int m0 = (blockIdx.x / tilesN) * BM, n0 = (blockIdx.x % tilesN) * BN;

    Fp4Masks km;
    km.m1 = reg_const(0x11111111u); km.m2 = reg_const(0x22222222u);
    km.m4 = reg_const(0x44444444u); km.m8 = reg_const(0x88888888u);

    // ---- loader.  A vector v = tid + NT u covers (row, plane of the digit, piece c):
    // v = (row * LA + pl) * CH + c; B likewise with 16-byte pieces.
    int a_h0[A_SLOTS], a_w0[A_SLOTS], a_pix[A_SLOTS];
    if (CONV) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            const int gm = m0 + (tid + NT * u) / (LA * CH);
            int wo, ho, n;
            conv_row_to_pixel(p, gm, n, ho, wo);
            a_h0[u] = ho * p.stride - p.pad;
            a_w0[u] = wo * p.stride - p.pad;
            a_pix[u] = n * p.H * p.W;
        }
    }
    VecA ra[A_SLOTS];
    uint4 rb[B_SLOTS];
    auto fetch = [&](int da, int db, int kc) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            const int v = tid + NT * u, c = v % CH, rp = v / CH;
            const bool validity = KA == OPK_PM1Z && rp % LA == 1;                  // made up, not loaded
            const int row = rp / LA, plane = validity ? 0 : 2 * da * (LA - 1) + da * (2 - LA) + rp % LA;   // LA = 2: 2 da + pl; LA = 1: da
            const int gm = m0 + row, kk = kc * KC + c * VW;
            ra[u] = vec_zero<VW>();
            if (v < A_VECS && gm < p.M && kk < p.Kw && plane < p.PA) {
                if (CONV) {
                    const int tap = static_cast<int>((static_cast<float>(kk) + 0.5f) * p.invCw);
                    const int cw = kk - tap * p.Cw;
                    int r, sc;
                    tap_to_rs(p, tap, r, sc);
                    const int h = a_h0[u] + r, w = a_w0[u] + sc;
                    if (h >= 0 && h < p.H && w >= 0 && w < p.W) {
                        const int64_t pix = a_pix[u] + h * p.W + w;
                        if (validity) ra[u] = vec_ones<VW>();
                        else ra[u] = *reinterpret_cast<const VecA *>(p.A + (pix * p.PA + plane) * p.Cw + cw);
                    }
                } else {
                    ra[u] = *reinterpret_cast<const VecA *>(p.A + (static_cast<int64_t>(gm) * p.PA + plane) * p.ldwA + kk);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) {
            const int v = tid + NT * u, c = v % (KC / 4), rp = v / (KC / 4);
            const int row = rp / LB, plane = 2 * db * (LB - 1) + db * (2 - LB) + rp % LB;
            const int gn = n0 + row, kk = kc * KC + 4 * c;
            rb[u] = make_uint4(0, 0, 0, 0);
            if (v < B_VECS && gn < p.N && kk < p.Kw && plane < p.PB) {
                const uint32_t *src = p.B + (static_cast<int64_t>(gn) * p.PB + plane) * p.ldwB + kk;
                if (!CONV) {
                    rb[u] = *reinterpret_cast<const uint4 *>(src);
                } else {                        // conv weight rows are 8-byte aligned and an even number of words long
                    const uint2 lo = *reinterpret_cast<const uint2 *>(src);
                    uint2 hi = make_uint2(0, 0);
                    if (kk + 4 <= p.Kw) hi = *reinterpret_cast<const uint2 *>(src + 2);
                    rb[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                }
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            const int v = tid + NT * u, c = v % CH, rp = v / CH;
            if (v < A_VECS) *reinterpret_cast<VecA *>(&sA[buf][(rp / LA) * RSA + (rp % LA) * KC + c * VW]) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) {
            const int v = tid + NT * u, c = v % (KC / 4), rp = v / (KC / 4);
            if (v < B_VECS) *reinterpret_cast<uint4 *>(&sB[buf][(rp / LB) * RSB + (rp % LB) * KC + 4 * c]) = rb[u];
        }
    };

    v16f_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // digit pairs diagonal by diagonal (da + db descending), as the plane pairs of
    // the AND+popcount kernel, so that Eq. 1 becomes a Horner evaluation in base 4
    const int dmax = p.DA + p.DB - 2;
    auto first_a = [&](int d) { return max(0, d - (p.DB - 1)); };
    auto next_pair = [&](int &a_, int &b_) {
        if (a_ + 1 < p.DA && b_ - 1 >= 0) { ++a_; --b_; return false; }
        const int d = a_ + b_ - 1;
        if (d < 0) return false;
        a_ = first_a(d); b_ = d - a_;
        return true;
    };
    const int total_it = p.DA * p.DB * p.nk;
    int fa_ = first_a(dmax), fb_ = dmax - fa_, fk = 0;  // pair / chunk being fetched
    int ca = fa_, cb = fb_, ck = 0;                     // pair / chunk being computed

    // K-split blocks are latency bound: fetch the epilogue's per-channel parameters
    // and residual codes now, so that their latency hides behind the main loop
    constexpr int RPW = 16 / NSPLIT;
    float pre_sc[FN], pre_bi[FN];
    uint32_t pre_res[NSPLIT > 1 ? FM * FN : 1];       // per 32 x 32 tile: the words of the wave's eight rows (load_res_rows8)
    if constexpr (NSPLIT > 1) {
        static_assert(RPW == 4, "a K-split wave finishes one group of eight rows per 32 x 32 tile");
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int gn = n0 + j * 32 + lr;
            pre_sc[j] = pre_bi[j] = 0.0f;
            if (p.scale && gn < p.N) { pre_sc[j] = p.scale[gn]; pre_bi[j] = p.bias[gn]; }
#pragma unroll
            for (int i = 0; i < FM; ++i)
                pre_res[i * FN + j] = p.pool ? 0u : load_res_rows8(p, m0 + i * 32 + 8 * ks, (n0 + j * 32) >> 5, lane);
        }
    }

    if (total_it > 0) {
        fetch(fa_, fb_, 0);
        if (++fk == p.nk) { fk = 0; next_pair(fa_, fb_); }
        stage(0);
    }
    __syncthreads();

    for (int it = 0; it < total_it; ++it) {
        const int buf = it & 1;
        if (it + 1 < total_it) {
            fetch(fa_, fb_, fk);
            if (++fk == p.nk) { fk = 0; next_pair(fa_, fb_); }
        }

        // this lane's words of the chunk: NS steps x planes of the digit, for its tile rows
        uint32_t wa[FM][LA][NSW], wb[FN][LB][NSW];
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int pl = 0; pl < LA; ++pl)
#pragma unroll
                for (int g = 0; g < NSW / 4; ++g) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(
                        &sA[buf][(wm * FM * 32 + f * 32 + lr) * RSA + pl * KC + NS * lh + NSW * ks + 4 * g]);
                    wa[f][pl][4 * g] = v.x; wa[f][pl][4 * g + 1] = v.y; wa[f][pl][4 * g + 2] = v.z; wa[f][pl][4 * g + 3] = v.w;
                }
#pragma unroll
        for (int f = 0; f < FN; ++f)
#pragma unroll
            for (int pl = 0; pl < LB; ++pl)
#pragma unroll
                for (int g = 0; g < NSW / 4; ++g) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(
                        &sB[buf][(wn * FN * 32 + f * 32 + lr) * RSB + pl * KC + NS * lh + NSW * ks + 4 * g]);
                    wb[f][pl][4 * g] = v.x; wb[f][pl][4 * g + 1] = v.y; wb[f][pl][4 * g + 2] = v.z; wb[f][pl][4 * g + 3] = v.w;
                }
#pragma unroll
        for (int st = 0; st < NSW; ++st) {
            v8i_t fa[FM], fb[FN];
#pragma unroll
            for (int f = 0; f < FM; ++f) expand_fp4<KA>(wa[f][0][st], wa[f][LA - 1][st], km, fa[f]);
#pragma unroll
            for (int f = 0; f < FN; ++f) expand_fp4<KB>(wb[f][0][st], wb[f][LB - 1][st], km, fb[f]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], acc[i][j], 4, 4, 0,
                                                                                 0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
        if (++ck == p.nk) {                     // digit pair finished
            ck = 0;
            if (next_pair(ca, cb)) {            // next diagonal: one Horner step in base 4
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[i][j][r] *= 4.0f;
            }
        }
        if (it + 1 < total_it) stage(buf ^ 1);
        __syncthreads();
    }

    if constexpr (NSPLIT == 1) {
        constexpr int SLAB_STRIDE = BN + 4;                     // words; the pad keeps the two lane halves on different banks
        constexpr bool SLAB_FITS = NWM * 32 * SLAB_STRIDE <= TILE_WORDS;
        if (SLAB_FITS && p.Y && !p.scale && (p.N & 3) == 0 && !p.pool) {
            // Plain int32 output: a lane's accumulators are 128-byte row fragments
            // scattered over 16 rows per tile.  They are transposed through LDS (one
            // slab of 32 rows per wave row at a time; the operand tiles are dead) so
            // that the stores leave as whole BN-column row segments, 16 bytes per lane.
            int32_t *slab = reinterpret_cast<int32_t *>(smem);
            static_for<FM>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                __syncthreads();                                // previous slab has been read
                static_for<FN * 16>([&](auto jrc) {
                    constexpr int j = decltype(jrc)::value / 16, r = decltype(jrc)::value % 16;
                    const int srow = wm * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    slab[srow * SLAB_STRIDE + wn * FN * 32 + j * 32 + lr] =
                        static_cast<int>(acc[i][j][r] * p.out_scale) + p.c0;
                });
                __syncthreads();
                for (int v = tid; v < NWM * 32 * (BN / 4); v += NT) {
                    const int srow = v / (BN / 4), c4 = (v % (BN / 4)) * 4;
                    const int gm = m0 + (srow >> 5) * FM * 32 + i * 32 + (srow & 31), gn = n0 + c4;
                    if (gm < p.M && gn < p.N)
                        *reinterpret_cast<int4 *>(p.Y + static_cast<int64_t>(gm) * p.N + gn) =
                            *reinterpret_cast<const int4 *>(&slab[srow * SLAB_STRIDE + c4]);
                }
            });
            return;
        }
        // compile-time indices keep the accumulators in registers
        MfmaParams pq = p;                              // pooled outputs: a quarter of the rows, corrections per grid
        pq.M = p.M >> 2;
        pq.c0 = p.pool == 2 ? 4 * p.c0 : p.c0;
        static_for<FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int gn = n0 + wn * FN * 32 + j * 32 + lr;
            float sc = 0.0f, bi = 0.0f;
            if (p.scale && gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
            if (p.pool) {
                static_for<FM * 4>([&](auto ikc) {
                    constexpr int i = decltype(ikc)::value / 4, k = decltype(ikc)::value % 4;
                    const float v = pool4(p.pool, acc[i][j][4 * k], acc[i][j][4 * k + 1], acc[i][j][4 * k + 2], acc[i][j][4 * k + 3]);
                    finish_value(pq, v, (m0 + wm * FM * 32 + i * 32 + 8 * k + 4 * lh) >> 2, gn, sc, bi, false, 0u, lr, lh);
                });
            } else {
                static_for<FM * 4>([&](auto ikc) {
                    constexpr int i = decltype(ikc)::value / 4, k = decltype(ikc)::value % 4;
                    const int row0 = m0 + wm * FM * 32 + i * 32 + 8 * k;
                    const float v4[4] = {acc[i][j][4 * k], acc[i][j][4 * k + 1], acc[i][j][4 * k + 2], acc[i][j][4 * k + 3]};
                    finish_rows8(p, v4, row0, gn, sc, bi, load_res_rows8(p, row0, gn >> 5, lane), lane, lr, lh);
                });
            }
        });
    } else {
        // K-split block: the waves' partial tiles are added through LDS; wave ks then
        // finishes accumulator registers 4 ks .. 4 ks + 3, i.e. rows 8 ks .. 8 ks + 7 of
        // every 32 x 32 tile, so the epilogue work is shared as well.
        float (*sRed)[FM * FN * 16][64] = reinterpret_cast<float (*)[FM * FN * 16][64]>(smem);   // tiles are dead: the main loop ended with a barrier
        static_for<FM * FN * 16>([&](auto c) {
            constexpr int f = decltype(c)::value / 16, r = decltype(c)::value % 16;
            sRed[ks][f * 16 + r][lane] = acc[f / FN][f % FN][r];
        });
        __syncthreads();
        static_for<FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int gn = n0 + j * 32 + lr;
            if (p.pool) {                               // RPW = 4: the wave's registers of a tile are one pooling grid
                static_assert(NSPLIT == 1 || RPW == 4, "a K-split wave finishes whole pooling grids");
                MfmaParams pq = p;
                pq.M = p.M >> 2;
                pq.c0 = p.pool == 2 ? 4 * p.c0 : p.c0;
                static_for<FM>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    float v4[4];
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        v4[rr] = 0.0f;
#pragma unroll
                        for (int k = 0; k < NSPLIT; ++k) v4[rr] += sRed[k][(i * FN + j) * 16 + ks * 4 + rr][lane];
                    }
                    finish_value(pq, pool4(p.pool, v4[0], v4[1], v4[2], v4[3]), (m0 + i * 32 + 8 * ks + 4 * lh) >> 2, gn,
                                 pre_sc[j], pre_bi[j], false, 0u, lr, lh);
                });
                return;
            }
            static_for<FM>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                float v4[4];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    v4[rr] = 0.0f;
#pragma unroll
                    for (int k = 0; k < NSPLIT; ++k) v4[rr] += sRed[k][(i * FN + j) * 16 + ks * 4 + rr][lane];
                }
                finish_rows8(p, v4, m0 + i * 32 + 8 * ks, gn, pre_sc[j], pre_bi[j], pre_res[i * FN + j], lane, lr, lh);
            });
        });
    }
}

}  // namespace apnn
