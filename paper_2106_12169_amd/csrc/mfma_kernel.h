// Matrix-core variant of the plane-pair product for operands of at most two
// bits (the paper's flagship w1a2 case and its neighbours).
//
// CDNA4 has no 1-bit matrix instruction, but its FP4 (E2M1) matrix instruction
// represents exactly the values a 1- or 2-bit operand can take: {0,1,2,3} and
// {-1,+1}.  The kernel keeps the packed bit-plane operands of the ABI in HBM and
// in LDS (Sec. 4.2 (a) data organisation, Sec. 4.1 (a) shared-memory caching) and
// re-composes, per lane and in registers, the planes of 32 consecutive K
// positions into 32 FP4 codes (Eq. 2 read backwards); one
// v_mfma_scale_f32_32x32x64_f8f6f4 then performs 32x32x64 multiply-adds.  All
// products and partial sums are small integers, exact in the fp32 accumulators as
// long as K * max|a| * max|b| < 2^24 (checked by the host, which otherwise uses
// the AND+popcount kernel).  Because -1/+1 is encoded directly, Cases II and III
// of Sec. 3.2 need no XOR and no J-term here; the only correction is for K pad
// positions when both operands are -1/+1 (0 pad bits read as (-1)(-1) = +1).
//
// Geometry: 256 threads = 4 waves (2 x 2), block tile 256 x 256, wave tile
// 128 x 128 = 4 x 4 matrix-instruction tiles (256 fp32 accumulators per lane).
// A K chunk is KC = 8 words = 256 K positions = 4 matrix-instruction steps; the
// summation order over K is free, so lane-half h of a step takes word
// (h*KC/2 + step) of the chunk, which lets every lane fetch its four steps of one
// (row, plane) with a single 16-byte LDS read.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace apnn {

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));

enum { OPK_U1 = 0, OPK_U2 = 1, OPK_PM1 = 2 };   // operand kinds

struct MfmaParams {
    const uint32_t *A, *B;   // row / column operand planes, matrix layout
    int M, N;
    int ldwA, ldwB;          // words per plane row
    int nk;                  // K chunks of 8 words
    int c0;                  // additive correction (pad positions of a -1/+1 x -1/+1 product)
    int32_t *Y;              // [M][N] int32
};

__device__ __forceinline__ uint32_t rotr(uint32_t x, int s) { return __builtin_amdgcn_alignbit(x, x, s); }

// 32 K positions of one operand row -> 4 dwords of 8 FP4 codes; nibble i of
// dword r holds the element at bit (r + 4 i) of the plane words.
template <int KIND> __device__ __forceinline__ void expand_fp4(const uint32_t *w, int stride, v8i_t &out)
{
    if (KIND == OPK_U1) {                       // 0 -> 0000 (0.0), 1 -> 0010 (1.0)
        const uint32_t x = w[0];
        out[0] = rotr(x, 31) & 0x22222222u;
        out[1] = x & 0x22222222u;
        out[2] = rotr(x, 1) & 0x22222222u;
        out[3] = rotr(x, 2) & 0x22222222u;
    } else if (KIND == OPK_PM1) {               // 1 -> 0010 (+1.0), 0 -> 1010 (-1.0)
        const uint32_t nx = ~w[0];
        out[0] = (rotr(nx, 29) & 0x88888888u) | 0x22222222u;
        out[1] = (rotr(nx, 30) & 0x88888888u) | 0x22222222u;
        out[2] = (rotr(nx, 31) & 0x88888888u) | 0x22222222u;
        out[3] = (nx & 0x88888888u) | 0x22222222u;
    } else {                                    // 0,1,2,3 -> 0000, 0010, 0100, 0101
        const uint32_t x0 = w[0], x1 = w[stride];
        const uint32_t m0 = x0 & x1, m1 = x0 ^ m0, m2 = x1;
        out[0] = (rotr(m2, 30) & 0x44444444u) | (rotr(m1, 31) & 0x22222222u) | (m0 & 0x11111111u);
        out[1] = (rotr(m2, 31) & 0x44444444u) | (m1 & 0x22222222u) | (rotr(m0, 1) & 0x11111111u);
        out[2] = (m2 & 0x44444444u) | (rotr(m1, 1) & 0x22222222u) | (rotr(m0, 2) & 0x11111111u);
        out[3] = (rotr(m2, 1) & 0x44444444u) | (rotr(m1, 2) & 0x22222222u) | (rotr(m0, 3) & 0x11111111u);
    }
    out[4] = out[5] = out[6] = out[7] = 0;
}

template <int KIND> struct OpPlanes { static constexpr int value = (KIND == OPK_U2) ? 2 : 1; };

template <int KA, int KB>
__global__ __launch_bounds__(256, 1) void mfma_fp4_kernel(const MfmaParams p)
{
    constexpr int KC = 8;                               // words per chunk
    constexpr int PA = OpPlanes<KA>::value, PB = OpPlanes<KB>::value;
    constexpr int BT = 256;                             // block tile edge
    constexpr int RSA = PA * KC + 4, RSB = PB * KC + 4; // padded LDS row strides (words)
    constexpr int A_VECS = BT * PA * 2, B_VECS = BT * PB * 2;   // 16-byte vectors per chunk
    constexpr int A_SLOTS = A_VECS / 256, B_SLOTS = B_VECS / 256;

    __shared__ __attribute__((aligned(16))) uint32_t sA[2][BT * RSA];
    __shared__ __attribute__((aligned(16))) uint32_t sB[2][BT * RSB];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;            // wave position in the 2 x 2 arrangement
    const int lr = lane & 31, lh = lane >> 5;           // row / column inside a 32-wide tile, K half

    const int tilesN = (p.N + BT - 1) / BT;
    const int m0 = (blockIdx.x / tilesN) * BT, n0 = (blockIdx.x % tilesN) * BT;

    // loader: vector v = tid + 256 u covers (row, plane, half-chunk c): v = (row*P + plane)*2 + c
    uint4 ra[A_SLOTS], rb[B_SLOTS];
    auto fetch = [&](int kc) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            const int v = tid + 256 * u, c = v & 1, rp = v >> 1;
            const int row = rp / PA, pl = rp % PA, kk = kc * KC + 4 * c;
            ra[u] = make_uint4(0, 0, 0, 0);
            if (m0 + row < p.M && kk < p.ldwA)
                ra[u] = *reinterpret_cast<const uint4 *>(p.A + (static_cast<int64_t>(m0 + row) * PA + pl) * p.ldwA + kk);
        }
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) {
            const int v = tid + 256 * u, c = v & 1, rp = v >> 1;
            const int row = rp / PB, pl = rp % PB, kk = kc * KC + 4 * c;
            rb[u] = make_uint4(0, 0, 0, 0);
            if (n0 + row < p.N && kk < p.ldwB)
                rb[u] = *reinterpret_cast<const uint4 *>(p.B + (static_cast<int64_t>(n0 + row) * PB + pl) * p.ldwB + kk);
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            const int v = tid + 256 * u, c = v & 1, rp = v >> 1;
            *reinterpret_cast<uint4 *>(&sA[buf][(rp / PA) * RSA + (rp % PA) * KC + 4 * c]) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) {
            const int v = tid + 256 * u, c = v & 1, rp = v >> 1;
            *reinterpret_cast<uint4 *>(&sB[buf][(rp / PB) * RSB + (rp % PB) * KC + 4 * c]) = rb[u];
        }
    };

    v16f_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    if (p.nk > 0) {
        fetch(0);
        stage(0);
    }
    __syncthreads();

    for (int kc = 0; kc < p.nk; ++kc) {
        const int buf = kc & 1;
        if (kc + 1 < p.nk) fetch(kc + 1);

        // this lane's words of the chunk: 4 steps x planes, for its 4 + 4 tile rows
        uint32_t wa[4][PA][4], wb[4][PB][4];
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int pl = 0; pl < PA; ++pl) {
                const uint4 v = *reinterpret_cast<const uint4 *>(&sA[buf][(wm * 128 + f * 32 + lr) * RSA + pl * KC + 4 * lh]);
                wa[f][pl][0] = v.x; wa[f][pl][1] = v.y; wa[f][pl][2] = v.z; wa[f][pl][3] = v.w;
            }
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int pl = 0; pl < PB; ++pl) {
                const uint4 v = *reinterpret_cast<const uint4 *>(&sB[buf][(wn * 128 + f * 32 + lr) * RSB + pl * KC + 4 * lh]);
                wb[f][pl][0] = v.x; wb[f][pl][1] = v.y; wb[f][pl][2] = v.z; wb[f][pl][3] = v.w;
            }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            v8i_t fa[4], fb[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                uint32_t t[2];
                t[0] = wa[f][0][st]; t[1] = wa[f][PA - 1][st];
                expand_fp4<KA>(t, 1, fa[f]);
            }
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                uint32_t t[2];
                t[0] = wb[f][0][st]; t[1] = wb[f][PB - 1][st];
                expand_fp4<KB>(t, 1, fb[f]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], acc[i][j], 4, 4, 0,
                                                                                 0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
        if (kc + 1 < p.nk) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- int32 store.  Accumulator register r of lane (lh, lr) in tile (i, j) is
    // row 8*(r/4) + 4*lh + r%4, column lr of that 32 x 32 tile.
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int gm = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (gm < p.M) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int gn = n0 + wn * 128 + j * 32 + lr;
                    if (gn < p.N) p.Y[static_cast<int64_t>(gm) * p.N + gn] = static_cast<int>(acc[i][j][r]) + p.c0;
                }
            }
        }
}

}  // namespace apnn
