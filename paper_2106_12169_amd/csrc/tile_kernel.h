// The bit-plane tile kernel: one template serves apnn_gemm, apnn_conv2d and
// apnn_layer.
//
// Operand A supplies the output rows (M of them), operand B the output columns
// (N of them); both are K-contiguous packed 1-bit planes.  A block of 256
// threads (16 x 16) owns a (16*RA) x (16*RB) output tile and every thread an
// RA x RB register tile.  The AP-Bit template of Sec. 3.1 is evaluated one plane
// pair (s, t) at a time: for that pair the block walks K in chunks of KC words,
// stages the two 1-bit tiles in LDS (the "shared memory caching" level of
// Sec. 4.1 (a)) and accumulates popcount(A_s & B_t) (or XOR) into registers with
// v_and/v_xor + v_bcnt (the "fragment caching" level: the accumulators never
// leave registers).  When a pair is finished its partial sums are shift-added
// into the running total by 2^(s+t) (Eq. 1, "memory-efficient bit combination",
// Sec. 4.1 (b): the combination never touches memory).  The pair loop is
// flattened with the K loop so that global loads for the next chunk are always
// in flight while the current one is computed (LDS double buffer, one barrier
// per chunk).
//
// Encoding recovery (Sec. 3.2), with S the combined AND/XOR popcount sum:
//   Case I   (0/1 x 0/1)   Y = S
//   Case II  (+-1 x +-1)   Y = K - 2 S            (XOR)
//   Case III (+-1 x 0/1)   Y = 2 S - rowsum(0/1 operand)   (the "J X" term)
// expressed as Y = alpha*S + uA*rsA[row] + uB*rsB[col] + c0.  The row sums are
// popcounts of words the loader threads hold anyway on their way to LDS, so
// the J-term costs a handful of operations per chunk.
//
// In convolution mode (Sec. 4.2) the A rows are output pixels and the K loop
// runs over (kernel row, kernel column, channel word): the loader gathers each
// tap's channel words from the channel-major fmap and substitutes zero words
// for taps outside the frame (zero-contribution padding, valid for Cases I and
// III, Sec. 4.2 (b)).
//
// The epilogue (Sec. 4.1 (b) element-wise routine, Sec. 5.2 fusion) runs on the
// register tile: optional int32 store, fp32 fma with the folded per-channel
// scale/bias, optional residual, floor/clamp to q_out bits, bit decomposition
// and cross-lane packing of 32 channels per word.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace apnn {

struct TileParams {
    const uint32_t *A;   // row operand planes
    const uint32_t *B;   // column operand planes
    int M, N;            // output rows / columns
    int PA, PB;          // planes of A / B
    int ldwA, ldwB;      // words per plane row (A: matrix mode only)
    int Kw;              // words per plane along K that the loop covers
    int nk;              // ceil(Kw / KC)
    int alpha, uA, uB, c0;
    // convolution geometry of the A operand (conv mode only)
    int H, W, Cw, R, S, stride, pad, Ho, Wo;
    float invCw;
    // outputs
    int32_t *Y;          // [M][N] int32 or nullptr
    float *T;            // [M][N] fp32 or nullptr
    const float *scale;  // [N] or nullptr
    const float *bias;   // [N]
    const uint32_t *res; // packed codes [M][q_res][NW] or nullptr
    int q_res;
    float res_scale;
    uint32_t *out;       // packed codes [M][q_out][NW] or nullptr
    int q_out;
    int NW;              // words per plane row of res/out: N / 32
    int xcd_remap;       // grid is a multiple of 8: spread logical tiles per XCD
};

template <int VW> struct VecT;
template <> struct VecT<4> { using type = uint4; };
template <> struct VecT<2> { using type = uint2; };
template <> struct VecT<1> { using type = uint32_t; };

template <int VW> __device__ __forceinline__ typename VecT<VW>::type vec_zero();
template <> __device__ __forceinline__ uint4 vec_zero<4>() { return make_uint4(0, 0, 0, 0); }
template <> __device__ __forceinline__ uint2 vec_zero<2>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint32_t vec_zero<1>() { return 0u; }

__device__ __forceinline__ int vec_popc(uint4 v) { return __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w); }
__device__ __forceinline__ int vec_popc(uint2 v) { return __popc(v.x) + __popc(v.y); }
__device__ __forceinline__ int vec_popc(uint32_t v) { return __popc(v); }

// LDS word offset of tile row r: KC words per row plus one 16-byte pad after
// every RR rows, so that the 16 threads of a half-row group (rows tx*RR + j)
// hit distinct bank groups when they read 16-byte vectors.
template <int KC, int RR> __device__ __forceinline__ int lds_row(int r) { return r * KC + 4 * (r / RR); }

template <int RA, int RB, int KC, int VW, bool CONV, bool XOR>
__global__ __launch_bounds__(256) void tile_kernel(const TileParams p)
{
    constexpr int BM = 16 * RA, BN = 16 * RB;
    constexpr int CH = KC / VW;                       // vectors per tile row and chunk
    constexpr int A_VECS = BM * CH, B_VECS = BN * CH;
    constexpr int A_SLOTS = (A_VECS + 255) / 256, B_SLOTS = (B_VECS + 255) / 256;
    constexpr int A_WORDS = BM * KC + 4 * 16, B_WORDS = BN * KC + 4 * 16;
    using Vec = typename VecT<VW>::type;

    __shared__ __attribute__((aligned(16))) uint32_t sA[2][A_WORDS];
    __shared__ __attribute__((aligned(16))) uint32_t sB[2][B_WORDS];
    __shared__ int sRsA[BM];
    __shared__ int sRsB[BN];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;

    // ---- block -> tile.  Blocks are dealt round-robin to the 8 XCDs; giving
    // XCD x the x-th contiguous eighth of the tile list keeps the operand rows a
    // die works on inside its own L2.
    const int tilesN = (p.N + BN - 1) / BN;
    int bid = blockIdx.x;
    if (p.xcd_remap) bid = (bid & 7) * (gridDim.x >> 3) + (bid >> 3);
    const int m0 = (bid / tilesN) * BM, n0 = (bid % tilesN) * BN;

    if (tid < BM) sRsA[tid] = 0;
    if (tid < BN) sRsB[tid] = 0;

    // ---- loader slots: slot u of this thread moves vector v = tid + 256 u
    int a_row[A_SLOTS], a_off[A_SLOTS];      // tile row, word offset inside chunk
    int a_h0[A_SLOTS], a_w0[A_SLOTS];        // conv: top-left input coordinate
    int64_t a_base[A_SLOTS];                 // matrix: word offset of (row, plane 0); conv: pixel index of image start
    bool a_ok[A_SLOTS];
#pragma unroll
    for (int u = 0; u < A_SLOTS; ++u) {
        const int v = tid + 256 * u;
        a_row[u] = v / CH;
        a_off[u] = (v % CH) * VW;
        const int gm = m0 + a_row[u];
        a_ok[u] = (v < A_VECS) && (gm < p.M);
        if (CONV) {
            const int wo = gm % p.Wo, ho = (gm / p.Wo) % p.Ho, n = gm / (p.Wo * p.Ho);
            a_h0[u] = ho * p.stride - p.pad;
            a_w0[u] = wo * p.stride - p.pad;
            a_base[u] = static_cast<int64_t>(n) * p.H * p.W;
        } else {
            a_h0[u] = a_w0[u] = 0;
            a_base[u] = static_cast<int64_t>(gm) * p.PA * p.ldwA;
        }
    }
    int b_row[B_SLOTS], b_off[B_SLOTS];
    int64_t b_base[B_SLOTS];
    bool b_ok[B_SLOTS];
#pragma unroll
    for (int u = 0; u < B_SLOTS; ++u) {
        const int v = tid + 256 * u;
        b_row[u] = v / CH;
        b_off[u] = (v % CH) * VW;
        const int gn = n0 + b_row[u];
        b_ok[u] = (v < B_VECS) && (gn < p.N);
        b_base[u] = static_cast<int64_t>(gn) * p.PB * p.ldwB;
    }

    auto load_a = [&](int u, int s, int k0) -> Vec {
        Vec v = vec_zero<VW>();
        const int kk = k0 + a_off[u];
        if (a_ok[u] && kk < p.Kw) {
            if (CONV) {
                const int tap = static_cast<int>((static_cast<float>(kk) + 0.5f) * p.invCw);
                const int cw = kk - tap * p.Cw;
                const int r = tap / p.S, sc = tap - r * p.S;
                const int h = a_h0[u] + r, w = a_w0[u] + sc;
                if (h >= 0 && h < p.H && w >= 0 && w < p.W) {
                    const int64_t pix = a_base[u] + static_cast<int64_t>(h) * p.W + w;
                    v = *reinterpret_cast<const Vec *>(p.A + (pix * p.PA + s) * p.Cw + cw);
                }
            } else {
                v = *reinterpret_cast<const Vec *>(p.A + a_base[u] + static_cast<int64_t>(s) * p.ldwA + kk);
            }
        }
        return v;
    };
    auto load_b = [&](int u, int t, int k0) -> Vec {
        Vec v = vec_zero<VW>();
        const int kk = k0 + b_off[u];
        if (b_ok[u] && kk < p.Kw) v = *reinterpret_cast<const Vec *>(p.B + b_base[u] + static_cast<int64_t>(t) * p.ldwB + kk);
        return v;
    };

    int tot[RA][RB], acc[RA][RB];
#pragma unroll
    for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int j = 0; j < RB; ++j) tot[i][j] = acc[i][j] = 0;
    int rsA[A_SLOTS], rsB[B_SLOTS];
#pragma unroll
    for (int u = 0; u < A_SLOTS; ++u) rsA[u] = 0;
#pragma unroll
    for (int u = 0; u < B_SLOTS; ++u) rsB[u] = 0;

    const int total_it = p.PA * p.PB * p.nk;
    Vec ra[A_SLOTS], rb[B_SLOTS];

    // plane pair / chunk of the tile being fetched
    int fs = 0, ft = 0, fk = 0;
    auto fetch = [&]() {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            ra[u] = load_a(u, fs, fk * KC);
            if (p.uA != 0 && ft == 0) rsA[u] += vec_popc(ra[u]) << fs;
        }
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) {
            rb[u] = load_b(u, ft, fk * KC);
            if (p.uB != 0 && fs == 0) rsB[u] += vec_popc(rb[u]) << ft;
        }
        if (++fk == p.nk) { fk = 0; if (++ft == p.PB) { ft = 0; ++fs; } }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u)
            if (tid + 256 * u < A_VECS) *reinterpret_cast<Vec *>(&sA[buf][lds_row<KC, RA>(a_row[u]) + a_off[u]]) = ra[u];
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u)
            if (tid + 256 * u < B_VECS) *reinterpret_cast<Vec *>(&sB[buf][lds_row<KC, RB>(b_row[u]) + b_off[u]]) = rb[u];
    };

    if (total_it > 0) {
        fetch();
        stage(0);
    }
    __syncthreads();

    int cs = 0, ct = 0, ck = 0;               // plane pair / chunk being computed
    for (int it = 0; it < total_it; ++it) {
        const int buf = it & 1;
        if (it + 1 < total_it) fetch();       // global loads for the next chunk fly during the compute below

        const int words = min(KC, p.Kw - ck * KC);
        const int nch = (words + 3) >> 2;
        const uint32_t *pa = &sA[buf][lds_row<KC, RA>(ty * RA)];
        const uint32_t *pb = &sB[buf][lds_row<KC, RB>(tx * RB)];
        for (int c = 0; c < nch; ++c) {
            uint4 a[RA], b[RB];
#pragma unroll
            for (int i = 0; i < RA; ++i) a[i] = *reinterpret_cast<const uint4 *>(pa + i * KC + 4 * c);
#pragma unroll
            for (int j = 0; j < RB; ++j) b[j] = *reinterpret_cast<const uint4 *>(pb + j * KC + 4 * c);
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    if (XOR) {
                        acc[i][j] += __popc(a[i].x ^ b[j].x);
                        acc[i][j] += __popc(a[i].y ^ b[j].y);
                        acc[i][j] += __popc(a[i].z ^ b[j].z);
                        acc[i][j] += __popc(a[i].w ^ b[j].w);
                    } else {
                        acc[i][j] += __popc(a[i].x & b[j].x);
                        acc[i][j] += __popc(a[i].y & b[j].y);
                        acc[i][j] += __popc(a[i].z & b[j].z);
                        acc[i][j] += __popc(a[i].w & b[j].w);
                    }
                }
        }
        if (++ck == p.nk) {                   // plane pair finished: shift-add by 2^(s+t)
            const int sh = cs + ct;
#pragma unroll
            for (int i = 0; i < RA; ++i)
#pragma unroll
                for (int j = 0; j < RB; ++j) { tot[i][j] += acc[i][j] << sh; acc[i][j] = 0; }
            ck = 0;
            if (++ct == p.PB) { ct = 0; ++cs; }
        }
        if (it + 1 < total_it) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- row sums for the Case III term
    if (p.uA != 0) {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u)
            if (tid + 256 * u < A_VECS && rsA[u] != 0) atomicAdd(&sRsA[a_row[u]], rsA[u]);
    }
    if (p.uB != 0) {
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u)
            if (tid + 256 * u < B_VECS && rsB[u] != 0) atomicAdd(&sRsB[b_row[u]], rsB[u]);
    }
    __syncthreads();

    // ---- epilogue on the register tile
    const int gn0 = n0 + tx * RB;
    int colfix[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) colfix[j] = p.uB * sRsB[tx * RB + j] + p.c0;
    float sc[RB], bi[RB];
    if (p.scale) {
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const bool ok = gn0 + j < p.N;
            sc[j] = ok ? p.scale[gn0 + j] : 0.0f;
            bi[j] = ok ? p.bias[gn0 + j] : 0.0f;
        }
    }
    constexpr int LPW = 32 / RB;              // lanes that share one packed output word
    const int wcol = gn0 >> 5;                // word column of this thread's channels
    const int bit0 = gn0 & 31;
    const float qmax = static_cast<float>((1 << (p.q_out > 0 ? p.q_out : 1)) - 1);

#pragma unroll
    for (int i = 0; i < RA; ++i) {
        const int gm = m0 + ty * RA + i;
        const bool rok = gm < p.M;
        const int rowfix = p.uA * sRsA[ty * RA + i];
        int y[RB];
#pragma unroll
        for (int j = 0; j < RB; ++j) y[j] = p.alpha * tot[i][j] + rowfix + colfix[j];

        if (p.Y && rok) {
            int32_t *dst = p.Y + static_cast<int64_t>(gm) * p.N + gn0;
            if ((RB % 4 == 0) && (p.N % 4 == 0) && gn0 + RB <= p.N) {
#pragma unroll
                for (int j = 0; j < RB; j += 4)
                    *reinterpret_cast<int4 *>(dst + j) = make_int4(y[j], y[j + 1], y[j + 2], y[j + 3]);
            } else {
#pragma unroll
                for (int j = 0; j < RB; ++j)
                    if (gn0 + j < p.N) dst[j] = y[j];
            }
        }
        if (p.scale) {
            float t[RB];
#pragma unroll
            for (int j = 0; j < RB; ++j) t[j] = __fmaf_rn(sc[j], static_cast<float>(y[j]), bi[j]);
            if (p.res) {
                uint32_t rw[8];
#pragma unroll
                for (int b = 0; b < 8; ++b)
                    rw[b] = (b < p.q_res && rok && gn0 < p.N)
                                ? p.res[(static_cast<int64_t>(gm) * p.q_res + b) * p.NW + wcol] : 0u;
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    uint32_t code = 0;
#pragma unroll
                    for (int b = 0; b < 8; ++b) code |= ((rw[b] >> (bit0 + j)) & 1u) << b;
                    t[j] = __fmaf_rn(p.res_scale, static_cast<float>(code), t[j]);
                }
            }
            if (p.T && rok) {
#pragma unroll
                for (int j = 0; j < RB; ++j)
                    if (gn0 + j < p.N) p.T[static_cast<int64_t>(gm) * p.N + gn0 + j] = t[j];
            }
            if (p.out) {
                uint32_t code[RB];
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    float f = floorf(t[j]);
                    f = (f >= 0.0f) ? f : 0.0f;
                    f = (f > qmax) ? qmax : f;
                    code[j] = (gn0 + j < p.N) ? static_cast<uint32_t>(f) : 0u;
                }
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    if (b < p.q_out) {
                        uint32_t word = 0;
#pragma unroll
                        for (int j = 0; j < RB; ++j) word |= ((code[j] >> b) & 1u) << (bit0 + j);
#pragma unroll
                        for (int msk = 1; msk < LPW; msk <<= 1) word |= __shfl_xor(word, msk, 64);
                        if ((tx % LPW) == 0 && rok && gn0 < p.N)
                            p.out[(static_cast<int64_t>(gm) * p.q_out + b) * p.NW + wcol] = word;
                    }
                }
            }
        }
    }
}

}  // namespace apnn
