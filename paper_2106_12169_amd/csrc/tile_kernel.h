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
// -1/+1 features (PMZ instances; Sec. 4.2 (b), padding for Case II and for the
// mirror of Case III): a 0 bit means -1, so zero words would not contribute 0.
// With V the validity of a position (1 inside the frame) a feature is
// a = 2 a^ - V, and for a weight plane B_t
//     sum_k a_k B_t,k = 2 popc(a^ & B_t) - popc(V & B_t):
// the features become a two-plane operand (plane 1 = the stored bits, which are
// 0 outside the frame; plane 0 = V, made up by the loader, never read from
// memory) whose plane 0 counts negatively.  -popc(x) = popc(~x) - 32, so the V
// passes accumulate popc(~(V & B_t)) with the same two instructions per word
// and the host folds -32 per word and weight of the pass into c0.  For -1/+1
// weights the remaining row term popc(V) - 2 popc(a^) comes from the loader-side
// popcounts that Case III uses.
//
// Fused 2 x 2 grid pooling (Sec. 5.2): rows are enumerated as
// 4 (pooled pixel) + 2 dy + dx, so a grid is four consecutive tile rows: the
// four (RA >= 4) or two (RA = 2, the other two one lane exchange away) rows a
// thread holds.  The maximum / sum is taken on the recovered int32 results and
// the rest of the epilogue runs once per grid.
//
// The epilogue (Sec. 4.1 (b) element-wise routine, Sec. 5.2 fusion) runs on the
// register tile: optional int32 store, fp32 fma with the folded per-channel
// scale/bias, optional residual, floor/clamp to q_out bits, bit decomposition
// and cross-lane packing of 32 channels per word.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "vec_util.h"

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
    int xm, xn;          // 8 XCDs arranged as an xm x xn grid of tile regions (0: plain order)
    int pool, Hp, Wp;    // fused 2 x 2 grid pooling (0 none, 1 maximum, 2 sum) and the pooled frame; M counts 4 rows per pooled pixel
};

// registers -> LDS in pieces of at most LV words (LDS rows are LV-word aligned)
template <int LV> __device__ __forceinline__ void lds_store(uint32_t *dst, uint4 v)
{
    if (LV >= 4) {
        *reinterpret_cast<uint4 *>(dst) = v;
    } else {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(v.x, v.y);
        *reinterpret_cast<uint2 *>(dst + 2) = make_uint2(v.z, v.w);
    }
}
template <int LV> __device__ __forceinline__ void lds_store(uint32_t *dst, uint2 v) { *reinterpret_cast<uint2 *>(dst) = v; }
template <int LV> __device__ __forceinline__ void lds_store(uint32_t *dst, uint32_t v) { *dst = v; }

// LV words of one tile row from LDS
template <int LV> struct LdsVec;
template <> struct LdsVec<4> {
    uint32_t w[4];
    __device__ __forceinline__ void load(const uint32_t *src)
    {
        const uint4 v = *reinterpret_cast<const uint4 *>(src);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    }
};
template <> struct LdsVec<2> {
    uint32_t w[2];
    __device__ __forceinline__ void load(const uint32_t *src)
    {
        const uint2 v = *reinterpret_cast<const uint2 *>(src);
        w[0] = v.x; w[1] = v.y;
    }
};

// LDS word offset of tile row r: KC words per row plus LV pad words after every
// RR rows, so that the 16 threads of a half-row group (rows tx*RR + j) hit
// distinct banks when they read LV-word vectors.
template <int KC, int RR, int LV> __device__ __forceinline__ int lds_row(int r) { return r * KC + LV * (r / RR); }

template <int RA, int RB, int KC, int VW, int LV, bool CONV, bool XOR, bool PMZ = false>
__global__ __launch_bounds__(256, (RA * RB >= 64 ? 2 : 4)) void tile_kernel(const TileParams p)
{
    static_assert(!PMZ || (CONV && !XOR), "validity-plane features exist for convolutions only");
    constexpr int BM = 16 * RA, BN = 16 * RB;
    constexpr int CH = KC / VW;                       // loader vectors per tile row and chunk
    constexpr int A_VECS = BM * CH, B_VECS = BN * CH;
    constexpr int A_SLOTS = (A_VECS + 255) / 256, B_SLOTS = (B_VECS + 255) / 256;
    constexpr int A_WORDS = BM * KC + LV * 16, B_WORDS = BN * KC + LV * 16;
    constexpr int NG = KC / LV;                       // LDS read groups per chunk
    using Vec = typename VecT<VW>::type;

    __shared__ __attribute__((aligned(16))) uint32_t sA[2][A_WORDS];
    __shared__ __attribute__((aligned(16))) uint32_t sB[2][B_WORDS];
    __shared__ int sRsA[BM];
    __shared__ int sRsB[BN];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;

    // ---- block -> tile.  Blocks are dealt round-robin to the 8 XCDs, each with
    // its own L2: the tile grid is cut into xm x xn rectangular regions, one per
    // XCD, so the operand rows a die touches (region rows of A + region columns of
    // B) stay inside its L2; inside a region tiles run column-fastest.
    const int tilesN = (p.N + BN - 1) / BN;
    int tm, tn;
    if (p.xm > 0) {
        const int tilesM = (p.M + BM - 1) / BM;
        const int rm = tilesM / p.xm, rn = tilesN / p.xn;
        const int xcd = blockIdx.x & 7, tile = blockIdx.x >> 3;
        tm = (xcd / p.xn) * rm + tile / rn;
        tn = (xcd % p.xn) * rn + tile % rn;
    } else {
        tm = blockIdx.x / tilesN;
        tn = blockIdx.x % tilesN;
    }
    const int m0 = tm * BM, n0 = tn * BN;

    // Plane pairs are visited diagonal by diagonal, d = s + t from PA+PB-2 down to 0
    // (within a diagonal s ascending), so that Eq. 1 can be evaluated by Horner's
    // rule directly in the accumulators: tot = 2*tot when the diagonal changes.
    const int dmax = p.PA + p.PB - 2;
    auto first_s = [&](int d) { return max(0, d - (p.PB - 1)); };
    auto next_pair = [&](int &s_, int &t_) {           // returns true when the diagonal changes
        if (s_ + 1 < p.PA && t_ - 1 >= 0) { ++s_; --t_; return false; }
        const int d = s_ + t_ - 1;
        if (d < 0) return false;
        s_ = first_s(d); t_ = d - s_;
        return true;
    };
    const int total_it = p.PA * p.PB * p.nk;

    {
        if (tid < BM) sRsA[tid] = 0;
        if (tid < BN) sRsB[tid] = 0;

        // ---- loader: slot u of this thread moves vector v = tid + 256 u of the tile:
        // tile row v / CH, words (v % CH) * VW .. + VW of the chunk.
        int a_h0[A_SLOTS], a_w0[A_SLOTS], a_pix[A_SLOTS];      // conv: top-left input coordinate, image base pixel
        if (CONV) {
#pragma unroll
            for (int u = 0; u < A_SLOTS; ++u) {
                const int gm = m0 + (tid + 256 * u) / CH;
                int wo, ho, n;
                if (p.pool) {                                      // row = 4 (pooled pixel) + 2 dy + dx
                    const int g = gm >> 2;
                    wo = 2 * (g % p.Wp) + (gm & 1);
                    ho = 2 * ((g / p.Wp) % p.Hp) + ((gm >> 1) & 1);
                    n = g / (p.Wp * p.Hp);
                } else {
                    wo = gm % p.Wo; ho = (gm / p.Wo) % p.Ho; n = gm / (p.Wo * p.Ho);
                }
                a_h0[u] = ho * p.stride - p.pad;
                a_w0[u] = wo * p.stride - p.pad;
                a_pix[u] = n * p.H * p.W;
            }
        }
        auto load_a = [&](int u, int s, int k0) -> Vec {
            Vec v = vec_zero<VW>();
            const int vi = tid + 256 * u;
            const int gm = m0 + vi / CH, kk = k0 + (vi % CH) * VW;
            if (vi < A_VECS && gm < p.M && kk < p.Kw) {
                if (CONV) {
                    const int tap = static_cast<int>((static_cast<float>(kk) + 0.5f) * p.invCw);
                    const int cw = kk - tap * p.Cw;
                    const int r = tap / p.S, sc = tap - r * p.S;
                    const int h = a_h0[u] + r, w = a_w0[u] + sc;
                    if (h >= 0 && h < p.H && w >= 0 && w < p.W) {
                        const int64_t pix = a_pix[u] + h * p.W + w;
                        if (PMZ) {                                 // one stored plane; plane 0 of the operand is the validity
                            if (s == 0) v = vec_ones<VW>();
                            else v = *reinterpret_cast<const Vec *>(p.A + pix * p.Cw + cw);
                        } else {
                            v = *reinterpret_cast<const Vec *>(p.A + (pix * p.PA + s) * p.Cw + cw);
                        }
                    }
                } else {
                    v = *reinterpret_cast<const Vec *>(p.A + (static_cast<int64_t>(gm) * p.PA + s) * p.ldwA + kk);
                }
            }
            return v;
        };
        auto load_b = [&](int u, int t, int k0) -> Vec {
            Vec v = vec_zero<VW>();
            const int vi = tid + 256 * u;
            const int gn = n0 + vi / CH, kk = k0 + (vi % CH) * VW;
            if (vi < B_VECS && gn < p.N && kk < p.Kw)
                v = *reinterpret_cast<const Vec *>(p.B + (static_cast<int64_t>(gn) * p.PB + t) * p.ldwB + kk);
            return v;
        };

        int tot[RA][RB];
#pragma unroll
        for (int i = 0; i < RA; ++i)
#pragma unroll
            for (int j = 0; j < RB; ++j) tot[i][j] = 0;
        int rsA[A_SLOTS], rsB[B_SLOTS];
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) rsA[u] = 0;
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) rsB[u] = 0;

        Vec ra[A_SLOTS], rb[B_SLOTS];
        int fs = first_s(dmax), ft = dmax - fs, fk = 0;   // plane pair / chunk being fetched
        int ls = 0, lt = 0;                               // plane pair of the tile held in ra/rb
        auto fetch = [&]() {                   // issue the global loads only; nothing waits on them here
#pragma unroll
            for (int u = 0; u < A_SLOTS; ++u) ra[u] = load_a(u, fs, fk * KC);
#pragma unroll
            for (int u = 0; u < B_SLOTS; ++u) rb[u] = load_b(u, ft, fk * KC);
            ls = fs; lt = ft;
            if (++fk == p.nk) { fk = 0; next_pair(fs, ft); }
        };
        auto stage = [&](int buf) {            // registers -> LDS, plus the row-sum popcounts (J X term)
            if (p.uA != 0 && lt == 0) {
#pragma unroll
                for (int u = 0; u < A_SLOTS; ++u)
                    rsA[u] += PMZ ? (ls == 0 ? vec_popc(ra[u]) : -2 * vec_popc(ra[u])) : vec_popc(ra[u]) << ls;
            }
            if (p.uB != 0 && ls == 0) {
#pragma unroll
                for (int u = 0; u < B_SLOTS; ++u) rsB[u] += vec_popc(rb[u]) << lt;
            }
#pragma unroll
            for (int u = 0; u < A_SLOTS; ++u) {
                const int vi = tid + 256 * u;
                if (vi < A_VECS) lds_store<LV>(&sA[buf][lds_row<KC, RA, LV>(vi / CH) + (vi % CH) * VW], ra[u]);
            }
#pragma unroll
            for (int u = 0; u < B_SLOTS; ++u) {
                const int vi = tid + 256 * u;
                if (vi < B_VECS) lds_store<LV>(&sB[buf][lds_row<KC, RB, LV>(vi / CH) + (vi % CH) * VW], rb[u]);
            }
        };

        if (total_it > 0) {
            fetch();
            stage(0);
        }
        __syncthreads();

        int cs = first_s(dmax), ct = dmax - cs, ck = 0;   // plane pair / chunk being computed
        for (int it = 0; it < total_it; ++it) {
            const int buf = it & 1;
            if (it + 1 < total_it) fetch();    // global loads for the next chunk fly during the compute below

            const int words = min(KC, p.Kw - ck * KC);
            const int ng = (words + LV - 1) / LV;
            const uint32_t *pa = &sA[buf][lds_row<KC, RA, LV>(ty * RA)];
            const uint32_t *pb = &sB[buf][lds_row<KC, RB, LV>(tx * RB)];
            // register double buffer over LV-word groups: the LDS reads of group g+1
            // are issued before the AND/popcount block of group g
            LdsVec<LV> a[2][RA], b[2][RB];
#pragma unroll
            for (int i = 0; i < RA; ++i) a[0][i].load(pa + i * KC);
#pragma unroll
            for (int j = 0; j < RB; ++j) b[0][j].load(pb + j * KC);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g < ng) {
                    const int cur = g & 1, nxt = cur ^ 1;
                    if (g + 1 < NG && g + 1 < ng) {
#pragma unroll
                        for (int i = 0; i < RA; ++i) a[nxt][i].load(pa + i * KC + LV * (g + 1));
#pragma unroll
                        for (int j = 0; j < RB; ++j) b[nxt][j].load(pb + j * KC + LV * (g + 1));
                    }
                    // validity plane of -1/+1 features: counts negatively, -popc(x) = popc(~x) - 32 (one three-input
                    // bit operation either way)
                    const uint32_t inv = (PMZ && cs == 0) ? ~0u : 0u;
#pragma unroll
                    for (int i = 0; i < RA; ++i)
#pragma unroll
                        for (int j = 0; j < RB; ++j)
#pragma unroll
                            for (int w = 0; w < LV; ++w)
                                tot[i][j] += XOR   ? __popc(a[cur][i].w[w] ^ b[cur][j].w[w])
                                             : PMZ ? __popc((a[cur][i].w[w] & b[cur][j].w[w]) ^ inv)
                                                   : __popc(a[cur][i].w[w] & b[cur][j].w[w]);
                }
            }
            if (++ck == p.nk) {                // plane pair finished
                ck = 0;
                if (next_pair(cs, ct)) {       // next diagonal: one Horner step of Eq. 1
#pragma unroll
                    for (int i = 0; i < RA; ++i)
#pragma unroll
                        for (int j = 0; j < RB; ++j) tot[i][j] <<= 1;
                }
            }
            if (it + 1 < total_it) stage(buf ^ 1);
            __syncthreads();
        }

        // ---- row sums for the Case III term
        if (p.uA != 0) {
#pragma unroll
            for (int u = 0; u < A_SLOTS; ++u)
                if (tid + 256 * u < A_VECS && rsA[u] != 0) atomicAdd(&sRsA[(tid + 256 * u) / CH], rsA[u]);
        }
        if (p.uB != 0) {
#pragma unroll
            for (int u = 0; u < B_SLOTS; ++u)
                if (tid + 256 * u < B_VECS && rsB[u] != 0) atomicAdd(&sRsB[(tid + 256 * u) / CH], rsB[u]);
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

        // one output row: optional int32 store, scale/bias, residual, requantise, repack
        auto finish_row = [&](int gm, bool rok, const int (&y)[RB]) __attribute__((always_inline)) {
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
        };

        // encoding recovery in place (Sec. 3.2)
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const int rowfix = p.uA * sRsA[ty * RA + i];
#pragma unroll
            for (int j = 0; j < RB; ++j) tot[i][j] = p.alpha * tot[i][j] + rowfix + colfix[j];
        }
        if (CONV && p.pool) {
            // 2 x 2 grid pooling of the int32 results: tile rows 4 g .. 4 g + 3 are one grid (Sec. 5.2)
            auto pool2 = [&](int a, int b) { return p.pool == 1 ? max(a, b) : a + b; };
            const int Mp = p.M >> 2;
            if constexpr (RA >= 4) {
#pragma unroll
                for (int g = 0; g < RA / 4; ++g) {
                    int y[RB];
#pragma unroll
                    for (int j = 0; j < RB; ++j)
                        y[j] = pool2(pool2(tot[4 * g][j], tot[4 * g + 1][j]), pool2(tot[4 * g + 2][j], tot[4 * g + 3][j]));
                    const int gm = (m0 + ty * RA + 4 * g) >> 2;
                    finish_row(gm, gm < Mp, y);
                }
            } else {
                // two rows here, the other two in the thread 16 lanes away (ty ^ 1); the even one finishes the grid
                int y[RB];
#pragma unroll
                for (int j = 0; j < RB; ++j) {
                    const int h = pool2(tot[0][j], tot[RA - 1][j]);
                    y[j] = pool2(h, __shfl_xor(h, 16, 64));
                }
                const int gm = (m0 + ty * RA) >> 2;
                finish_row(gm, gm < Mp && (ty & 1) == 0, y);
            }
        } else {
#pragma unroll
            for (int i = 0; i < RA; ++i) {
                const int gm = m0 + ty * RA + i;
                finish_row(gm, gm < p.M, tot[i]);
            }
        }
    }
}

}  // namespace apnn
