// Matrix-core kernel for small layers: the whole K extent of a 32 x 32 output
// tile is resident in LDS.
//
// Late network layers have few output pixels and a K that fits on chip (at
// most KCMAX words per plane), so they are bound by latency, not throughput: a
// chunked loop would pay one exposed memory round trip per chunk.  Here every
// thread issues all of its global loads at once, the block synchronises once
// per digit pair, and the four waves split the matrix-instruction steps of the
// tile between them (partial tiles added through LDS, epilogue rows shared out
// as in the K-split mode of the chunked kernel).  Arithmetic, operand encodings
// and epilogue are those of mfma_fp4_kernel.
//
// Step geometry (run time): nsteps = ceil(Kw / 2) steps would do; it is rounded
// up to NSe, a multiple of 16, so that every wave owns whole groups of four
// steps.  Lane-half h of step s takes word h*NSe + s of the LDS row (any
// pairing of K positions with steps is valid as long as both operands use the
// same one); words at and beyond Kw are zero.
#pragma once
#include "mfma_kernel.h"

namespace apnn {

template <int KA, int KB, int KCMAX, bool CONV>
__global__ __launch_bounds__(256, 2) void mfma_small_kernel(const MfmaParams p)
{
    static_assert(KCMAX % 32 == 0, "LDS rows hold two halves of a multiple of 16 steps");
    constexpr int LA = DigitPlanes<KA>::value, LB = DigitPlanes<KB>::value;
    constexpr int VWA = CONV ? 2 : 4, VWB = CONV ? 2 : 4;         // loader vector widths (conv rows are 8-byte aligned)
    constexpr int RSA = LA * KCMAX + 4, RSB = LB * KCMAX + 4;     // padded LDS row strides (words)
    constexpr int A_SLOTS = LA * KCMAX / VWA / 8, B_SLOTS = LB * KCMAX / VWB / 8;   // pieces per thread (8 threads per row)
    constexpr int TILE_WORDS = 32 * RSA + 32 * RSB, RED_WORDS = 4 * 16 * 64;
    using VecA = typename VecT<VWA>::type;
    using VecB = typename VecT<VWB>::type;

    __shared__ __attribute__((aligned(16))) uint32_t smem[TILE_WORDS > RED_WORDS ? TILE_WORDS : RED_WORDS];
    uint32_t *sA = smem, *sB = smem + 32 * RSA;

    const int tid = threadIdx.x;
    const int lane = tid & 63, ks = tid >> 6;           // wave = K-split index
    const int lr = lane & 31, lh = lane >> 5;

    const int tilesN = (p.N + 31) / 32;
    const int m0 = (blockIdx.x / tilesN) * 32, n0 = (blockIdx.x % tilesN) * 32;

    const int NSe = (((p.Kw + 1) >> 1) + 15) & ~15;     // steps per digit pair, multiple of 16
    const int G = NSe >> 4;                             // groups of four steps per wave
    const int row_words = 2 * NSe;                      // LDS words per (row, plane) that the steps read

    Fp4Masks km;
    km.m1 = reg_const(0x11111111u); km.m2 = reg_const(0x22222222u);
    km.m4 = reg_const(0x44444444u); km.m8 = reg_const(0x88888888u);

    // ---- loader.  Eight consecutive threads share a tile row and read consecutive
    // pieces of it, so a wave touches few cache lines per load instruction; a
    // thread keeps its row (one set of pixel coordinates) for all of its loads.
    // The planes of one digit are adjacent in memory (fmap: [pixel][plane][Cw],
    // matrix: [row][plane][ldw]), so piece j of a row is tap j / PPT and word
    // (j % PPT) * VW of that tap's run of LA * RUN words.
    const int lrow = tid >> 3, lsub = tid & 7;
    const int runA = CONV ? p.Cw : p.ldwA, runB = p.ldwB;           // words per plane of one contiguous run
    const int pptA = LA * runA / VWA, pptB = LB * runB / VWB;       // pieces per run
    const float inv_pptA = 1.0f / static_cast<float>(pptA), inv_runA = 1.0f / static_cast<float>(runA);
    const float inv_runB = 1.0f / static_cast<float>(runB);
    const int piecesA = LA * p.Kw / VWA, piecesB = LB * p.Kw / VWB;  // pieces per tile row that carry data
    int a_h0 = 0, a_w0 = 0, a_pix = 0;
    if (CONV) {
        const int gm = m0 + lrow;
        const int wo = gm % p.Wo, ho = (gm / p.Wo) % p.Ho, n = gm / (p.Wo * p.Ho);
        a_h0 = ho * p.stride - p.pad;
        a_w0 = wo * p.stride - p.pad;
        a_pix = n * p.H * p.W;
    }
    VecA ra[A_SLOTS];
    VecB rb[B_SLOTS];
    int la[A_SLOTS], lb[B_SLOTS];                       // LDS word offsets of the pieces (or -1)
    auto fetch = [&](int da, int db) {
        const int gm = m0 + lrow, gn = n0 + lrow;
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u) {
            const int j = 8 * u + lsub;
            ra[u] = vec_zero<VWA>();
            la[u] = -1;
            if (j < piecesA) {
                const int tap = static_cast<int>((static_cast<float>(j) + 0.5f) * inv_pptA);
                const int off = (j - tap * pptA) * VWA;                         // word inside the run of LA planes
                const int pl = static_cast<int>((static_cast<float>(off) + 0.5f) * inv_runA);
                const int cw = off - pl * runA;
                const int plane = (LA == 2 ? 2 * da : da) + pl;
                la[u] = lrow * RSA + pl * KCMAX + tap * runA + cw;
                if (gm < p.M && plane < p.PA) {
                    if (CONV) {
                        const int r = tap / p.S, sc = tap - r * p.S;
                        const int h = a_h0 + r, w = a_w0 + sc;
                        if (h >= 0 && h < p.H && w >= 0 && w < p.W) {
                            const int64_t pix = a_pix + h * p.W + w;
                            ra[u] = *reinterpret_cast<const VecA *>(p.A + (pix * p.PA + plane) * p.Cw + cw);
                        }
                    } else {
                        ra[u] = *reinterpret_cast<const VecA *>(p.A + (static_cast<int64_t>(gm) * p.PA + plane) * p.ldwA + cw);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u) {
            const int j = 8 * u + lsub;
            rb[u] = vec_zero<VWB>();
            lb[u] = -1;
            if (j < piecesB) {
                const int off = j * VWB;
                const int pl = static_cast<int>((static_cast<float>(off) + 0.5f) * inv_runB);
                const int cw = off - pl * runB;
                const int plane = (LB == 2 ? 2 * db : db) + pl;
                lb[u] = lrow * RSB + pl * KCMAX + cw;
                if (gn < p.N && plane < p.PB)
                    rb[u] = *reinterpret_cast<const VecB *>(p.B + (static_cast<int64_t>(gn) * p.PB + plane) * p.ldwB + cw);
            }
        }
    };
    // LDS words [Kw, row_words) of every (row, plane) must read as zero: they are
    // cleared once (from the last 16-byte boundary below Kw; the data pieces are
    // written after the barrier and rewritten per digit pair)
    {
        const int kz = p.Kw & ~3, nz = (row_words - kz) >> 2;       // uint4 vectors to clear per (row, plane)
        for (int i = tid; i < 32 * LA * nz; i += 256) {
            const int rp = i / nz, c = i - rp * nz;
            *reinterpret_cast<uint4 *>(&sA[(rp / LA) * RSA + (rp % LA) * KCMAX + kz + 4 * c]) = make_uint4(0, 0, 0, 0);
        }
        for (int i = tid; i < 32 * LB * nz; i += 256) {
            const int rp = i / nz, c = i - rp * nz;
            *reinterpret_cast<uint4 *>(&sB[(rp / LB) * RSB + (rp % LB) * KCMAX + kz + 4 * c]) = make_uint4(0, 0, 0, 0);
        }
    }
    __syncthreads();
    auto stage = [&]() {
#pragma unroll
        for (int u = 0; u < A_SLOTS; ++u)
            if (la[u] >= 0) *reinterpret_cast<VecA *>(&sA[la[u]]) = ra[u];
#pragma unroll
        for (int u = 0; u < B_SLOTS; ++u)
            if (lb[u] >= 0) *reinterpret_cast<VecB *>(&sB[lb[u]]) = rb[u];
    };

    // digit pairs diagonal by diagonal, Horner evaluation in base 4 (as in mfma_fp4_kernel)
    const int dmax = p.DA + p.DB - 2;
    auto first_a = [&](int d) { return max(0, d - (p.DB - 1)); };
    auto next_pair = [&](int &a_, int &b_) {
        if (a_ + 1 < p.DA && b_ - 1 >= 0) { ++a_; --b_; return false; }
        const int d = a_ + b_ - 1;
        if (d < 0) return false;
        a_ = first_a(d); b_ = d - a_;
        return true;
    };
    const int npairs = p.Kw > 0 ? p.DA * p.DB : 0;
    int da = first_a(dmax), db = dmax - da;
    if (npairs > 0) fetch(da, db);

    // the epilogue's per-channel parameters and residual codes: their latency hides behind the loads above
    const int gn = n0 + lr;
    float sc = 0.0f, bi = 0.0f;
    if (p.scale && gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
    uint32_t pre_res[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int gm = m0 + 8 * ks + 4 * lh + rr;       // accumulator register 4 ks + rr
        uint32_t code = 0;
        if (p.res && gm < p.M && gn < p.N) {
            const uint32_t *rp = p.res + static_cast<int64_t>(gm) * p.q_res * p.NW + (gn >> 5);
            for (int b = 0; b < p.q_res; ++b) code |= ((rp[b * p.NW] >> lr) & 1u) << b;
        }
        pre_res[rr] = code;
    }

    v16f_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    for (int pair = 0; pair < npairs; ++pair) {
        stage();
        __syncthreads();
        int na = da, nb = db;
        const bool new_diag = next_pair(na, nb);
        if (pair + 1 < npairs) fetch(na, nb);           // next pair's loads fly during this pair's steps

        const uint32_t *pa = &sA[lr * RSA + lh * NSe + ks * G * 4];
        const uint32_t *pb = &sB[lr * RSB + lh * NSe + ks * G * 4];
        for (int g = 0; g < G; ++g) {
            uint4 wa[LA], wb[LB];
#pragma unroll
            for (int pl = 0; pl < LA; ++pl) wa[pl] = *reinterpret_cast<const uint4 *>(pa + pl * KCMAX + 4 * g);
#pragma unroll
            for (int pl = 0; pl < LB; ++pl) wb[pl] = *reinterpret_cast<const uint4 *>(pb + pl * KCMAX + 4 * g);
            const uint32_t a0[4] = {wa[0].x, wa[0].y, wa[0].z, wa[0].w};
            const uint32_t a1[4] = {wa[LA - 1].x, wa[LA - 1].y, wa[LA - 1].z, wa[LA - 1].w};
            const uint32_t b0[4] = {wb[0].x, wb[0].y, wb[0].z, wb[0].w};
            const uint32_t b1[4] = {wb[LB - 1].x, wb[LB - 1].y, wb[LB - 1].z, wb[LB - 1].w};
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                v8i_t fa, fb;
                expand_fp4<KA>(a0[st], a1[st], km, fa);
                expand_fp4<KB>(b0[st], b1[st], km, fb);
                acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc, 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
            }
        }
        if (new_diag && pair + 1 < npairs) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] *= 4.0f;
        }
        da = na; db = nb;
        __syncthreads();                                // all waves are done with the tile before it is overwritten
    }

    // ---- add the four partial tiles; wave ks finishes accumulator registers 4 ks .. 4 ks + 3
    float (*sRed)[16][64] = reinterpret_cast<float (*)[16][64]>(smem);
#pragma unroll
    for (int r = 0; r < 16; ++r) sRed[ks][r][lane] = acc[r];
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * ks + rr;
        const float v = sRed[0][r][lane] + sRed[1][r][lane] + sRed[2][r][lane] + sRed[3][r][lane];
        finish_value(p, v, m0 + 8 * ks + 4 * lh + rr, gn, sc, bi, true, pre_res[rr], lr, lh);
    }
}

}  // namespace apnn
