// Small-layer matrix-core kernel with wave tiles of 32 x 32 FN outputs (FN column tiles of 32 channels per wave
// tile): the form for large convolution layers, where every wave owns its own tile (no K split) and the kernel is
// bound by the instructions its waves issue.  The row operand of a wave tile - pixel decoding, tap addresses,
// loads, expansion to FP4 codes - is then shared by 32 FN output channels: at batch 128 the stage-1 layers of the
// ResNet-18 shape take 41 - 54 us with FN = 2 against 59 - 74 us with FN = 1 (FN = 4 with its larger register
// footprint was slower again).  Loader, arithmetic and epilogue are those of mfma_small_kernel, which keeps its own
// FN = 1 body: the general form compiles to slightly slower code for the small layers it was tuned on.
#pragma once
#include "mfma_kernel.h"

namespace apnn {

template <int KA, int KB, int VW, bool CONV, int NSPLIT, int GMAX, int FN>
__device__ __forceinline__ void mfma_small_wide_body(const MfmaParams &p, const int block)
{
    // GMAX: groups of four steps whose loads are in flight together.  The load buffers set the register count and
    // with it the number of blocks a compute unit holds at once: 1 or 2 for layers with a short K and many blocks,
    // 5 for a long K.  FN: 32-column tiles per wave tile: a row operand is loaded, expanded and its
    // pixel decoded once for 32 FN output channels.  A large layer is bound by the instructions its waves issue,
    // and the row side is about a third of them.
    constexpr int LA = DigitPlanes<KA>::value, LB = DigitPlanes<KB>::value;
    constexpr int RPW = 16 / NSPLIT;                    // accumulator registers per 32 x 32 tile a wave finishes in the epilogue

    __shared__ float sRed[NSPLIT > 1 ? NSPLIT : 1][NSPLIT > 1 ? 16 * FN : 1][64];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 31, lh = lane >> 5;
    const int ks = NSPLIT > 1 ? wave : 0;               // K-split index of this wave

    // tile of this wave: with NSPLIT = 1 the block covers four consecutive tiles of the row-major tile grid
    const int tilesN = (p.N + 32 * FN - 1) / (32 * FN), tilesM = (p.M + 31) / 32;
    const int tile = NSPLIT > 1 ? block : block * 4 + wave;
    const bool live = tile < tilesM * tilesN;           // trailing waves of the last block have no tile
    const int m0 = (tile / tilesN) * 32, n0 = (tile % tilesN) * 32 * FN;

    const int NSe = (((p.Kw + 1) >> 1) + 3) / 4 * 4;
    const int GT = NSe / 4;                             // groups of four steps in all; wave ks takes groups ks, ks + NSPLIT, ...
    const int G = (GT - ks + NSPLIT - 1) / NSPLIT;      // ... of which this wave has G (waves of a block may differ by one)

    Fp4Masks km;
    km.m1 = reg_const(0x11111111u); km.m2 = reg_const(0x22222222u);
    km.m4 = reg_const(0x44444444u); km.m8 = reg_const(0x88888888u);

    // this lane's operand rows
    const int gmA = m0 + lr;
    const bool a_ok = live && gmA < p.M;
    int a_h0 = 0, a_w0 = 0;
    int64_t a_pix = 0;
    if (CONV) {
        int wo, ho, n;
        conv_row_to_pixel(p, gmA, n, ho, wo);
        a_h0 = ho * p.stride - p.pad;
        a_w0 = wo * p.stride - p.pad;
        a_pix = static_cast<int64_t>(n) * p.H * p.W;
    }
    const uint32_t *a_row = p.A + static_cast<int64_t>(gmA) * p.PA * p.ldwA;      // matrix mode
    const uint32_t *b_row[FN];
    bool b_ok[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int gnB = n0 + 32 * j + lr;
        b_ok[j] = live && gnB < p.N;
        b_row[j] = p.B + static_cast<int64_t>(gnB) * p.PB * p.ldwB;
    }

    // Words kk .. kk+3 of plane `plane` of this lane's A row (zero beyond Kw / outside the frame).
    auto load_a = [&](int plane, int kk) -> uint4 {
        uint4 v = make_uint4(0, 0, 0, 0);
        const bool validity = KA == OPK_PM1Z && plane == 1;     // all ones for taps inside the frame, made up here
        if (validity) plane = 0;
        if (!a_ok || kk >= p.Kw || plane >= p.PA) return v;
        if (CONV) {
            // VW = 4: the four words lie in one tap; VW = 2: two taps of two words each
#pragma unroll
            for (int part = 0; part < 4 / VW; ++part) {
                const int k = kk + part * VW;
                if (k < p.Kw) {
                    const int tap = static_cast<int>((static_cast<float>(k) + 0.5f) * p.invCw);
                    const int cw = k - tap * p.Cw;
                    int r, sc;
                    tap_to_rs(p, tap, r, sc);
                    const int h = a_h0 + r, w = a_w0 + sc;
                    if (h >= 0 && h < p.H && w >= 0 && w < p.W) {
                        const uint32_t *src = p.A + ((a_pix + h * p.W + w) * p.PA + plane) * p.Cw + cw;
                        if (validity) {
                            if (VW == 4) v = make_uint4(~0u, ~0u, ~0u, ~0u);
                            else if (part == 0) { v.x = ~0u; v.y = ~0u; } else { v.z = ~0u; v.w = ~0u; }
                        } else if (VW == 4) {
                            v = *reinterpret_cast<const uint4 *>(src);
                        } else {
                            const uint2 t = *reinterpret_cast<const uint2 *>(src);
                            if (part == 0) { v.x = t.x; v.y = t.y; } else { v.z = t.x; v.w = t.y; }
                        }
                    }
                }
            }
        } else {
            v = *reinterpret_cast<const uint4 *>(a_row + static_cast<int64_t>(plane) * p.ldwA + kk);
        }
        return v;
    };
    auto load_b = [&](int j, int plane, int kk) -> uint4 {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (!b_ok[j] || kk >= p.Kw || plane >= p.PB) return v;
        const uint32_t *src = b_row[j] + static_cast<int64_t>(plane) * p.ldwB + kk;
        if (!CONV) {
            v = *reinterpret_cast<const uint4 *>(src);
        } else {                                // conv weight rows are 8-byte aligned and an even number of words long
            const uint2 lo = *reinterpret_cast<const uint2 *>(src);
            v.x = lo.x; v.y = lo.y;
            if (kk + 4 <= p.Kw) {
                const uint2 hi = *reinterpret_cast<const uint2 *>(src + 2);
                v.z = hi.x; v.w = hi.y;
            }
        }
        return v;
    };

    // the epilogue's per-channel parameters and residual words: their latency hides behind the main loop
    // (residual: one load per wave and group of eight rows: lane l holds the word of row l & 7, plane l >> 3)
    constexpr int NG = RPW / 4;                         // groups of four registers = eight rows this wave finishes per tile
    float sc[FN], bi[FN];
    uint32_t pre_res[FN][NG];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int gn = n0 + 32 * j + lr;
        sc[j] = 0.0f; bi[j] = 0.0f;
        if (p.scale && live && gn < p.N) { sc[j] = p.scale[gn]; bi[j] = p.bias[gn]; }
#pragma unroll
        for (int g = 0; g < NG; ++g)
            pre_res[j][g] = (live && !p.pool) ? load_res_rows8(p, m0 + 8 * (NSPLIT > 1 ? ks : g), gn >> 5, lane) : 0u;
    }

    // Digit pairs (da, db) and the groups of four steps of each are walked as one
    // flat sequence, GMAX entries at a time with all their loads in flight together,
    // so that a multi-digit layer (e.g. 8-bit features: four passes) pays one memory
    // round trip, not one per pass.  The weight 4^(da + db) of a pair (Eq. 1) enters
    // as the block scales of the matrix instruction, which makes the order free.
    const int total = p.Kw > 0 ? p.DA * p.DB * G : 0;
    const int kbase = lh * NSe + 4 * ks;                // first K word of this lane's first group; the next is 4 NSPLIT further

    v16f_t acc[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    // the four steps of one group: operand words of the lowest and highest plane of the digit (one and the same
    // for single-plane kinds), block scales of the digit pair
    auto run_group = [&](const uint4 (&wa)[LA], const uint4 (&wb)[FN][LB], int sa, int sb) {
        const uint32_t a0[4] = {wa[0].x, wa[0].y, wa[0].z, wa[0].w};
        const uint32_t a1[4] = {wa[LA - 1].x, wa[LA - 1].y, wa[LA - 1].z, wa[LA - 1].w};
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            v8i_t fa;
            expand_fp4<KA>(a0[st], a1[st], km, fa);
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const uint32_t b0[4] = {wb[j][0].x, wb[j][0].y, wb[j][0].z, wb[j][0].w};
                const uint32_t b1[4] = {wb[j][LB - 1].x, wb[j][LB - 1].y, wb[j][LB - 1].z, wb[j][LB - 1].w};
                v8i_t fb;
                expand_fp4<KB>(b0[st], b1[st], km, fb);
                acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc[j], 4, 4, 0, sa, 0, sb);
            }
        }
    };

    if (p.DA * p.DB == 1) {                             // one digit pair (most layers): unit scales, plain group loop
        for (int g0 = 0; g0 < (p.Kw > 0 ? G : 0); g0 += GMAX) {
            uint4 wa[GMAX][LA], wb[GMAX][FN][LB];
#pragma unroll
            for (int g = 0; g < GMAX; ++g) {
                const int kk = (g0 + g < G) ? kbase + 4 * NSPLIT * (g0 + g) : p.Kw;   // beyond G: reads as zero, not used
#pragma unroll
                for (int pl = 0; pl < LA; ++pl) wa[g][pl] = load_a(pl, kk);
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int pl = 0; pl < LB; ++pl) wb[g][j][pl] = load_b(j, pl, kk);
            }
#pragma unroll
            for (int g = 0; g < GMAX; ++g)
                if (g0 + g < G) run_group(wa[g], wb[g], 0x7f7f7f7f, 0x7f7f7f7f);
        }
    }
    int da = 0, db = 0, grp = 0;                        // position in the flat sequence (scalar counters, no divisions)
    for (int e0 = 0; e0 < (p.DA * p.DB == 1 ? 0 : total); e0 += GMAX) {
        uint4 wa[GMAX][LA], wb[GMAX][FN][LB];
        int sa[GMAX], sb[GMAX];
#pragma unroll
        for (int g = 0; g < GMAX; ++g) {
            const int planeA = LA == 2 ? 2 * da : da, planeB = LB == 2 ? 2 * db : db;
            const int kk = e0 + g < total ? kbase + 4 * NSPLIT * grp : p.Kw;    // beyond the end: reads as zero, not used
            sa[g] = 0x7f7f7f7f + 0x02020202 * da;
            sb[g] = 0x7f7f7f7f + 0x02020202 * db;
#pragma unroll
            for (int pl = 0; pl < LA; ++pl) wa[g][pl] = load_a(planeA + pl, kk);
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int pl = 0; pl < LB; ++pl) wb[g][j][pl] = load_b(j, planeB + pl, kk);
            ++grp;                                      // next group, then next digit of B, then next digit of A
            const bool wg = grp == G;
            grp = wg ? 0 : grp;
            db += wg ? 1 : 0;
            const bool wd = db == p.DB;
            db = wd ? 0 : db;
            da += wd ? 1 : 0;
        }
#pragma unroll
        for (int g = 0; g < GMAX; ++g)
            if (e0 + g < total) run_group(wa[g], wb[g], sa[g], sb[g]);
    }

    MfmaParams pq = p;                          // pooled outputs: a quarter of the rows, corrections per grid
    pq.M = p.M >> 2;
    pq.c0 = p.pool == 2 ? 4 * p.c0 : p.c0;
    if constexpr (NSPLIT == 1) {
        if (!live) return;                      // wave-uniform: the ballots below stay whole-wave
        static_for<FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int gn = n0 + 32 * j + lr;
            if (p.pool) {                       // registers 4 k .. 4 k + 3 of a lane are one pooling grid
                static_for<4>([&](auto kc) {
                    constexpr int k = decltype(kc)::value;
                    finish_value(pq, pool4(p.pool, acc[j][4 * k], acc[j][4 * k + 1], acc[j][4 * k + 2], acc[j][4 * k + 3]),
                                 (m0 + 8 * k + 4 * lh) >> 2, gn, sc[j], bi[j], false, 0u, lr, lh);
                });
            } else {
                static_for<4>([&](auto kc) {
                    constexpr int k = decltype(kc)::value;
                    const float v4[4] = {acc[j][4 * k], acc[j][4 * k + 1], acc[j][4 * k + 2], acc[j][4 * k + 3]};
                    finish_rows8(p, v4, m0 + 8 * k, gn, sc[j], bi[j], pre_res[j][k], lane, lr, lh);
                });
            }
        });
    } else {
        // add the partial tiles; wave ks finishes accumulator registers 4 ks .. 4 ks + 3 of every 32 x 32 tile:
        // one group of eight rows, or one pooling grid per lane
        static_assert(NSPLIT == 1 || RPW == 4, "a K-split wave finishes one group of eight rows");
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) sRed[ks][16 * j + r][lane] = acc[j][r];
        __syncthreads();
        static_for<FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int gn = n0 + 32 * j + lr;
            float v4[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                v4[rr] = 0.0f;
#pragma unroll
                for (int k = 0; k < NSPLIT; ++k) v4[rr] += sRed[k][16 * j + ks * 4 + rr][lane];
            }
            if (p.pool)
                finish_value(pq, pool4(p.pool, v4[0], v4[1], v4[2], v4[3]), (m0 + 8 * ks + 4 * lh) >> 2, gn, sc[j], bi[j],
                             false, 0u, lr, lh);
            else
                finish_rows8(p, v4, m0 + 8 * ks, gn, sc[j], bi[j], pre_res[j][0], lane, lr, lh);
        });
    }
}

template <int KA, int KB, int VW, int FN>
__global__ __launch_bounds__(256) void mfma_small_wide_kernel(const MfmaParams p)
{
    mfma_small_wide_body<KA, KB, VW, true, 1, 2, FN>(p, blockIdx.x);
}

}  // namespace apnn
