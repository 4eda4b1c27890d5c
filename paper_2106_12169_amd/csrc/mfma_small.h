// Matrix-core kernel for small layers: no LDS staging, every lane loads its own
// operand words.
//
// Late network layers have few output pixels, so a launch runs about one wave
// per SIMD and its duration is the length of the instruction stream of a wave.
// A cooperative global -> register -> LDS -> register pipeline costs more
// instructions than the arithmetic itself, so here lane (half lh, row lr) of a
// wave reads, straight from global memory, the 16-byte pieces of its own tile
// row that its matrix-instruction steps consume: piece (row lr, words 4i..4i+3)
// is needed by exactly one lane of the block, nothing is loaded twice and there
// is no barrier before the arithmetic.  All loads of up to GMAX groups of four
// steps are issued before the first of them is used.  With NSPLIT = 4 the four
// waves of a block share one 32 x 32 tile and split its steps (layers with a long
// K and few tiles); with NSPLIT = 1 every wave owns its own tile (layers with a
// short K and many tiles).  Arithmetic, operand encodings, digit passes and the
// epilogue are those of mfma_fp4_kernel.
//
// Step geometry (run time): ceil(Kw / 2) steps would do; that is rounded up to
// NSe, a multiple of 4: groups of four steps, dealt to the NSPLIT waves of a block
// in turn.  Lane-half h of step s takes K word h*NSe + s (any pairing of K
// positions with steps is valid as long as both operands use the same one);
// words at and beyond Kw read as zero.
#pragma once
#include "mfma_kernel.h"

namespace apnn {

template <int KA, int KB, int VW, bool CONV, int NSPLIT, int GMAX>
__device__ __forceinline__ void mfma_small_body(const MfmaParams &p, const int block)
{
    // GMAX: groups of four steps whose loads are in flight together.  The load buffers set the register count and
    // with it the number of blocks a compute unit holds at once: 2 for layers with a short K and many blocks
    // (six waves per SIMD), 5 for a long K.
    constexpr int LA = DigitPlanes<KA>::value, LB = DigitPlanes<KB>::value;
    constexpr int RPW = 16 / NSPLIT;                    // accumulator registers a wave finishes in the epilogue

    __shared__ float sRed[NSPLIT > 1 ? NSPLIT : 1][NSPLIT > 1 ? 16 : 1][64];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 31, lh = lane >> 5;
    const int ks = NSPLIT > 1 ? wave : 0;               // K-split index of this wave

    // tile of this wave: with NSPLIT = 1 the block covers four consecutive tiles of the row-major tile grid
    const int tilesN = (p.N + 31) / 32, tilesM = (p.M + 31) / 32;
    const int tile = NSPLIT > 1 ? block : block * 4 + wave;
    const bool live = tile < tilesM * tilesN;           // trailing waves of the last block have no tile
    const int m0 = (tile / tilesN) * 32, n0 = (tile % tilesN) * 32;

    const int NSe = (((p.Kw + 1) >> 1) + 3) / 4 * 4;
    const int GT = NSe / 4;                             // groups of four steps in all; wave ks takes groups ks, ks + NSPLIT, ...
    const int G = (GT - ks + NSPLIT - 1) / NSPLIT;      // ... of which this wave has G (waves of a block may differ by one)

    Fp4Masks km;
    km.m1 = reg_const(0x11111111u); km.m2 = reg_const(0x22222222u);
    km.m4 = reg_const(0x44444444u); km.m8 = reg_const(0x88888888u);

    // this lane's operand rows
    const int gmA = m0 + lr, gnB = n0 + lr;
    const bool a_ok = live && gmA < p.M, b_ok = live && gnB < p.N;
    int a_h0 = 0, a_w0 = 0;
    int64_t a_pix = 0;
    if (CONV) {
        int wo, ho, n;
        conv_row_to_pixel(p, gmA, n, ho, wo);
        a_h0 = ho * p.stride - p.pad;
        a_w0 = wo * p.stride - p.pad;
        a_pix = static_cast<int64_t>(n) * p.H * p.W;
    }
    const uint32_t *b_row = p.B + static_cast<int64_t>(gnB) * p.PB * p.ldwB;
    const uint32_t *a_row = p.A + static_cast<int64_t>(gmA) * p.PA * p.ldwA;      // matrix mode

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
    auto load_b = [&](int plane, int kk) -> uint4 {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (!b_ok || kk >= p.Kw || plane >= p.PB) return v;
        const uint32_t *src = b_row + static_cast<int64_t>(plane) * p.ldwB + kk;
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

    // the epilogue's per-channel parameters and residual codes: their latency hides behind the main loop
    const int gn = n0 + lr;
    float sc = 0.0f, bi = 0.0f;
    if (p.scale && live && gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
    // (one load per wave and group of eight rows: lane l holds the word of row l & 7, plane l >> 3)
    constexpr int NG = RPW / 4;                         // groups of four registers = eight rows this wave finishes
    uint32_t pre_res[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g)
        pre_res[g] = (live && !p.pool) ? load_res_rows8(p, m0 + 8 * (NSPLIT > 1 ? ks : g), gn >> 5, lane) : 0u;

    // Digit pairs (da, db) and the groups of four steps of each are walked as one
    // flat sequence, GMAX entries at a time with all their loads in flight together,
    // so that a multi-digit layer (e.g. 8-bit features: four passes) pays one memory
    // round trip, not one per pass.  The weight 4^(da + db) of a pair (Eq. 1) enters
    // as the block scales of the matrix instruction, which makes the order free.
    const int total = p.Kw > 0 ? p.DA * p.DB * G : 0;
    const int kbase = lh * NSe + 4 * ks;                // first K word of this lane's first group; the next is 4 NSPLIT further

    v16f_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    if (p.DA * p.DB == 1) {                             // one digit pair (most layers): unit scales, plain group loop
        for (int g0 = 0; g0 < (p.Kw > 0 ? G : 0); g0 += GMAX) {
            uint4 wa[GMAX][LA], wb[GMAX][LB];
#pragma unroll
            for (int g = 0; g < GMAX; ++g) {
                const int kk = (g0 + g < G) ? kbase + 4 * NSPLIT * (g0 + g) : p.Kw;   // beyond G: reads as zero, not used
#pragma unroll
                for (int pl = 0; pl < LA; ++pl) wa[g][pl] = load_a(pl, kk);
#pragma unroll
                for (int pl = 0; pl < LB; ++pl) wb[g][pl] = load_b(pl, kk);
            }
#pragma unroll
            for (int g = 0; g < GMAX; ++g) {
                if (g0 + g < G) {
                    const uint32_t a0[4] = {wa[g][0].x, wa[g][0].y, wa[g][0].z, wa[g][0].w};
                    const uint32_t a1[4] = {wa[g][LA - 1].x, wa[g][LA - 1].y, wa[g][LA - 1].z, wa[g][LA - 1].w};
                    const uint32_t b0[4] = {wb[g][0].x, wb[g][0].y, wb[g][0].z, wb[g][0].w};
                    const uint32_t b1[4] = {wb[g][LB - 1].x, wb[g][LB - 1].y, wb[g][LB - 1].z, wb[g][LB - 1].w};
#pragma unroll
                    for (int st = 0; st < 4; ++st) {
                        v8i_t fa, fb;
                        expand_fp4<KA>(a0[st], a1[st], km, fa);
                        expand_fp4<KB>(b0[st], b1[st], km, fb);
                        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc, 4, 4, 0, 0x7f7f7f7f, 0,
                                                                               0x7f7f7f7f);
                    }
                }
            }
        }
    }
    int da = 0, db = 0, grp = 0;                        // position in the flat sequence (scalar counters, no divisions)
    for (int e0 = 0; e0 < (p.DA * p.DB == 1 ? 0 : total); e0 += GMAX) {
        uint4 wa[GMAX][LA], wb[GMAX][LB];
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
            for (int pl = 0; pl < LB; ++pl) wb[g][pl] = load_b(planeB + pl, kk);
            ++grp;                                      // next group, then next digit of B, then next digit of A
            const bool wg = grp == G;
            grp = wg ? 0 : grp;
            db += wg ? 1 : 0;
            const bool wd = db == p.DB;
            db = wd ? 0 : db;
            da += wd ? 1 : 0;
        }
#pragma unroll
        for (int g = 0; g < GMAX; ++g) {
            if (e0 + g < total) {
                const uint32_t a0[4] = {wa[g][0].x, wa[g][0].y, wa[g][0].z, wa[g][0].w};
                const uint32_t a1[4] = {wa[g][LA - 1].x, wa[g][LA - 1].y, wa[g][LA - 1].z, wa[g][LA - 1].w};
                const uint32_t b0[4] = {wb[g][0].x, wb[g][0].y, wb[g][0].z, wb[g][0].w};
                const uint32_t b1[4] = {wb[g][LB - 1].x, wb[g][LB - 1].y, wb[g][LB - 1].z, wb[g][LB - 1].w};
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    v8i_t fa, fb;
                    expand_fp4<KA>(a0[st], a1[st], km, fa);
                    expand_fp4<KB>(b0[st], b1[st], km, fb);
                    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc, 4, 4, 0, sa[g], 0, sb[g]);
                }
            }
        }
    }

    MfmaParams pq = p;                          // pooled outputs: a quarter of the rows, corrections per grid
    pq.M = p.M >> 2;
    pq.c0 = p.pool == 2 ? 4 * p.c0 : p.c0;
    if constexpr (NSPLIT == 1) {
        if (!live) return;                      // wave-uniform: the ballots below stay whole-wave
        if (p.pool) {                           // registers 4 k .. 4 k + 3 of a lane are one pooling grid
            static_for<4>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                finish_value(pq, pool4(p.pool, acc[4 * k], acc[4 * k + 1], acc[4 * k + 2], acc[4 * k + 3]),
                             (m0 + 8 * k + 4 * lh) >> 2, gn, sc, bi, false, 0u, lr, lh);
            });
            return;
        }
        static_for<4>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            const float v4[4] = {acc[4 * k], acc[4 * k + 1], acc[4 * k + 2], acc[4 * k + 3]};
            finish_rows8(p, v4, m0 + 8 * k, gn, sc, bi, pre_res[k], lane, lr, lh);
        });
    } else {
        // add the partial tiles; wave ks finishes accumulator registers RPW ks .. RPW ks + RPW - 1
#pragma unroll
        for (int r = 0; r < 16; ++r) sRed[ks][r][lane] = acc[r];
        __syncthreads();
        if (p.pool) {                           // RPW = 4: this wave's share of the tile is one pooling grid per lane
            static_assert(NSPLIT == 1 || RPW == 4, "a K-split wave finishes whole pooling grids");
            float v4[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                v4[rr] = 0.0f;
#pragma unroll
                for (int k = 0; k < NSPLIT; ++k) v4[rr] += sRed[k][ks * 4 + rr][lane];
            }
            finish_value(pq, pool4(p.pool, v4[0], v4[1], v4[2], v4[3]), (m0 + 8 * ks + 4 * lh) >> 2, gn, sc, bi, false, 0u, lr, lh);
            return;
        }
        static_assert(RPW == 4, "a K-split wave finishes one group of eight rows");
        float v4[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            v4[rr] = 0.0f;
#pragma unroll
            for (int k = 0; k < NSPLIT; ++k) v4[rr] += sRed[k][ks * 4 + rr][lane];
        }
        finish_rows8(p, v4, m0 + 8 * ks, gn, sc, bi, pre_res[0], lane, lr, lh);
    }
}

template <int KA, int KB, int VW, bool CONV, int NSPLIT, int GMAX = 5>
__global__ __launch_bounds__(256) void mfma_small_kernel(const MfmaParams p)
{
    mfma_small_body<KA, KB, VW, CONV, NSPLIT, GMAX>(p, blockIdx.x);
}

// Two independent convolution layers in one launch (K split over the four waves of a block): blocks
// 0 .. blocks0 - 1 work on the first, the others on the second.  A layer this small is mostly launch and
// drain, so two that do not depend on each other (the 3 x 3 convolution and the 1 x 1 shortcut convolution of a
// down-sampling residual block, Sec. 5.1) share both.
struct MfmaPairParams {
    MfmaParams p[2];
    int blocks0;
};

template <int KA, int KB, int VW, int GMAX>
__global__ __launch_bounds__(256) void mfma_small_pair_kernel(const MfmaPairParams pp)
{
    const int second = blockIdx.x >= pp.blocks0 ? 1 : 0;            // block-uniform
    mfma_small_body<KA, KB, VW, true, 4, GMAX>(pp.p[second], blockIdx.x - (second ? pp.blocks0 : 0));
}

}  // namespace apnn
