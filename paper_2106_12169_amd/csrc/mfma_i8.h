// Single-pass form of the arbitrary-precision product for operands of more than
// two bits, on the 8-bit integer matrix instruction (v_mfma_i32_32x32x32_i8).
//
// The bit planes of the ABI stay packed in HBM and in LDS.  Per lane and in
// registers, the plane words of 32 K positions are transposed into 32 bytes, each
// holding all the bits of one element (Eq. 2 read backwards: the decoded integer),
// and one matrix instruction multiplies 32 x 32 x 32 of them with int32
// accumulation.  Where the 1-bit emulation takes p q plane-pair passes and the
// two-plane FP4 form ceil(p/2) ceil(q/2) digit passes, this takes one; the paper
// observes the same about built-in 8-bit arithmetic once operands grow (Sec. 6.1.1).
// Results are the same integers (no range condition: the accumulator is int32, as
// Sec. 4.1 requires of the output).
//
// Encodings (Sec. 3.2).  The instruction multiplies signed bytes.
//   unsigned, up to 7 planes   the byte is the value.
//   unsigned, 8 planes         the top plane is inverted, which makes the byte
//                              value - 128; the product is put right with the row
//                              sums of the other operand (the J-term of Case III,
//                              with 128 in place of 1).
//   -1/+1                      the stored bit b enters as the byte b, and
//                              (2b - 1) x = 2 b x - x is recovered exactly as in
//                              Case III: twice the sum less the other operand's
//                              row sum.
// In general, with a = alphaA a' + oA and b = alphaB b' + oB (a', b' the bytes):
//   Y = alphaA alphaB sum(a' b') + alphaA oB sum(a') + alphaB oA sum(b') + K oA oB.
// The host folds this into Y = accmul acc + mulA RA[m] + mulB RB[n] + c0, RA and RB
// being the decoded row sums sum_s 2^s popc(plane s), which the lanes accumulate
// from the plane words they hold anyway (popcount, as in the AND+popcount kernel).
//
// Schedule.  Block tile (2 FM 32) x (2 FN 32), 2 x 2 waves, each FM x FN
// instruction tiles.  K advances in chunks of 4 words (128 positions = 4 instruction
// steps): global memory -> LDS directly, 16 bytes per lane (one plane row of the
// chunk), double buffered, the 16-byte pieces XOR-swizzled by row; lane half h of
// row r reads words 2h, 2h + 1 of every plane of its fragment rows (8-byte LDS
// reads), transposes them, and the two words give the bytes of steps (0, 1) and
// (2, 3).  The K order inside a step is free as long as both operands agree: dword j,
// byte g of a transposed word is the element at bit 8 g + j.
#pragma once
#include "mfma_big.h"

namespace apnn {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

// plane classes: how many planes the LDS rows and the transposition are built for
enum { I8_C2 = 0, I8_C4 = 1, I8_C8 = 2 };
template <int C> struct I8Slots { static constexpr int value = C == I8_C8 ? 8 : C == I8_C4 ? 4 : 2; };

// (a & m) | (b & ~m) in one instruction (truth table a:0xF0, b:0xCC, m:0xAA)
__device__ __forceinline__ uint32_t bit_select(uint32_t a, uint32_t b, uint32_t m)
{
    constexpr int SEL = (0xF0 & 0xAA) | (0xCC & 0x55);
    return __builtin_amdgcn_bitop3_b32(a, b, m, SEL);
}

struct I8Masks { uint32_t m0f, m33, m55, m03; };

// One stage of the bit-matrix transposition on the pair (lo, hi): the D-bit blocks selected by ~m of lo and
// by m of hi change places.
template <int D> __device__ __forceinline__ void swap_blocks(uint32_t &lo, uint32_t &hi, uint32_t m)
{
    const uint32_t a = lo, b = hi;
    lo = bit_select(a, b << D, m);
    hi = bit_select(a >> D, b, m);
}

// Plane words w[0 .. slots) of 32 K positions -> 8 dwords of 4 bytes: byte g of d[j] is the element at bit 8 g + j,
// i.e. sum_s 2^s bit(w[s], 8 g + j).
template <int C> __device__ __forceinline__ void planes_to_bytes(const uint32_t (&w)[I8Slots<C>::value], const I8Masks &k, uint32_t (&d)[8])
{
    if constexpr (C == I8_C8) {
        // 8 x 8 bit-matrix transposition (plane s, bit j of a byte) inside every byte column, three stages
        uint32_t x[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) x[s] = w[s];
#pragma unroll
        for (int s = 0; s < 4; ++s) swap_blocks<4>(x[s], x[s + 4], k.m0f);
#pragma unroll
        for (int s = 0; s < 8; ++s)
            if ((s & 2) == 0) swap_blocks<2>(x[s], x[s + 2], k.m33);
#pragma unroll
        for (int s = 0; s < 8; s += 2) swap_blocks<1>(x[s], x[s + 1], k.m55);
#pragma unroll
        for (int j = 0; j < 8; ++j) d[j] = x[j];
    } else if constexpr (C == I8_C4) {
        // 4 x 4 transposition inside every nibble: nibble n of x[i] becomes the value at position 4 n + i; then the
        // nibbles are spread over the bytes
        uint32_t x[4] = {w[0], w[1], w[2], w[3]};
        swap_blocks<2>(x[0], x[2], k.m33);
        swap_blocks<2>(x[1], x[3], k.m33);
        swap_blocks<1>(x[0], x[1], k.m55);
        swap_blocks<1>(x[2], x[3], k.m55);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            d[i] = x[i] & k.m0f;
            d[4 + i] = (x[i] >> 4) & k.m0f;
        }
    } else {
        // 2 x 2 transposition inside every bit pair: pair t of x0 is the value at position 2 t, of x1 at 2 t + 1
        uint32_t x0 = w[0], x1 = w[1];
        swap_blocks<1>(x0, x1, k.m55);
        d[0] = x0 & k.m03;
        d[1] = x1 & k.m03;
        d[2] = (x0 >> 2) & k.m03;
        d[3] = (x1 >> 2) & k.m03;
        d[4] = (x0 >> 4) & k.m03;
        d[5] = (x1 >> 4) & k.m03;
        d[6] = (x0 >> 6) & k.m03;
        d[7] = (x1 >> 6) & k.m03;
    }
}

template <int CA, int CB, int FM, int FN>
__global__ __launch_bounds__(256, FM * FN >= 16 ? 1 : 2) void mfma_i8_kernel(const MfmaParams p)
{
    constexpr int SA = I8Slots<CA>::value, SB = I8Slots<CB>::value;     // 16-byte pieces (one per plane) of an LDS row
    constexpr int BM = 2 * FM * 32, BN = 2 * FN * 32;
    constexpr int NA = BM * SA / 256, NB = BN * SB / 256;               // load instructions per wave and chunk
    static_assert(BM * SA % 256 == 0 && BN * SB % 256 == 0, "every wave issues the same number of loads");
    constexpr int A_WORDS = BM * SA * 4, B_WORDS = BN * SB * 4;
    __shared__ __attribute__((aligned(1024))) uint32_t smem[2 * (A_WORDS + B_WORDS)];    // A 0, A 1, B 0, B 1
    typedef __attribute__((address_space(3))) uint32_t *lds_ptr_t;
    const uint32_t smem_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)smem));

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lh = lane >> 5;

    const int tilesN = (p.N + BN - 1) / BN;
    int tile = blockIdx.x;
    if (p.xcd_regions) {                                // one rectangular region of tiles per XCD (see mfma_big_kernel)
        const int tilesM = (p.M + BM - 1) / BM;
        const int rw = tilesN >> 2, rh = tilesM >> 1, xcd = tile & 7, idx = tile >> 3;
        tile = ((xcd >> 2) * rh + idx / rw) * tilesN + (xcd & 3) * rw + idx % rw;
    }
    const int m0 = (tile / tilesN) * BM, n0 = (tile % tilesN) * BN;

    I8Masks km;
    km.m0f = reg_const(0x0F0F0F0Fu); km.m33 = reg_const(0x33333333u);
    km.m55 = reg_const(0x55555555u); km.m03 = reg_const(0x03030303u);

    // ---- loader.  A wave-wide load deposits 64 pieces contiguously, i.e. 64 / S whole rows of S pieces; the
    // piece in slot c of row r is plane c ^ swz(r), so that the 8-byte reads of consecutive rows spread over the
    // banks.  A plane that does not exist, or a chunk beyond K, is sent out of the descriptor's range: zeros.
    auto swz = [](int r, int S) { return S == 8 ? (r & 7) : S == 4 ? ((r >> 1) & 3) : ((r >> 2) & 1); };
    const uint32_t bytesA = 4u * static_cast<uint32_t>(p.M) * p.PA * p.ldwA, bytesB = 4u * static_cast<uint32_t>(p.N) * p.PB * p.ldwB;
    const v4u_t descA = make_raw_desc(p.A, bytesA), descB = make_raw_desc(p.B, bytesB);
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;      // operands are smaller than 2 GiB (host check)
    uint32_t offA[NA], offB[NB];
#pragma unroll
    for (int u = 0; u < NA; ++u) {
        const int L = 64 * (wave * NA + u) + lane, row = L / SA, plane = (L % SA) ^ swz(row, SA);
        offA[u] = 4u * ((static_cast<uint32_t>(min(m0 + row, p.M - 1)) * p.PA + plane) * p.ldwA) | (plane < p.PA ? 0u : OUT_OF_RANGE);
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int L = 64 * (wave * NB + u) + lane, row = L / SB, plane = (L % SB) ^ swz(row, SB);
        offB[u] = 4u * ((static_cast<uint32_t>(min(n0 + row, p.N - 1)) * p.PB + plane) * p.ldwB) | (plane < p.PB ? 0u : OUT_OF_RANGE);
    }
    auto fetch = [&](int kc, int buf) {                 // chunk kc -> buffer buf
        const uint32_t dead = 4 * kc < p.Kw ? 0u : OUT_OF_RANGE;
        const int soff = __builtin_amdgcn_readfirstlane(16 * kc);
        // (the LDS addresses are wave-uniform; saying so keeps them in scalar registers)
        const uint32_t ldsA = __builtin_amdgcn_readfirstlane(smem_base + 4 * (buf * A_WORDS + wave * NA * 256));
        const uint32_t ldsB = __builtin_amdgcn_readfirstlane(smem_base + 4 * (2 * A_WORDS + buf * B_WORDS + wave * NB * 256));
#pragma unroll
        for (int u = 0; u < NA; ++u) load_to_lds_16(descA, ldsA + 1024 * u, offA[u] | dead, soff);
#pragma unroll
        for (int u = 0; u < NB; ++u) load_to_lds_16(descB, ldsB + 1024 * u, offB[u] | dead, soff);
    };
    constexpr int NLOAD = NA + NB;
    constexpr int WAIT_PREVIOUS = 0x0F70 | (NLOAD & 0xF) | ((NLOAD >> 4) << 14);   // s_waitcnt vmcnt(NLOAD): all but the newest chunk
    constexpr int WAIT_ALL = 0x0F70;

    // ---- reader: word offsets of (fragment row 0, plane s) of this lane; fragment f is 32 rows further
    int rdA[SA], rdB[SB];
#pragma unroll
    for (int s = 0; s < SA; ++s) rdA[s] = ((wm * FM * 32 + lr) * SA + (s ^ swz(lr, SA))) * 4 + 2 * lh;
#pragma unroll
    for (int s = 0; s < SB; ++s) rdB[s] = 2 * A_WORDS + ((wn * FN * 32 + lr) * SB + (s ^ swz(lr, SB))) * 4 + 2 * lh;

    v16i_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    uint32_t ra[FM], rb[FN];                            // decoded row sums of this lane's words (Sec. 3.2 Case III: J X)
#pragma unroll
    for (int i = 0; i < FM; ++i) ra[i] = 0;
#pragma unroll
    for (int j = 0; j < FN; ++j) rb[j] = 0;
    const bool need_ra = p.mulA != 0, need_rb = p.mulB != 0;

    fetch(0, 0);
    fetch(1, 1);
    __builtin_amdgcn_s_waitcnt(WAIT_PREVIOUS);
    __syncthreads();

    for (int it = 0; it < p.nk; ++it) {
        const int buf = it & 1;
        uint2 wa[FM][SA], wb[FN][SB];
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int s = 0; s < SA; ++s)
                wa[f][s] = *reinterpret_cast<const uint2 *>(&smem[buf * A_WORDS + rdA[s] + f * 32 * SA * 4]);
#pragma unroll
        for (int f = 0; f < FN; ++f)
#pragma unroll
            for (int s = 0; s < SB; ++s)
                wb[f][s] = *reinterpret_cast<const uint2 *>(&smem[buf * B_WORDS + rdB[s] + f * 32 * SB * 4]);
        if (CA == I8_C8) {                              // an 8-bit operand enters as value - 128: top plane inverted
#pragma unroll
            for (int f = 0; f < FM; ++f) { wa[f][SA - 1].x ^= p.flipA; wa[f][SA - 1].y ^= p.flipA; }
        }
        if (CB == I8_C8) {
#pragma unroll
            for (int f = 0; f < FN; ++f) { wb[f][SB - 1].x ^= p.flipB; wb[f][SB - 1].y ^= p.flipB; }
        }
        __syncthreads();                                // every wave has read buffer buf: it can take chunk it + 2
        fetch(it + 2, buf);
        if (need_ra) {
#pragma unroll
            for (int f = 0; f < FM; ++f)
#pragma unroll
                for (int s = 0; s < SA; ++s) {
                    const uint32_t fl = (CA == I8_C8 && s == SA - 1) ? p.flipA : 0u;
                    ra[f] += static_cast<uint32_t>(__popc(wa[f][s].x ^ fl) + __popc(wa[f][s].y ^ fl)) << s;
                }
        }
        if (need_rb) {
#pragma unroll
            for (int f = 0; f < FN; ++f)
#pragma unroll
                for (int s = 0; s < SB; ++s) {
                    const uint32_t fl = (CB == I8_C8 && s == SB - 1) ? p.flipB : 0u;
                    rb[f] += static_cast<uint32_t>(__popc(wb[f][s].x ^ fl) + __popc(wb[f][s].y ^ fl)) << s;
                }
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {                   // word e of the lane's two: instruction steps 2 e, 2 e + 1
            uint32_t da[FM][8], db[FN][8];
#pragma unroll
            for (int f = 0; f < FM; ++f) {
                uint32_t w[SA];
#pragma unroll
                for (int s = 0; s < SA; ++s) w[s] = e ? wa[f][s].y : wa[f][s].x;
                planes_to_bytes<CA>(w, km, da[f]);
            }
#pragma unroll
            for (int f = 0; f < FN; ++f) {
                uint32_t w[SB];
#pragma unroll
                for (int s = 0; s < SB; ++s) w[s] = e ? wb[f][s].y : wb[f][s].x;
                planes_to_bytes<CB>(w, km, db[f]);
            }
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    const v4i_t a = {static_cast<int>(da[i][4 * h]), static_cast<int>(da[i][4 * h + 1]),
                                     static_cast<int>(da[i][4 * h + 2]), static_cast<int>(da[i][4 * h + 3])};
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const v4i_t b = {static_cast<int>(db[j][4 * h]), static_cast<int>(db[j][4 * h + 1]),
                                         static_cast<int>(db[j][4 * h + 2]), static_cast<int>(db[j][4 * h + 3])};
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i][j], 0, 0, 0);
                    }
                }
        }
        __builtin_amdgcn_s_waitcnt(WAIT_PREVIOUS);      // chunk it + 1 has landed (chunk it + 2 may still fly)
        __syncthreads();
    }
    __builtin_amdgcn_s_waitcnt(WAIT_ALL);               // the loads issued for chunks beyond the last one have landed

    // ---- encoding recovery (Sec. 3.2): Y = accmul acc + mulA RA[row] + mulB RB[column] + c0, in wrapping 32-bit
    // arithmetic (the result fits int32, the host checks K (2^p - 1)(2^q - 1) < 2^31).
    // The two lane halves hold the sums of different words of the same row.
#pragma unroll
    for (int i = 0; i < FM; ++i) ra[i] = (ra[i] + static_cast<uint32_t>(__shfl_xor(static_cast<int>(ra[i]), 32))) * static_cast<uint32_t>(p.mulA);
#pragma unroll
    for (int j = 0; j < FN; ++j)
        rb[j] = (rb[j] + static_cast<uint32_t>(__shfl_xor(static_cast<int>(rb[j]), 32))) * static_cast<uint32_t>(p.mulB) + static_cast<uint32_t>(p.c0);
    // accumulator register r of lane (lh, lr) is row 8 (r / 4) + 4 lh + r % 4, column lr
    static_for<FM>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        static_for<16>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
            const uint32_t rowterm = need_ra ? static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(4 * row, static_cast<int>(ra[i]))) : 0u;
            static_for<FN>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                acc[i][j][r] = static_cast<int>(static_cast<uint32_t>(acc[i][j][r]) * static_cast<uint32_t>(p.accmul) + rowterm + rb[j]);
            });
        });
    });

    if (p.Y) {
        // int32 output straight from the accumulators: one store instruction writes two 128-byte row segments.
        // The whole byte offset travels in the per-lane offset, which the hardware checks against M x N.
        const __amdgpu_buffer_rsrc_t rsrcY =
            __builtin_amdgcn_make_buffer_rsrc(p.Y, 0, 4u * static_cast<uint32_t>(p.M) * p.N, 0x00020000);
        const int gn0 = n0 + wn * FN * 32 + lr;
        const uint32_t vbase = 4u * (static_cast<uint32_t>(m0 + wm * FM * 32 + 4 * lh) * p.N + gn0);
        static_for<FM * FN * 16>([&](auto c) {
            constexpr int i = decltype(c)::value / (FN * 16), j = decltype(c)::value / 16 % FN, r = decltype(c)::value % 16;
            constexpr int row = i * 32 + 8 * (r >> 2) + (r & 3);
            const uint32_t voff = (vbase + 128u * j) | (gn0 + 32 * j < p.N ? 0u : OUT_OF_RANGE);
            __builtin_amdgcn_raw_buffer_store_b32(acc[i][j][r], rsrcY, voff + 4u * row * static_cast<uint32_t>(p.N), 0, 0);
        });
    }
    if (!p.scale) return;
    MfmaParams pe = p;                                  // the shared epilogue sees finished integers
    pe.out_scale = 1.0f; pe.c0 = 0; pe.Y = nullptr;
    static_for<FN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int gn = n0 + wn * FN * 32 + j * 32 + lr;
        float sc = 0.0f, bi = 0.0f;
        if (gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
        static_for<FM * 4>([&](auto ikc) {
            constexpr int i = decltype(ikc)::value / 4, k = decltype(ikc)::value % 4;
            const int row0 = m0 + wm * FM * 32 + i * 32 + 8 * k;
            const float v4[4] = {static_cast<float>(acc[i][j][4 * k]), static_cast<float>(acc[i][j][4 * k + 1]),
                                 static_cast<float>(acc[i][j][4 * k + 2]), static_cast<float>(acc[i][j][4 * k + 3])};
            finish_rows8(pe, v4, row0, gn, sc, bi, load_res_rows8(pe, row0, gn >> 5, lane), lane, lr, lh);
        });
    });
}

}  // namespace apnn
