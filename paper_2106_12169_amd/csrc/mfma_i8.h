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
// instruction tiles, one wave per SIMD.  K advances in chunks of 4 words (128
// positions = 4 instruction steps) and is fetched in groups of two or four chunks
// (32 or 64 bytes of every plane row): global memory -> LDS directly, 16 bytes per
// lane, adjacent lanes taking adjacent pieces of one plane row, two group buffers,
// one barrier per group, the 16-byte pieces XOR-swizzled by row; lane half h of row r reads words 2h,
// 2h + 1 of every plane of its fragment rows (8-byte LDS reads) one chunk ahead, and
// each word, transposed, gives the bytes of two instruction steps.  The kernel is
// bound by the vector instructions of the transposition (about 20 per matrix
// instruction), so the matrix instructions of one word are issued between the pieces
// of the next word's transposition and run underneath them.  The K order inside a
// step is free as long as both operands agree: dword j, byte g of a transposed word
// is the element at bit 8 g + j.
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

// One stage of a bit-matrix transposition on two pairs (a0, b0), (a1, b1): the D-bit blocks selected by ~m of a and
// by m of b change places.  The two left shifts and the two right shifts are each one 64-bit shift of a register
// pair (issued at the rate of a 32-bit one); the bits that cross between the halves land where m drops them.
template <int D> __device__ __forceinline__ void swap_blocks2(uint32_t &a0, uint32_t &b0, uint32_t &a1, uint32_t &b1, uint32_t m)
{
    const uint64_t up = pair_shl<D>(make_pair(b0, b1)), down = pair_shr<D>(make_pair(a0, a1));
    const uint32_t na0 = bit_select(a0, half_of<0>(up), m), na1 = bit_select(a1, half_of<1>(up), m);
    b0 = bit_select(half_of<0>(down), b0, m);
    b1 = bit_select(half_of<1>(down), b1, m);
    a0 = na0;
    a1 = na1;
}

// Plane words w[0 .. slots) of 32 K positions -> 8 dwords of 4 bytes: byte g of d[j] is the element at bit 8 g + j,
// i.e. sum_s 2^s bit(w[s], 8 g + j).  Two parts, so that matrix instructions can be issued in between; x carries
// the state from part 0 to part 1.
template <int C, int PART>
__device__ __forceinline__ void planes_to_bytes(const uint32_t (&w)[I8Slots<C>::value], const I8Masks &k, uint32_t (&x)[8], uint32_t (&d)[8])
{
    if constexpr (C == I8_C8) {
        // 8 x 8 bit-matrix transposition (plane s, bit j of a byte) inside every byte column, three stages
        if constexpr (PART == 0) {
#pragma unroll
            for (int s = 0; s < 8; ++s) x[s] = w[s];
            swap_blocks2<4>(x[0], x[4], x[1], x[5], k.m0f);
            swap_blocks2<4>(x[2], x[6], x[3], x[7], k.m0f);
            swap_blocks2<2>(x[0], x[2], x[1], x[3], k.m33);
        } else {
            swap_blocks2<2>(x[4], x[6], x[5], x[7], k.m33);
            swap_blocks2<1>(x[0], x[1], x[2], x[3], k.m55);
            swap_blocks2<1>(x[4], x[5], x[6], x[7], k.m55);
#pragma unroll
            for (int j = 0; j < 8; ++j) d[j] = x[j];
        }
    } else if constexpr (C == I8_C4) {
        // 4 x 4 transposition inside every nibble: nibble n of x[i] becomes the value at position 4 n + i; then the
        // nibbles are spread over the bytes
        if constexpr (PART == 0) {
            x[0] = w[0]; x[1] = w[1]; x[2] = w[2]; x[3] = w[3];
            swap_blocks2<2>(x[0], x[2], x[1], x[3], k.m33);
            swap_blocks2<1>(x[0], x[1], x[2], x[3], k.m55);
        } else {
            const uint64_t h01 = pair_shr<4>(make_pair(x[0], x[1])), h23 = pair_shr<4>(make_pair(x[2], x[3]));
#pragma unroll
            for (int i = 0; i < 4; ++i) d[i] = x[i] & k.m0f;
            d[4] = half_of<0>(h01) & k.m0f;
            d[5] = half_of<1>(h01) & k.m0f;
            d[6] = half_of<0>(h23) & k.m0f;
            d[7] = half_of<1>(h23) & k.m0f;
        }
    } else {
        // 2 x 2 transposition inside every bit pair: pair t of x0 is the value at position 2 t, of x1 at 2 t + 1
        if constexpr (PART == 0) {
            const uint32_t a = w[0], b = w[1];
            x[0] = bit_select(a, b << 1, k.m55);
            x[1] = bit_select(a >> 1, b, k.m55);
            const uint64_t h = pair_shr<2>(make_pair(x[0], x[1]));
            d[0] = x[0] & k.m03;
            d[1] = x[1] & k.m03;
            d[2] = half_of<0>(h) & k.m03;
            d[3] = half_of<1>(h) & k.m03;
        } else {
            const uint64_t h4 = pair_shr<4>(make_pair(x[0], x[1])), h6 = pair_shr<6>(make_pair(x[0], x[1]));
            d[4] = half_of<0>(h4) & k.m03;
            d[5] = half_of<1>(h4) & k.m03;
            d[6] = half_of<0>(h6) & k.m03;
            d[7] = half_of<1>(h6) & k.m03;
        }
    }
}

// Bytes of LDS the kernel needs for PA + PB planes: two group buffers; with K split over wave pairs, room for the
// exchange of half of every wave's accumulators (35 registers of 64 lanes for each of 8 waves).
constexpr int mfma_i8_lds_bytes(int PA, int PB, int G, int NKS)
{
    const int tiles = 2 * (PA + PB) * 128 * G * 16, exchange = NKS == 2 ? 8 * 35 * 256 : 0;
    return tiles > exchange ? tiles : exchange;
}

// NKS = 2: eight waves, two per SIMD; the two waves of a pair own the same 64 x 64 outputs and take alternate
// chunks of K, and add their halves through LDS at the end.  A lone wave issues a vector instruction only every
// six cycles or so (measured; two waves together reach one per four), and this kernel is bound by them.
template <int CA, int CB, int FM, int FN, int G, int NKS>
__global__ __launch_bounds__(256 * NKS, 1) void mfma_i8_kernel(const MfmaParams p)
{
    static_assert(G == 2 || G == 4, "a group is two or four chunks");
    static_assert(NKS == 1 || NKS == 2, "K is split over at most two waves");
    static_assert(FM == 2 && FN == 2, "128 x 128 block tile");
    constexpr int SA = I8Slots<CA>::value, SB = I8Slots<CB>::value;     // most planes of the class: width of the transposition
    constexpr int BM = 2 * FM * 32, BN = 2 * FN * 32;
    constexpr int NW = 4 * NKS;                         // waves
    constexpr int RB = 64 / G;                          // rows one load instruction covers (G pieces each)
    constexpr int NBR = BM / RB;                        // row blocks (load instructions) per plane
    constexpr int CPW = G / NKS;                        // chunks of a group that one wave multiplies
    // A group buffer holds, for G chunks: A planes [PA][BM rows][G pieces of 16 bytes], then B planes [PB][BN][G].
    extern __shared__ __attribute__((aligned(1024))) uint32_t smem[];
    typedef __attribute__((address_space(3))) uint32_t *lds_ptr_t;
    const uint32_t smem_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)smem));
    const int a_bytes = p.PA * BM * G * 16, buf_bytes = a_bytes + p.PB * BN * G * 16;
    // Plane counts for the "does this plane exist" tests around loads and reads.  Kept opaque (see fresh_counts) so
    // that every test is a scalar compare where it stands; hoisted out of the loop, the two dozen tests lived as lane
    // masks in scalar register pairs, which spilled.
    int n_pa = p.PA, n_pb = p.PB;
    auto fresh_counts = [&]() __attribute__((always_inline)) { asm volatile("" : "+s"(n_pa), "+s"(n_pb)); };

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pair = wave & 3, ks = wave >> 2;          // position in the 2 x 2 arrangement of wave tiles, K share
    const int wm = pair >> 1, wn = pair & 1;
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

    // ---- loader.  One load instruction moves the G pieces of RB consecutive rows of one plane: lanes G r' .. G r' +
    // G - 1 fetch consecutive 16-byte pieces of one plane row, i.e. of one cache line (a first version had every lane
    // in a line of its own and was bound by the tag look-ups of the first-level cache).  Piece j of row r' lands in
    // slot j ^ swz(r') of the row, so that the reads of 8 consecutive rows spread over all banks.  The per-lane part
    // of the byte offset is the same for every instruction; the rest (plane, row block, group) is wave-uniform and
    // added on, and the whole sum is what the hardware checks against the operand's size: rows beyond M read zeros.
    // The (plane, row block) pairs of an operand are dealt to the waves in turn.
    auto swz = [](int r) { return G == 4 ? ((r >> 1) & 3) : ((r >> 2) & 1); };
    const uint32_t bytesA = 4u * static_cast<uint32_t>(p.M) * p.PA * p.ldwA, bytesB = 4u * static_cast<uint32_t>(p.N) * p.PB * p.ldwB;
    const v4u_t descA = make_raw_desc(p.A, bytesA), descB = make_raw_desc(p.B, bytesB);
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;      // operands are smaller than 2 GiB (host check)
    const int ld_row = lane / G, ld_piece = (lane % G) ^ swz(ld_row);
    const uint32_t lane_offA = 4u * static_cast<uint32_t>(m0 + ld_row) * p.PA * p.ldwA + 16u * ld_piece;
    const uint32_t lane_offB = 4u * static_cast<uint32_t>(n0 + ld_row) * p.PB * p.ldwB + 16u * ld_piece;
    // state of the group being requested: per-lane offsets (out of range where its piece lies beyond K), buffer
    uint32_t gl_offA = 0, gl_offB = 0;
    uint32_t gl_lds = 0;
    int gl_k = 0;
    auto begin_group = [&](int group, uint32_t lds_bytes_base) __attribute__((always_inline)) {
        const uint32_t dead = 4 * (group * G + ld_piece) < p.Kw ? 0u : OUT_OF_RANGE;
        gl_offA = lane_offA | dead;
        gl_offB = lane_offB | dead;
        gl_lds = lds_bytes_base;
        gl_k = __builtin_amdgcn_readfirstlane(group * G * 16);
    };
    // load instruction d of this wave for the group: (plane, row block) number wave + NW d of A, then of B;
    // skipped for planes that do not exist
    constexpr int NDA = (SA * NBR + NW - 1) / NW, NDB = (SB * NBR + NW - 1) / NW, NLOAD = NDA + NDB;
    auto uniform_desc = [](v4u_t d) __attribute__((always_inline)) {     // (wave-uniform by construction; saying so at the point of use
        v4u_t r;                                        // keeps the four words in scalar registers for the instruction)
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_readfirstlane(d[i]);
        return r;
    };
    auto load_one = [&](auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        if constexpr (d < NDA) {
            const int n = wave + NW * d, s = n / NBR, b = n % NBR;
            if (s < n_pa) {
                const uint32_t uni = 4u * static_cast<uint32_t>(b * RB * p.PA + s) * p.ldwA + gl_k;
                load_to_lds_16(uniform_desc(descA), __builtin_amdgcn_readfirstlane(gl_lds + n * 1024), gl_offA + uni, 0);
            }
        } else {
            const int n = wave + NW * (d - NDA), s = n / NBR, b = n % NBR;
            if (s < n_pb) {
                const uint32_t uni = 4u * static_cast<uint32_t>(b * RB * p.PB + s) * p.ldwB + gl_k;
                load_to_lds_16(uniform_desc(descB), __builtin_amdgcn_readfirstlane(gl_lds + a_bytes + n * 1024), gl_offB + uni, 0);
            }
        }
    };
    constexpr int WAIT_LOADS = 0x0F70;                  // s_waitcnt vmcnt(0) (expcnt, lgkmcnt untouched)

    // ---- reader.  Lane (half h, row r) reads words 2h, 2h + 1 of chunk j of plane s of fragment row f at byte
    //   buffer + ((s BM + tile row) G + (j ^ swz(r))) 16 + 8 h;
    // the per-lane part (one register for each of this wave's chunks of a group, rebuilt when the buffer changes)
    // plus a constant that fits the instruction's offset field.  This wave's chunks of a group: ks, ks + NKS, ...
    uint32_t rd0A[CPW], rd0B[CPW], rdA[CPW], rdB[CPW];
#pragma unroll
    for (int t = 0; t < CPW; ++t) {
        const int j = t * NKS + ks;
        rd0A[t] = ((wm * FM * 32 + lr) * G + (j ^ swz(lr & (RB - 1)))) * 16 + 8 * lh;
        rd0B[t] = a_bytes + ((wn * FN * 32 + lr) * G + (j ^ swz(lr & (RB - 1)))) * 16 + 8 * lh;
    }
    auto set_read_buffer = [&](uint32_t byte_base) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < CPW; ++t) { rdA[t] = rd0A[t] + byte_base; rdB[t] = rd0B[t] + byte_base; }
    };
    struct Words { uint2 a[FM][SA], b[FN][SB]; };       // this lane's two words of every plane of its fragment rows
    constexpr int NREAD = FM * SA + FN * SB;
    // read r of this wave's chunk t of the group: (fragment, plane) of A, then of B; words of planes that do not
    // exist stay zero
    auto read_one = [&](auto tc, auto rc, Words &w) __attribute__((always_inline)) {
        constexpr int t = decltype(tc)::value, r = decltype(rc)::value;
        const char *lds = reinterpret_cast<const char *>(smem);
        if constexpr (r < FM * SA) {
            constexpr int f = r / SA, s = r % SA;
            if (s < n_pa) w.a[f][s] = *reinterpret_cast<const uint2 *>(lds + rdA[t] + (s * BM + 32 * f) * G * 16);
        } else {
            constexpr int f = (r - FM * SA) / SB, s = (r - FM * SA) % SB;
            if (s < n_pb) w.b[f][s] = *reinterpret_cast<const uint2 *>(lds + rdB[t] + (s * BN + 32 * f) * G * 16);
        }
    };

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
    auto row_sums = [&](const Words &w) __attribute__((always_inline)) {      // (before the top plane of an 8-bit operand is inverted)
        if (need_ra) {
#pragma unroll
            for (int f = 0; f < FM; ++f)
#pragma unroll
                for (int s = 0; s < SA; ++s) ra[f] += static_cast<uint32_t>(__popc(w.a[f][s].x) + __popc(w.a[f][s].y)) << s;
        }
        if (need_rb) {
#pragma unroll
            for (int f = 0; f < FN; ++f)
#pragma unroll
                for (int s = 0; s < SB; ++s) rb[f] += static_cast<uint32_t>(__popc(w.b[f][s].x) + __popc(w.b[f][s].y)) << s;
        }
    };
    struct Bytes { uint32_t a[FM][8], b[FN][8]; };      // the bytes of two instruction steps (dwords 0-3, 4-7) per fragment

    // One phase: the 2 FM FN matrix instructions of one word (bytes `cur`), each followed by its share of the
    // transposition of word E of `wsrc` into `nxt` (cut into 2 (FM + FN) pieces) and by whatever memory
    // instructions `hook` deals to that slot.  A wave issues in order: loads and LDS reads issued in a burst
    // held up the vector instructions behind them, spread out like this they run underneath.
    constexpr int NMI = 2 * FM * FN, NPART = 2 * (FM + FN);
    auto phase = [&](const Bytes &cur, const Words &wsrc, auto enc, Bytes &nxt, auto &&hook) __attribute__((always_inline)) {
        constexpr int E = decltype(enc)::value;
        uint32_t x[8];
        auto part = [&](auto pc) __attribute__((always_inline)) {
            constexpr int pi = decltype(pc)::value, f = pi / 2, half = pi % 2;
            if constexpr (f < FM) {
                uint32_t w[SA];
#pragma unroll
                for (int s = 0; s < SA; ++s) w[s] = E ? wsrc.a[f][s].y : wsrc.a[f][s].x;
                if (CA == I8_C8 && half == 0) w[SA - 1] ^= p.flipA;       // an 8-bit operand enters as value - 128
                planes_to_bytes<CA, half>(w, km, x, nxt.a[f]);
            } else {
                constexpr int g = f - FM;
                uint32_t w[SB];
#pragma unroll
                for (int s = 0; s < SB; ++s) w[s] = E ? wsrc.b[g][s].y : wsrc.b[g][s].x;
                if (CB == I8_C8 && half == 0) w[SB - 1] ^= p.flipB;
                planes_to_bytes<CB, half>(w, km, x, nxt.b[g]);
            }
        };
        static_for<NMI>([&](auto qc) {
            constexpr int q = decltype(qc)::value, h = q / (FM * FN), i = q / FN % FM, j = q % FN;
            const v4i_t a = {static_cast<int>(cur.a[i][4 * h]), static_cast<int>(cur.a[i][4 * h + 1]),
                             static_cast<int>(cur.a[i][4 * h + 2]), static_cast<int>(cur.a[i][4 * h + 3])};
            const v4i_t b = {static_cast<int>(cur.b[j][4 * h]), static_cast<int>(cur.b[j][4 * h + 1]),
                             static_cast<int>(cur.b[j][4 * h + 2]), static_cast<int>(cur.b[j][4 * h + 3])};
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i][j], 0, 0, 0);
            static_for<NPART *(q + 1) / NMI - NPART * q / NMI>([&](auto tc) {
                part(std::integral_constant<int, NPART * q / NMI + decltype(tc)::value>{});
            });
            hook(qc);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using E0 = std::integral_constant<int, 0>;
    using E1 = std::integral_constant<int, 1>;

    // Group g (chunks G g .. G g + G - 1) lives in buffer g mod 2.  A wave's half-iteration multiplies one of its
    // chunks while it reads the words of its next chunk and transposes the second word of the one and the first of
    // the other.  In its last half-iteration of group g: group g + 1 has landed (wait, barrier -- the only ones of the
    // group), the reads move over to its buffer, and group g + 2 is requested into the buffer of group g, whose words
    // every wave has in registers by then; it is needed a whole group later.  Chunks beyond the last are zeros.
    Words w0, w1;
    Bytes by0, by1;
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int s = 0; s < SA; ++s) w0.a[f][s] = w1.a[f][s] = make_uint2(0u, 0u);
#pragma unroll
    for (int f = 0; f < FN; ++f)
#pragma unroll
        for (int s = 0; s < SB; ++s) w0.b[f][s] = w1.b[f][s] = make_uint2(0u, 0u);
    begin_group(0, smem_base);
    static_for<NLOAD>([&](auto dc) { load_one(dc); });
    begin_group(1, smem_base + buf_bytes);
    static_for<NLOAD>([&](auto dc) { load_one(dc); });
    __builtin_amdgcn_s_waitcnt(WAIT_LOADS);
    __syncthreads();
    uint32_t cur_base = 0;                              // byte offset of the buffer the reads come from
    set_read_buffer(cur_base);
    static_for<NREAD>([&](auto rc) { read_one(E0{}, rc, w0); });
    auto no_hook = [](auto) {};
    {
        Bytes dummy;                                    // (the matrix instructions of this warm-up phase multiply zeros into zero accumulators)
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int d = 0; d < 8; ++d) dummy.a[f][d] = 0;
#pragma unroll
        for (int f = 0; f < FN; ++f)
#pragma unroll
            for (int d = 0; d < 8; ++d) dummy.b[f][d] = 0;
        row_sums(w0);
        phase(dummy, w0, E0{}, by0, no_hook);
    }
    int group = 0;                                      // group of the chunk being multiplied
    auto half_iteration = [&](auto tc, Words &wc, Words &wn_) __attribute__((always_inline)) {
        constexpr int t = decltype(tc)::value, tn = (t + 1) % CPW;     // this wave's chunk of the group being multiplied / read
        constexpr bool LAST = t == CPW - 1;
        fresh_counts();
        if constexpr (LAST) {
            __builtin_amdgcn_s_waitcnt(WAIT_LOADS);     // this wave's share of group + 1 is in LDS
            __syncthreads();
            begin_group(group + 2, smem_base + cur_base);
            cur_base = cur_base ? 0u : static_cast<uint32_t>(buf_bytes);
            set_read_buffer(cur_base);
            ++group;
        }
        // first phase: the reads of the next chunk, and this wave's loads of the group (as early as the buffer is free)
        phase(by0, wc, E1{}, by1, [&](auto qc) {
            constexpr int q = decltype(qc)::value;
            static_for<NREAD *(q + 1) / NMI - NREAD * q / NMI>([&](auto ic) {
                read_one(std::integral_constant<int, tn>{}, std::integral_constant<int, NREAD * q / NMI + decltype(ic)::value>{}, wn_);
            });
            if constexpr (LAST)
                static_for<NLOAD *(q + 1) / NMI - NLOAD * q / NMI>([&](auto ic) {
                    load_one(std::integral_constant<int, NLOAD * q / NMI + decltype(ic)::value>{});
                });
        });
        row_sums(wn_);
        phase(by1, wn_, E0{}, by0, no_hook);
    };
    // (the host makes nk a multiple of 4: whole groups, and an even number of chunks for every wave)
    constexpr int UNROLL = CPW % 2 == 0 ? CPW : 2 * CPW;
    for (int u = 0; u < p.nk / NKS; u += UNROLL) {
        static_for<UNROLL / 2>([&](auto vc) {
            constexpr int v = decltype(vc)::value;
            half_iteration(std::integral_constant<int, (2 * v) % CPW>{}, w0, w1);
            half_iteration(std::integral_constant<int, (2 * v + 1) % CPW>{}, w1, w0);
        });
    }
    __builtin_amdgcn_s_waitcnt(WAIT_LOADS);             // the loads requested for groups beyond the last one have landed

    // The two lane halves hold the row sums of different words of the same row.
#pragma unroll
    for (int i = 0; i < FM; ++i) ra[i] += static_cast<uint32_t>(__shfl_xor(static_cast<int>(ra[i]), 32));
#pragma unroll
    for (int j = 0; j < FN; ++j) rb[j] += static_cast<uint32_t>(__shfl_xor(static_cast<int>(rb[j]), 32));

    // ---- one row of wave tiles (32 rows x FN tiles): encoding recovery (Sec. 3.2) and the outputs.
    //   Y = accmul acc + mulA RA[row] + mulB RB[column] + c0, in wrapping 32-bit arithmetic (the result fits int32,
    // the host checks K (2^p - 1)(2^q - 1) < 2^31).
    auto finish_tile_row = [&](int irow, v16i_t (&t)[FN], uint32_t ra_row) __attribute__((always_inline)) {
        const uint32_t ra_m = ra_row * static_cast<uint32_t>(p.mulA);
        uint32_t col[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) col[j] = rb[j] * static_cast<uint32_t>(p.mulB) + static_cast<uint32_t>(p.c0);
        // accumulator register r of lane (lh, lr) is row 8 (r / 4) + 4 lh + r % 4, column lr
        static_for<16>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
            const uint32_t rowterm = need_ra ? static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(4 * row, static_cast<int>(ra_m))) : 0u;
#pragma unroll
            for (int j = 0; j < FN; ++j)
                t[j][r] = static_cast<int>(static_cast<uint32_t>(t[j][r]) * static_cast<uint32_t>(p.accmul) + rowterm + col[j]);
        });
        const int mrow0 = m0 + wm * FM * 32 + irow * 32;            // first row of this row of wave tiles
        if (p.Y) {
            // int32 output straight from the accumulators: one store instruction writes two 128-byte row segments.
            // The whole byte offset travels in the per-lane offset, which the hardware checks against M x N.
            const __amdgpu_buffer_rsrc_t rsrcY =
                __builtin_amdgcn_make_buffer_rsrc(p.Y, 0, 4u * static_cast<uint32_t>(p.M) * p.N, 0x00020000);
            const int gn0 = n0 + wn * FN * 32 + lr;
            const uint32_t vbase = 4u * (static_cast<uint32_t>(mrow0 + 4 * lh) * p.N + gn0);
            static_for<FN * 16>([&](auto c) {
                constexpr int j = decltype(c)::value / 16, r = decltype(c)::value % 16;
                constexpr int row = 8 * (r >> 2) + (r & 3);
                const uint32_t voff = (vbase + 128u * j) | (gn0 + 32 * j < p.N ? 0u : OUT_OF_RANGE);
                __builtin_amdgcn_raw_buffer_store_b32(t[j][r], rsrcY, voff + 4u * row * static_cast<uint32_t>(p.N), 0, 0);
            });
        }
        if (!p.scale) return;
        MfmaParams pe = p;                              // the shared epilogue sees finished integers
        pe.out_scale = 1.0f; pe.c0 = 0; pe.Y = nullptr;
        static_for<FN>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int gn = n0 + wn * FN * 32 + j * 32 + lr;
            float sc = 0.0f, bi = 0.0f;
            if (gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
            static_for<4>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                const int row0 = mrow0 + 8 * k;
                const float v4[4] = {static_cast<float>(t[j][4 * k]), static_cast<float>(t[j][4 * k + 1]),
                                     static_cast<float>(t[j][4 * k + 2]), static_cast<float>(t[j][4 * k + 3])};
                finish_rows8(pe, v4, row0, gn, sc, bi, load_res_rows8(pe, row0, gn >> 5, lane), lane, lr, lh);
            });
        });
    };

    if constexpr (NKS == 1) {
        static_for<FM>([&](auto ic) { finish_tile_row(decltype(ic)::value, acc[decltype(ic)::value], ra[decltype(ic)::value]); });
    } else {
        // The waves of a pair add their halves: wave ks keeps tile row ks, hands the other one (and its row sums) to
        // its partner through LDS, and finishes its own.  Per wave: FN 16 accumulator registers, one row-sum register
        // of A, FN of B, of 64 lanes each.
        constexpr int XREGS = FN * 16 + 1 + FN;
        __syncthreads();                                // every wave is done with the operand tiles
        uint32_t *xch = smem + (wave * XREGS) * 64 + lane, *from = smem + ((wave ^ 4) * XREGS) * 64 + lane;
        v16i_t mine[FN];
        uint32_t ra_mine;
        if (ks == 0) {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                mine[j] = acc[0][j];
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[(j * 16 + r) * 64] = static_cast<uint32_t>(acc[1][j][r]);
            }
            ra_mine = ra[0];
            xch[FN * 16 * 64] = ra[1];
        } else {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                mine[j] = acc[1][j];
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[(j * 16 + r) * 64] = static_cast<uint32_t>(acc[0][j][r]);
            }
            ra_mine = ra[1];
            xch[FN * 16 * 64] = ra[0];
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) xch[(FN * 16 + 1 + j) * 64] = rb[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[j][r] += static_cast<int>(from[(j * 16 + r) * 64]);
            rb[j] += from[(FN * 16 + 1 + j) * 64];
        }
        ra_mine += from[FN * 16 * 64];
        finish_tile_row(ks, mine, ra_mine);
    }
}

}  // namespace apnn
