// The 8-bit integer matrix form (mfma_i8.h) with the K steps, not the outputs, shared out among the waves.
//
// mfma_i8_kernel is bound by the vector instructions that transpose plane words into bytes, and with 64 x 64 wave
// tiles one transposed fragment feeds only two matrix instructions.  Here a block still owns 128 x 128 outputs (so a
// 2048^2 product still has a block for every compute unit), but each of its four waves computes ALL of them -- 4 x 4
// instruction tiles, 256 accumulator registers, one wave per SIMD -- over its own quarter of K: wave w takes chunk w
// of every group of four chunks.  One transposed fragment now feeds four matrix instructions, half the vector
// instructions per matrix instruction (7 instead of 14.5 at 3 x 5 bits), and the four partial results are added
// through LDS once, at the end.
//
// What it buys, measured: the K-dependent part is a quarter shorter (4.5 against 5.95 us per 1024 of K at 4 x 4 bits,
// 2048^2 outputs), not half: a lone wave overlaps only about four vector instructions with a matrix instruction, the
// rest add to it; and the K-independent part is 3.7 us longer (the exchange of 4 x 256 accumulator registers
// through LDS).  So the dispatch takes this kernel for long K only.
//
// Loader, LDS layout, transposition and encodings are those of mfma_i8_kernel.  Registers: the bytes of the word being
// multiplied and of the next one (2 x 64), and the plane words of ONE fragment at a time, read from LDS two
// matrix instructions before its transposition; the 32 matrix instructions of a word each carry one piece of work.
#pragma once
#include "mfma_i8.h"

namespace apnn {

// LDS: two group buffers of four chunks; afterwards the exchange of the accumulators, one instruction-tile column at
// a time (64 registers of 64 lanes per wave) plus 8 row-sum registers per wave.
constexpr int mfma_i8_wide_lds_bytes(int PA, int PB)
{
    const int tiles = 2 * (PA + PB) * 128 * 4 * 16, exchange = 4 * (64 + 8) * 256;
    return tiles > exchange ? tiles : exchange;
}

// planes_to_bytes cut into four pieces of about the same number of instructions, so that every matrix instruction of
// the loop below carries one (a wave issues in order: an uneven split leaves the matrix unit idle behind the long
// pieces).  x carries the state between the pieces; d is complete after piece 3.
template <int C, int Q>
__device__ __forceinline__ void planes_to_bytes4(const uint32_t (&w)[I8Slots<C>::value], const I8Masks &k, uint32_t (&x)[8], uint32_t (&d)[8])
{
    if constexpr (C == I8_C8) {
        if constexpr (Q == 0) {
#pragma unroll
            for (int s = 0; s < 8; ++s) x[s] = w[s];
            swap_blocks2<4>(x[0], x[4], x[1], x[5], k.m0f);
            swap_blocks2<4>(x[2], x[6], x[3], x[7], k.m0f);
        } else if constexpr (Q == 1) {
            swap_blocks2<2>(x[0], x[2], x[1], x[3], k.m33);
            swap_blocks2<2>(x[4], x[6], x[5], x[7], k.m33);
        } else if constexpr (Q == 2) {
            swap_blocks2<1>(x[0], x[1], x[2], x[3], k.m55);
#pragma unroll
            for (int j = 0; j < 4; ++j) d[j] = x[j];
        } else {
            swap_blocks2<1>(x[4], x[5], x[6], x[7], k.m55);
#pragma unroll
            for (int j = 4; j < 8; ++j) d[j] = x[j];
        }
    } else if constexpr (C == I8_C4) {
        if constexpr (Q == 0) {
            x[0] = w[0]; x[1] = w[1]; x[2] = w[2]; x[3] = w[3];
            swap_blocks2<2>(x[0], x[2], x[1], x[3], k.m33);
        } else if constexpr (Q == 1) {
            swap_blocks2<1>(x[0], x[1], x[2], x[3], k.m55);
        } else if constexpr (Q == 2) {
            const uint64_t h01 = pair_shr<4>(make_pair(x[0], x[1]));
            d[0] = x[0] & k.m0f;
            d[1] = x[1] & k.m0f;
            d[4] = half_of<0>(h01) & k.m0f;
            d[5] = half_of<1>(h01) & k.m0f;
        } else {
            const uint64_t h23 = pair_shr<4>(make_pair(x[2], x[3]));
            d[2] = x[2] & k.m0f;
            d[3] = x[3] & k.m0f;
            d[6] = half_of<0>(h23) & k.m0f;
            d[7] = half_of<1>(h23) & k.m0f;
        }
    } else {
        if constexpr (Q == 0) {
            const uint32_t a = w[0], b = w[1];
            x[0] = bit_select(a, b << 1, k.m55);
            x[1] = bit_select(a >> 1, b, k.m55);
        } else if constexpr (Q == 1) {
            const uint64_t h = pair_shr<2>(make_pair(x[0], x[1]));
            d[0] = x[0] & k.m03;
            d[1] = x[1] & k.m03;
            d[2] = half_of<0>(h) & k.m03;
            d[3] = half_of<1>(h) & k.m03;
        } else if constexpr (Q == 2) {
            const uint64_t h4 = pair_shr<4>(make_pair(x[0], x[1]));
            d[4] = half_of<0>(h4) & k.m03;
            d[5] = half_of<1>(h4) & k.m03;
        } else {
            const uint64_t h6 = pair_shr<6>(make_pair(x[0], x[1]));
            d[6] = half_of<0>(h6) & k.m03;
            d[7] = half_of<1>(h6) & k.m03;
        }
    }
}

// Fewest planes an operand of a class can have: those slots always exist; the others are read from the operand's last
// plane and masked off (a test per read made the loop a thicket of branches).
template <int C> struct I8MinPlanes { static constexpr int value = C == I8_C8 ? 5 : C == I8_C4 ? 3 : 1; };

template <int CA, int CB>
__global__ __launch_bounds__(256, 1) void mfma_i8_wide_kernel(const MfmaParams p)
{
    constexpr int MINA = I8MinPlanes<CA>::value, MINB = I8MinPlanes<CB>::value;
    constexpr int SA = I8Slots<CA>::value, SB = I8Slots<CB>::value;
    constexpr int F = 4;                                // instruction tiles per wave, each way
    constexpr int BM = 128, BN = 128, G = 4, NW = 4;
    constexpr int RB = 64 / G, NBR = BM / RB;           // rows per load instruction, row blocks per plane
    extern __shared__ __attribute__((aligned(1024))) uint32_t smem[];
    typedef __attribute__((address_space(3))) uint32_t *lds_ptr_t;
    const uint32_t smem_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)smem));
    const int a_bytes = p.PA * BM * G * 16, buf_bytes = a_bytes + p.PB * BN * G * 16;
    int n_pa = p.PA, n_pb = p.PB;                       // kept opaque: plane tests stay scalar compares where they stand
    auto fresh_counts = [&]() __attribute__((always_inline)) { asm volatile("" : "+s"(n_pa), "+s"(n_pb)); };

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 31, lh = lane >> 5;

    const int tilesN = (p.N + BN - 1) / BN;
    int tile = blockIdx.x;
    if (p.xcd_regions) {                                // one rectangular region of tiles per XCD
        const int tilesM = (p.M + BM - 1) / BM;
        const int rw = tilesN >> 2, rh = tilesM >> 1, xcd = tile & 7, idx = tile >> 3;
        tile = ((xcd >> 2) * rh + idx / rw) * tilesN + (xcd & 3) * rw + idx % rw;
    }
    const int m0 = (tile / tilesN) * BM, n0 = (tile % tilesN) * BN;

    I8Masks km;
    km.m0f = reg_const(0x0F0F0F0Fu); km.m33 = reg_const(0x33333333u);
    km.m55 = reg_const(0x55555555u); km.m03 = reg_const(0x03030303u);

    // ---- loader (as in mfma_i8_kernel): one instruction moves the 4 pieces of 16 consecutive rows of one plane,
    // adjacent lanes on adjacent pieces of a row; piece j of row r' lands in slot j ^ swz(r').
    auto swz = [](int r) { return (r >> 1) & 3; };
    const uint32_t bytesA = 4u * static_cast<uint32_t>(p.M) * p.PA * p.ldwA, bytesB = 4u * static_cast<uint32_t>(p.N) * p.PB * p.ldwB;
    const v4u_t descA = make_raw_desc(p.A, bytesA), descB = make_raw_desc(p.B, bytesB);
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;      // operands are smaller than 2 GiB (host check)
    const int ld_row = lane / G, ld_piece = (lane % G) ^ swz(ld_row);
    const uint32_t lane_offA = 4u * static_cast<uint32_t>(m0 + ld_row) * p.PA * p.ldwA + 16u * ld_piece;
    const uint32_t lane_offB = 4u * static_cast<uint32_t>(n0 + ld_row) * p.PB * p.ldwB + 16u * ld_piece;
    uint32_t gl_offA = 0, gl_offB = 0, gl_lds = 0;
    int gl_k = 0;
    auto begin_group = [&](int group, uint32_t lds_bytes_base) __attribute__((always_inline)) {
        const uint32_t dead = 4 * (group * G + ld_piece) < p.Kw ? 0u : OUT_OF_RANGE;
        gl_offA = lane_offA | dead;
        gl_offB = lane_offB | dead;
        gl_lds = lds_bytes_base;
        gl_k = __builtin_amdgcn_readfirstlane(group * G * 16);
    };
    constexpr int NDA = SA * NBR / NW, NDB = SB * NBR / NW, NLOAD = NDA + NDB;     // (NBR = 8: whole numbers)
    auto uniform_desc = [](v4u_t d) __attribute__((always_inline)) {
        v4u_t r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_readfirstlane(d[i]);
        return r;
    };
    // load instruction d of this wave: plane d / 2, row block wave + 4 (d % 2) -- of A, then of B (with 4 waves and 8
    // row blocks the plane does not depend on the wave); planes a class may lack are tested, the others are not
    auto load_one = [&](auto dc) __attribute__((always_inline)) {
        constexpr int d = decltype(dc)::value;
        if constexpr (d < NDA) {
            constexpr int s = d / 2;
            const int n = s * NBR + wave + NW * (d % 2);
            if (s < MINA || s < n_pa) {
                const uint32_t uni = 4u * static_cast<uint32_t>((n % NBR) * RB * p.PA + s) * p.ldwA + gl_k;
                load_to_lds_16(uniform_desc(descA), __builtin_amdgcn_readfirstlane(gl_lds + n * 1024), gl_offA + uni, 0);
            }
        } else {
            constexpr int s = (d - NDA) / 2;
            const int n = s * NBR + wave + NW * ((d - NDA) % 2);
            if (s < MINB || s < n_pb) {
                const uint32_t uni = 4u * static_cast<uint32_t>((n % NBR) * RB * p.PB + s) * p.ldwB + gl_k;
                load_to_lds_16(uniform_desc(descB), __builtin_amdgcn_readfirstlane(gl_lds + a_bytes + n * 1024), gl_offB + uni, 0);
            }
        }
    };
    constexpr int WAIT_LOADS = 0x0F70;                  // s_waitcnt vmcnt(0)

    // ---- reader.  Lane (half h, row r) reads word 2h + e of this wave's chunk (piece `wave`) of plane s of fragment
    // row f at byte  buffer + ((s 128 + 32 f + r) 4 + (wave ^ swz(r))) 16 + 8 h + 4 e.
    // Slots beyond the fewest planes of the class have an address register of their own, which points at the
    // operand's last plane when the slot's plane does not exist (always inside the buffer), and a mask of zeros.
    const uint32_t rd0A = (lr * G + (wave ^ swz(lr & (RB - 1)))) * 16 + 8 * lh;
    uint32_t rdA = rd0A, rdB = rd0A + a_bytes;
    uint32_t rdAx[SA - MINA + 1], rdBx[SB - MINB + 1];  // (one spare each: arrays of no length are not allowed)
    uint32_t mkA[SA - MINA + 1], mkB[SB - MINB + 1];
#pragma unroll
    for (int s = MINA; s < SA; ++s) mkA[s - MINA] = __builtin_amdgcn_readfirstlane(s < p.PA ? ~0u : 0u);
#pragma unroll
    for (int s = MINB; s < SB; ++s) mkB[s - MINB] = __builtin_amdgcn_readfirstlane(s < p.PB ? ~0u : 0u);
    auto set_read_buffer = [&](uint32_t byte_base) __attribute__((always_inline)) {
        rdA = rd0A + byte_base;
        rdB = rd0A + a_bytes + byte_base;
#pragma unroll
        for (int s = MINA; s < SA; ++s) rdAx[s - MINA] = rdA + static_cast<uint32_t>(min(s, p.PA - 1)) * (BM * G * 16);
#pragma unroll
        for (int s = MINB; s < SB; ++s) rdBx[s - MINB] = rdB + static_cast<uint32_t>(min(s, p.PB - 1)) * (BN * G * 16);
    };
    set_read_buffer(0);

    v16i_t acc[F][F];
#pragma unroll
    for (int i = 0; i < F; ++i)
#pragma unroll
        for (int j = 0; j < F; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    uint32_t ra[F], rb[F];                              // decoded row sums of this lane's words (Sec. 3.2 Case III: J X)
#pragma unroll
    for (int i = 0; i < F; ++i) ra[i] = rb[i] = 0;
    const bool need_ra = p.mulA != 0, need_rb = p.mulB != 0;
    struct Bytes { uint32_t a[F][8], b[F][8]; };        // the bytes of two instruction steps (dwords 0-3, 4-7) per fragment

    // Fragment t (0-3: rows of A, 4-7: rows of B) of word e of the chunk: its plane words, read from LDS ...
    constexpr int SMAX = SA > SB ? SA : SB;
    uint32_t wq[SMAX];
    auto read_words = [&](auto tc, auto ec) __attribute__((always_inline)) {
        constexpr int t = decltype(tc)::value, e = decltype(ec)::value;
        const char *lds = reinterpret_cast<const char *>(smem);
        if constexpr (t < F) {
#pragma unroll
            for (int s = 0; s < SA; ++s)
                wq[s] = s < MINA ? *reinterpret_cast<const uint32_t *>(lds + rdA + (s * BM + 32 * t) * G * 16 + 4 * e)
                                 : *reinterpret_cast<const uint32_t *>(lds + rdAx[s < MINA ? 0 : s - MINA] + 32 * t * G * 16 + 4 * e);
        } else {
#pragma unroll
            for (int s = 0; s < SB; ++s)
                wq[s] = s < MINB ? *reinterpret_cast<const uint32_t *>(lds + rdB + (s * BN + 32 * (t - F)) * G * 16 + 4 * e)
                                 : *reinterpret_cast<const uint32_t *>(lds + rdBx[s < MINB ? 0 : s - MINB] + 32 * (t - F) * G * 16 + 4 * e);
        }
    };
    // ... and transposed into bytes in four pieces (x carries the state between them); piece 0 takes the words out of
    // wq, piece 1 the row sums from a copy
    uint32_t x[8], wcopy[SMAX];
    auto transpose_piece = [&](auto tc, auto qc, Bytes &nxt) __attribute__((always_inline)) {
        constexpr int t = decltype(tc)::value, Q = decltype(qc)::value;
        if constexpr (t < F) {
            uint32_t w[SA];
            if constexpr (Q == 0) {
#pragma unroll
                for (int s = 0; s < SA; ++s) wcopy[s] = w[s] = s < MINA ? wq[s] : (wq[s] & mkA[s < MINA ? 0 : s - MINA]);
                if (CA == I8_C8) w[SA - 1] ^= p.flipA;  // an 8-bit operand enters as value - 128
            }
            if constexpr (Q == 1) {
                if (need_ra) {
#pragma unroll
                    for (int s = 0; s < SA; ++s) ra[t] += static_cast<uint32_t>(__popc(wcopy[s])) << s;
                }
            }
            planes_to_bytes4<CA, Q>(w, km, x, nxt.a[t]);
        } else {
            uint32_t w[SB];
            if constexpr (Q == 0) {
#pragma unroll
                for (int s = 0; s < SB; ++s) wcopy[s] = w[s] = s < MINB ? wq[s] : (wq[s] & mkB[s < MINB ? 0 : s - MINB]);
                if (CB == I8_C8) w[SB - 1] ^= p.flipB;
            }
            if constexpr (Q == 1) {
                if (need_rb) {
#pragma unroll
                    for (int s = 0; s < SB; ++s) rb[t - F] += static_cast<uint32_t>(__popc(wcopy[s])) << s;
                }
            }
            planes_to_bytes4<CB, Q>(w, km, x, nxt.b[t - F]);
        }
    };

    // One period: the 32 matrix instructions of one word (bytes `cur`; two steps of 4 x 4 tiles), and under them the
    // next word made into `nxt`, one fragment (0-3: rows of A, 4-7: of B) per four matrix instructions, one piece of
    // its transposition behind each; the plane words of fragment t + 1 are read behind the third.  The words of
    // fragment 0 of the word after next are read at the end (`late`), and `hook` deals whatever else there is.  A
    // wave issues in order, so everything is spread out singly behind the matrix instructions, each slot fenced.
    auto period = [&](const Bytes &cur, Bytes &nxt, auto ec, auto late_ec, auto &&hook) __attribute__((always_inline)) {
        static_for<32>([&](auto qc) {
            constexpr int q = decltype(qc)::value, h = q / 16, i = q / 4 % 4, j = q % 4, t = q / 4, r = q % 4;
            const v4i_t a = {static_cast<int>(cur.a[i][4 * h]), static_cast<int>(cur.a[i][4 * h + 1]),
                             static_cast<int>(cur.a[i][4 * h + 2]), static_cast<int>(cur.a[i][4 * h + 3])};
            const v4i_t b = {static_cast<int>(cur.b[j][4 * h]), static_cast<int>(cur.b[j][4 * h + 1]),
                             static_cast<int>(cur.b[j][4 * h + 2]), static_cast<int>(cur.b[j][4 * h + 3])};
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i][j], 0, 0, 0);
            transpose_piece(std::integral_constant<int, t>{}, std::integral_constant<int, r>{}, nxt);
            hook(qc);                                   // (slot 28 of an even period: barrier and buffer change, before the late read)
            if constexpr (r == 2 && t < 2 * F - 1) read_words(std::integral_constant<int, t + 1>{}, ec);
            if constexpr (q == 30) read_words(std::integral_constant<int, 0>{}, late_ec);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using E0 = std::integral_constant<int, 0>;
    using E1 = std::integral_constant<int, 1>;
    auto no_hook = [](auto) {};

    // Group g (chunks 4 g .. 4 g + 3, this wave's is 4 g + wave) lives in buffer g mod 2.  Period 2 g multiplies the
    // first word of the wave's chunk and makes the second; period 2 g + 1 multiplies the second and makes the first
    // word of the chunk of group g + 1.  The last reads of group g are those of slot 26 of period 2 g; at slot 28 group
    // g + 1 has landed (wait, barrier: the only ones of the group), the reads move over to its buffer, and group g + 2
    // is requested into the buffer of group g, the loads dealt over the slots that follow.  Beyond the last: zeros.
    Bytes by0, by1;
    begin_group(0, smem_base);
    static_for<NLOAD>([&](auto dc) { load_one(dc); });
    begin_group(1, smem_base + buf_bytes);
    static_for<NLOAD>([&](auto dc) { load_one(dc); });
    __builtin_amdgcn_s_waitcnt(WAIT_LOADS);
    __syncthreads();
    uint32_t cur_base = 0;
    static_for<2 * F>([&](auto tc) {                    // the first word, with nothing to run under
        read_words(tc, E0{});
        static_for<4>([&](auto qc) { transpose_piece(tc, qc, by0); });
    });
    read_words(E0{}, E1{});                             // fragment 0 of the second word
    const int groups = p.nk / G;                        // (the host makes nk a multiple of 4)
    for (int group = 0; group < groups; ++group) {
        fresh_counts();
        period(by0, by1, E1{}, E0{}, [&](auto qc) {
            constexpr int q = decltype(qc)::value;
            if constexpr (q == 28) {
                __builtin_amdgcn_s_waitcnt(WAIT_LOADS); // this wave's share of group + 1 is in LDS
                __syncthreads();
                begin_group(group + 2, smem_base + cur_base);
                cur_base = cur_base ? 0u : static_cast<uint32_t>(buf_bytes);
                set_read_buffer(cur_base);
            }
            if constexpr (q > 28) load_one(std::integral_constant<int, q - 29>{});
        });
        fresh_counts();
        period(by1, by0, E0{}, E1{}, [&](auto qc) {
            constexpr int q = decltype(qc)::value;
            if constexpr (q + 3 < NLOAD) load_one(std::integral_constant<int, q + 3>{});
        });
    }
    __builtin_amdgcn_s_waitcnt(WAIT_LOADS);             // the loads requested for groups beyond the last one have landed

    // ---- the four partial results meet in LDS.  The two lane halves hold the row sums of different words of a row.
#pragma unroll
    for (int i = 0; i < F; ++i) {
        ra[i] += static_cast<uint32_t>(__shfl_xor(static_cast<int>(ra[i]), 32));
        rb[i] += static_cast<uint32_t>(__shfl_xor(static_cast<int>(rb[i]), 32));
    }
    __syncthreads();                                    // every wave is done with the operand tiles
    constexpr int XREGS = 64 + 8;                       // per wave: one column of instruction tiles, 4 + 4 row sums
    uint32_t *mine = smem + (wave * XREGS) * 64 + lane;
#pragma unroll
    for (int i = 0; i < F; ++i) {
        mine[(64 + i) * 64] = ra[i];
        mine[(68 + i) * 64] = rb[i];
    }
    // Wave w finishes tile row w (rows 32 w .. 32 w + 31, all 128 columns): column j of every wave goes through LDS
    // in round j, and each wave adds up the four copies of its own tile (its own included: a register array cannot
    // be indexed by the wave number).
    v16i_t fin[F];
    static_for<F>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        if (j > 0) __syncthreads();                     // the previous round has been read
#pragma unroll
        for (int i = 0; i < F; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[(i * 16 + r) * 64] = static_cast<uint32_t>(acc[i][j][r]);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            uint32_t sum = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += smem[(w * XREGS + wave * 16 + r) * 64 + lane];
            fin[j][r] = static_cast<int>(sum);
        }
    });
    uint32_t ra_row = 0, rb_col[F];
#pragma unroll
    for (int j = 0; j < F; ++j) rb_col[j] = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        ra_row += smem[(w * XREGS + 64 + wave) * 64 + lane];
#pragma unroll
        for (int j = 0; j < F; ++j) rb_col[j] += smem[(w * XREGS + 68 + j) * 64 + lane];
    }

    // ---- encoding recovery (Sec. 3.2) and the outputs of tile row `wave`:
    //   Y = accmul acc + mulA RA[row] + mulB RB[column] + c0, in wrapping 32-bit arithmetic (the result fits int32).
    const uint32_t ra_m = ra_row * static_cast<uint32_t>(p.mulA);
    uint32_t col[F];
#pragma unroll
    for (int j = 0; j < F; ++j) col[j] = rb_col[j] * static_cast<uint32_t>(p.mulB) + static_cast<uint32_t>(p.c0);
    // accumulator register r of lane (lh, lr) is row 8 (r / 4) + 4 lh + r % 4, column lr
    static_for<16>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
        const uint32_t rowterm = need_ra ? static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(4 * row, static_cast<int>(ra_m))) : 0u;
#pragma unroll
        for (int j = 0; j < F; ++j)
            fin[j][r] = static_cast<int>(static_cast<uint32_t>(fin[j][r]) * static_cast<uint32_t>(p.accmul) + rowterm + col[j]);
    });
    const int mrow0 = m0 + wave * 32;
    if (p.Y) {
        // int32 output straight from the registers: one store instruction writes two 128-byte row segments.  The whole
        // byte offset travels in the per-lane offset, which the hardware checks against M x N.
        const __amdgpu_buffer_rsrc_t rsrcY =
            __builtin_amdgcn_make_buffer_rsrc(p.Y, 0, 4u * static_cast<uint32_t>(p.M) * p.N, 0x00020000);
        const int gn0 = n0 + lr;
        const uint32_t vbase = 4u * (static_cast<uint32_t>(mrow0 + 4 * lh) * p.N + gn0);
        static_for<F * 16>([&](auto c) {
            constexpr int j = decltype(c)::value / 16, r = decltype(c)::value % 16;
            constexpr int row = 8 * (r >> 2) + (r & 3);
            const uint32_t voff = (vbase + 128u * j) | (gn0 + 32 * j < p.N ? 0u : OUT_OF_RANGE);
            __builtin_amdgcn_raw_buffer_store_b32(fin[j][r], rsrcY, voff + 4u * row * static_cast<uint32_t>(p.N), 0, 0);
        });
    }
    if (!p.scale) return;
    MfmaParams pe = p;                                  // the shared epilogue sees finished integers
    pe.out_scale = 1.0f; pe.c0 = 0; pe.Y = nullptr;
    static_for<F>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int gn = n0 + j * 32 + lr;
        float sc = 0.0f, bi = 0.0f;
        if (gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
        static_for<4>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            const int row0 = mrow0 + 8 * k;
            const float v4[4] = {static_cast<float>(fin[j][4 * k]), static_cast<float>(fin[j][4 * k + 1]),
                                 static_cast<float>(fin[j][4 * k + 2]), static_cast<float>(fin[j][4 * k + 3])};
            finish_rows8(pe, v4, row0, gn, sc, bi, load_res_rows8(pe, row0, gn >> 5, lane), lane, lr, lh);
        });
    });
}

}  // namespace apnn
