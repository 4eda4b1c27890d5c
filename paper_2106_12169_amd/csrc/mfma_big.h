// Matrix-core kernel for large matrix-layout products (block tile 256 x 256).
//
// Same arithmetic, operand encodings and digit passes as mfma_fp4_kernel: the
// packed bit planes of the ABI are re-composed, per lane and in registers, into
// FP4 (E2M1) codes and multiplied by v_mfma_scale_f32_32x32x64_f8f6f4 (Sec. 3.1
// template with a two-plane primitive; Eq. 1 weights; Sec. 3.2 encodings).  What
// differs is the schedule, which at this size decides the run time:
//   - every wave owns FM x FN = 4 x 4 matrix-instruction tiles (128 x 128 outputs),
//     so one expansion of a plane word into FP4 codes feeds four matrix
//     instructions; the 256 accumulator registers per lane live in the
//     accumulation half of the unified register file (one wave per SIMD);
//   - global memory -> LDS directly, 16 bytes per lane, into unpadded tiles whose
//     16-byte pieces are XOR-swizzled by row (no staging registers, no LDS stores);
//   - the digit weights 4^da 4^db of Eq. 1 and the power of two that undoes the
//     halved two-plane codes travel as the block scales of the matrix instruction,
//     so nothing but the matrix unit touches the accumulators before the epilogue;
//   - measured on gfx950: a lone wave per SIMD hides about 4 vector instructions
//     behind each matrix instruction, and a longer run of vector work stalls the
//     matrix pipe for a whole instruction time.  The plane -> FP4 expansion of
//     step s + 1 is therefore cut into tasks of at most 4 instructions, one task
//     after each matrix instruction of step s, each fenced against instruction
//     scheduling; shifts work on the words of two consecutive steps at once
//     (64-bit shifts: the bits that cross between the words fall outside the masks);
//   - the int32 output is stored straight from the accumulators with buffer stores whose
//     per-lane offset carries row and column, so the hardware's range check drops what
//     lies beyond M x N (two 128-byte row segments per instruction, no branches, no waits).
#pragma once
#include "mfma_kernel.h"

namespace apnn {

struct Fp4Masks2 { uint32_t m2, m3, m5, m8; };

typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (base, no stride, byte count, 32-bit raw data format).
__device__ __forceinline__ v4u_t make_raw_desc(const void *base, uint32_t bytes)
{
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    v4u_t d;
    d[0] = static_cast<uint32_t>(a);
    d[1] = static_cast<uint32_t>(a >> 32) & 0xFFFFu;
    d[2] = bytes;
    d[3] = 0x00020000u;
    return d;
}

// Global memory -> LDS, 16 bytes per lane, no registers in between: lane l's data
// lands at LDS byte address lds_base + 16 l (lds_base is wave-uniform and travels
// in M0); a lane whose offset lies outside the descriptor deposits zeros.  Written
// as an instruction sequence of its own so that completion is tracked only by the
// explicit vmcnt waits of the caller (a compiler that knows about the LDS write
// would wait for it before every later LDS read, which serialises the pipeline).
__device__ __forceinline__ void load_to_lds_16(v4u_t desc, uint32_t lds_base, uint32_t voffset, int soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(desc), "s"(soffset)
                 : "memory", "m0");
}

// Shifts of a register pair.  Each half holds an independent plane word; the few
// bits that cross from one half into the other land where the caller's masks are 0.
// (Plain C++ shifts would be split into two 32-bit shifts again by the optimiser,
// exactly because those bits are never used.)
template <int N> __device__ __forceinline__ uint64_t pair_shl(uint64_t x)
{
    uint64_t r;
    asm("v_lshlrev_b64 %0, %1, %2" : "=v"(r) : "i"(N), "v"(x));
    return r;
}
template <int N> __device__ __forceinline__ uint64_t pair_shr(uint64_t x)
{
    uint64_t r;
    asm("v_lshrrev_b64 %0, %1, %2" : "=v"(r) : "i"(N), "v"(x));
    return r;
}
__device__ __forceinline__ uint64_t make_pair(uint32_t lo, uint32_t hi) { return static_cast<uint64_t>(hi) << 32 | lo; }
template <int E> __device__ __forceinline__ uint32_t half_of(uint64_t x) { return E ? static_cast<uint32_t>(x >> 32) : static_cast<uint32_t>(x); }

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int i)
{
    return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

// ---- plane words -> FP4 codes, in tasks of at most 4 vector instructions.
// 32 K positions of one operand row become 4 dwords of 8 codes; nibble i of dword r
// holds the element at bit 4 i + rho(r), rho = (0, 2, 1, 3) (any K order is valid as
// long as both operands use the same one).
//   prep   (once per fragment row and pair of steps)  shifted copies of the word pairs
//   expand (per fragment row and step)                one task, or two for a two-plane digit
struct PairPrep { uint64_t s[3]; };

template <int KIND> __device__ __forceinline__ void prep_pair(uint64_t w0, uint64_t w1, PairPrep &pp)
{
    if (KIND == OPK_U1) {            // codes (x << 1) & m2, (x >> 1) & m2, x & m2, (x >> 2) & m2
        pp.s[0] = pair_shl<1>(w0); pp.s[1] = pair_shr<1>(w0); pp.s[2] = pair_shr<2>(w0);
    } else if (KIND == OPK_PM1) {    // sign bits from x << 3, x << 1, x << 2, x
        pp.s[0] = pair_shl<3>(w0); pp.s[1] = pair_shl<1>(w0); pp.s[2] = pair_shl<2>(w0);
    } else {                         // upper plane moved up by one, lower plane moved down by one
        pp.s[0] = pair_shl<1>(w1); pp.s[1] = pair_shr<1>(w0);
    }
}

struct PairTmp { uint32_t ze, zo; uint64_t zz; };

// E: which word of the pair (0: first step, 1: second step); x0, x1: that step's own words.
template <int KIND, int E, int TASK>
__device__ __forceinline__ void expand_task(uint32_t x0, uint32_t x1, const PairPrep &pp, PairTmp &t, const Fp4Masks2 &k, v8i_t &out)
{
    if (KIND == OPK_U1) {                       // 0 -> 0000 (0.0), 1 -> 0010 (1.0)
        out[0] = half_of<E>(pp.s[0]) & k.m2;
        out[1] = half_of<E>(pp.s[1]) & k.m2;
        out[2] = x0 & k.m2;
        out[3] = half_of<E>(pp.s[2]) & k.m2;
        out[4] = out[5] = out[6] = out[7] = 0;
    } else if (KIND == OPK_PM1) {               // 1 -> 0010 (+1.0), 0 -> 1010 (-1.0)
        out[0] = (~half_of<E>(pp.s[0]) & k.m8) | k.m2;
        out[1] = (~half_of<E>(pp.s[1]) & k.m8) | k.m2;
        out[2] = (~half_of<E>(pp.s[2]) & k.m8) | k.m2;
        out[3] = (~x0 & k.m8) | k.m2;
        out[4] = out[5] = out[6] = out[7] = 0;
    } else if (TASK == 0) {                     // code = x1 x0 = value / 2: interleave the planes pairwise ...
        // (a & m5) | (b & ~m5) as one three-input bit operation (truth table a:0xF0, b:0xCC, mask:0xAA)
        constexpr int SEL = (0xF0 & 0xAA) | (0xCC & 0x55);
        t.ze = __builtin_amdgcn_bitop3_b32(x0, half_of<E>(pp.s[0]), k.m5, SEL);      // pairs of the even positions
        t.zo = __builtin_amdgcn_bitop3_b32(half_of<E>(pp.s[1]), x1, k.m5, SEL);      // pairs of the odd positions
        t.zz = pair_shr<2>(make_pair(t.ze, t.zo));
    } else {                                    // ... and spread the pairs over the nibbles
        out[0] = t.ze & k.m3;
        out[1] = half_of<0>(t.zz) & k.m3;
        out[2] = t.zo & k.m3;
        out[3] = half_of<1>(t.zz) & k.m3;
        out[4] = out[5] = out[6] = out[7] = 0;
    }
}

template <int KA, int KB, int NWM, int NWN, int FM, int FN>
__global__ __launch_bounds__(64 * NWM * NWN, FM * FN >= 16 ? 1 : 2) void mfma_big_kernel(const MfmaParams p)
{
#ifdef APNN_BIG_TIMING                              // instrumented build (see the epilogue): time stamps of the 100 MHz clock
    const unsigned long long tt0 = wall_clock64();
#endif
    constexpr int KC = 16;                              // words per chunk = 8 matrix-instruction steps = 2 groups of 4
    constexpr int LA = DigitPlanes<KA>::value, LB = DigitPlanes<KB>::value;
    constexpr int BM = NWM * FM * 32, BN = NWN * FN * 32;
    constexpr int NW = NWM * NWN;                       // waves
    constexpr int RSA = LA * KC, RSB = LB * KC;         // LDS row strides (words): rows are unpadded, pieces swizzled
    constexpr int PCA = 4 * LA, PCB = 4 * LB;           // 16-byte pieces per row
    constexpr int RIA = 64 / PCA, RIB = 64 / PCB;       // rows one wave-wide load instruction covers
    static_assert(BM % (RIA * NW) == 0 && BN % (RIB * NW) == 0, "every wave issues the same number of loads");
    constexpr int A_SLOTS = BM / RIA / NW, B_SLOTS = BN / RIB / NW;    // load instructions per wave and chunk

    constexpr int A_WORDS = BM * RSA, B_WORDS = BN * RSB;
    constexpr int TILE_WORDS = 2 * A_WORDS + 2 * B_WORDS;
    __shared__ __attribute__((aligned(1024))) uint32_t smem[TILE_WORDS];   // A buffer 0, A buffer 1, B buffer 0, B buffer 1
    typedef __attribute__((address_space(3))) uint32_t *lds_ptr_t;
    const uint32_t smem_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)smem));   // LDS byte address of the arena

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave index in scalar registers
    const int wm = wave / NWN, wn = wave % NWN;
    const int lr = lane & 31, lh = lane >> 5;

    const int tilesN = (p.N + BN - 1) / BN;
    // Workgroups go to the eight XCDs in turn (block b runs on XCD b mod 8), and every XCD fills its own L2 from
    // HBM.  When the tile grid divides into 2 x 4 regions, XCD x gets region x instead of every eighth tile of the
    // row-major order, so the operand rows its L2 pulls are those of a compact rectangle (for 16 x 16 tiles: 8 row
    // panels + 4 column panels instead of 16 + 2).
    int tile = blockIdx.x;
    if (p.xcd_regions) {
        const int tilesM = (p.M + BM - 1) / BM;
        const int rw = tilesN >> 2, rh = tilesM >> 1, xcd = tile & 7, idx = tile >> 3;
        tile = ((xcd >> 2) * rh + idx / rw) * tilesN + (xcd & 3) * rw + idx % rw;
    }
    const int m0 = (tile / tilesN) * BM, n0 = (tile % tilesN) * BN;

    Fp4Masks2 km;
    km.m2 = reg_const(0x22222222u); km.m3 = reg_const(0x33333333u);
    km.m5 = reg_const(0x55555555u); km.m8 = reg_const(0x88888888u);

    // ---- loader.  A wave-wide 16-byte-per-lane load deposits its 64 pieces
    // contiguously (1 KiB) in LDS, i.e. RI whole tile rows.  The piece a lane fetches
    // for LDS slot s of row r is piece s ^ swz(r), which spreads the 16-byte reads of 8
    // or 16 consecutive rows over all banks.  Addressing: descriptor base (scalar) +
    // per-lane byte offset (constant over the whole loop) + scalar offset of (digit
    // plane, chunk); a lane whose piece or plane does not exist uses an offset beyond
    // the descriptor's range, for which the hardware writes zeros.
    auto swz4 = [](int r) { return (((r >> 1) ^ (r >> 3)) & 1) | ((r >> 1) & 2); };         // 4 pieces per row
    auto swz8 = [](int r) { return ((r ^ (r >> 3)) & 1) | (r & 6); };                       // 8 pieces per row
    auto swzA = [&](int r) { return PCA == 4 ? swz4(r) : swz8(r); };
    auto swzB = [&](int r) { return PCB == 4 ? swz4(r) : swz8(r); };
    const uint32_t bytesA = 4u * static_cast<uint32_t>(p.M) * p.PA * p.ldwA, bytesB = 4u * static_cast<uint32_t>(p.N) * p.PB * p.ldwB;
    const v4u_t descA = make_raw_desc(p.A, bytesA), descB = make_raw_desc(p.B, bytesB);
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;      // operands are smaller than 2 GiB (host check)
    // Load instruction u of this wave covers tile rows (wave SLOTS + u) RI ...; the low
    // four row bits, hence the swizzle, repeat with period 2 in u.
    static_assert(A_SLOTS % 2 == 0 && B_SLOTS % 2 == 0, "the swizzle period divides the loads of a wave");
    uint32_t offA[A_SLOTS], offB[B_SLOTS];              // byte offsets of this lane's (row, plane, piece) in chunk 0, digit 0
    int pcA[2], pcB[2];                                 // this lane's piece (plane * 4 + piece of the chunk) for even / odd u
#pragma unroll
    for (int u = 0; u < A_SLOTS; ++u) {
        const int row = (wave * A_SLOTS + u) * RIA + lane / PCA, pc = (lane % PCA) ^ swzA(row);
        if (u < 2) pcA[u] = pc;
        offA[u] = 4u * ((static_cast<uint32_t>(min(m0 + row, p.M - 1)) * p.PA + pc / 4) * p.ldwA + 4 * (pc % 4));
    }
#pragma unroll
    for (int u = 0; u < B_SLOTS; ++u) {
        const int row = (wave * B_SLOTS + u) * RIB + lane / PCB, pc = (lane % PCB) ^ swzB(row);
        if (u < 2) pcB[u] = pc;
        offB[u] = 4u * ((static_cast<uint32_t>(min(n0 + row, p.N - 1)) * p.PB + pc / 4) * p.ldwB + 4 * (pc % 4));
    }
    struct FetchState { int soffA, soffB; uint32_t badA[2], badB[2]; };
    auto fetch_begin = [&](FetchState &fs, int da, int db, int kc, bool live) {
        const int pa0 = LA == 2 ? 2 * da : da, pb0 = LB == 2 ? 2 * db : db;       // first plane of the digit
        fs.soffA = 4 * (pa0 * p.ldwA + kc * KC);
        fs.soffB = 4 * (pb0 * p.ldwB + kc * KC);
        const int remK = live ? p.Kw - kc * KC : 0;     // words of this chunk that exist
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            fs.badA[e] = (static_cast<int>(4 * (pcA[e] % 4) < remK) & static_cast<int>(pcA[e] / 4 < p.PA - pa0)) ? 0u : OUT_OF_RANGE;
            fs.badB[e] = (static_cast<int>(4 * (pcB[e] % 4) < remK) & static_cast<int>(pcB[e] / 4 < p.PB - pb0)) ? 0u : OUT_OF_RANGE;
        }
    };
    auto fetch_one = [&](const FetchState &fs, int buf, auto uc) {   // load u of this wave: A loads first, then B loads
        constexpr int u = decltype(uc)::value;
        if constexpr (u < A_SLOTS) {
            load_to_lds_16(descA, smem_base + 4 * (buf * A_WORDS + (wave * A_SLOTS + u) * 256), offA[u] | fs.badA[u % 2], fs.soffA);
        } else if constexpr (u < A_SLOTS + B_SLOTS) {
            constexpr int ub = u - A_SLOTS;
            load_to_lds_16(descB, smem_base + 4 * (2 * A_WORDS + buf * B_WORDS + (wave * B_SLOTS + ub) * 256), offB[ub] | fs.badB[ub % 2], fs.soffB);
        }
    };
    constexpr int VMCNT0 = 0x0F70;                      // s_waitcnt vmcnt(0) (expcnt, lgkmcnt untouched)

    // ---- reader: this lane's words of one group (four steps) of a chunk; lane half lh owns
    // words 8 lh .. 8 lh + 7, i.e. pieces 2 lh and 2 lh + 1 of a plane.  Word index of
    // (fragment row f, plane pl, group g) in a tile: row stride * row + 4 * ((4 pl + 2 lh + g) ^ swz(row)),
    // where swz depends on the low row bits, i.e. on lr, only.
    int rdA[LA][2], rdB[LB][2];                         // word offsets for fragment row 0, per (plane, group)
#pragma unroll
    for (int pl = 0; pl < LA; ++pl)
#pragma unroll
        for (int g = 0; g < 2; ++g) rdA[pl][g] = (wm * FM * 32 + lr) * RSA + 4 * ((4 * pl + 2 * lh + g) ^ swzA(lr));
#pragma unroll
    for (int pl = 0; pl < LB; ++pl)
#pragma unroll
        for (int g = 0; g < 2; ++g) rdB[pl][g] = 2 * A_WORDS + (wn * FN * 32 + lr) * RSB + 4 * ((4 * pl + 2 * lh + g) ^ swzB(lr));
    // one LDS read of a group: read r covers (fragment row f, plane pl) of A, then of B
    auto read_one = [&](int buf, auto gc, auto rc, uint4 (&wa)[FM][LA], uint4 (&wb)[FN][LB]) {
        constexpr int r = decltype(rc)::value, g = decltype(gc)::value;
        if constexpr (r < FM * LA) {
            constexpr int f = r / LA, pl = r % LA;
            wa[f][pl] = *reinterpret_cast<const uint4 *>(&smem[buf * A_WORDS + rdA[pl][g] + f * 32 * RSA]);
        } else if constexpr (r < FM * LA + FN * LB) {
            constexpr int f = (r - FM * LA) / LB, pl = (r - FM * LA) % LB;
            wb[f][pl] = *reinterpret_cast<const uint4 *>(&smem[buf * B_WORDS + rdB[pl][g] + f * 32 * RSB]);
        }
    };
    constexpr int NREAD = FM * LA + FN * LB;

    v16f_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // ---- one step = FM x FN matrix instructions on the FP4 fragments of 64 K positions,
    // each followed by its share of the tasks that prepare the fragments of the next
    // step (and the shifted word pairs of the step pair after that), and by at most one
    // LDS read and one global load.
    //   odd  step 2 k + 1:  prep B (pair k + 1), expand A and B of step 2 k + 2
    //   even step 2 k:      expand A and B of step 2 k + 1, prep A (pair k + 1)
    constexpr int NMI = FM * FN;
    constexpr int EA = KA == OPK_U2 ? 2 : 1, EB = KB == OPK_U2 ? 2 : 1;            // expansion tasks per fragment row
    constexpr int NLOAD = A_SLOTS + B_SLOTS;
    // memory instructions are dealt to the portions of a step like the tasks: portion q takes reads / loads
    // [N q / NMI, N (q + 1) / NMI)
    auto reads_of = [&](int buf, auto gc, auto qc, uint4 (&wa)[FM][LA], uint4 (&wb)[FN][LB]) {
        constexpr int q = decltype(qc)::value, lo = NREAD * q / NMI, hi = NREAD * (q + 1) / NMI;
        static_for<hi - lo>([&](auto ic) { read_one(buf, gc, std::integral_constant<int, lo + decltype(ic)::value>{}, wa, wb); });
    };
    auto loads_of = [&](const FetchState &fs, int buf, auto qc) {
        constexpr int q = decltype(qc)::value, lo = NLOAD * q / NMI, hi = NLOAD * (q + 1) / NMI;
        static_for<hi - lo>([&](auto ic) { fetch_one(fs, buf, std::integral_constant<int, lo + decltype(ic)::value>{}); });
    };
    PairPrep ppa[FM], ppb[FN];
    PairTmp tta[FM], ttb[FN];
    // ODD: parity of the step being multiplied.  xw*/XST: group words and index (0..3) of the step to expand;
    // pw*/PI: group words and pair (0: words x, y; 1: z, w) to prepare.
    auto step = [&](auto oddc, const v8i_t (&fa)[FM], const v8i_t (&fb)[FN], int sa, int sb,
                    const uint4 (&xwa)[FM][LA], const uint4 (&xwb)[FN][LB], auto xstc, v8i_t (&na)[FM], v8i_t (&nb)[FN],
                    const uint4 (&pwa)[FM][LA], const uint4 (&pwb)[FN][LB], auto pic, auto &&hook) {
        constexpr bool ODD = decltype(oddc)::value != 0;
        constexpr int XST = decltype(xstc)::value, E = XST & 1, PI = decltype(pic)::value;
        constexpr int T_PREP = ODD ? FN : FM, T_EXP = FM * EA + FN * EB, T = T_PREP + T_EXP;
        auto prep_task = [&](auto fc) {
            constexpr int f = decltype(fc)::value;
            if constexpr (ODD) {
                const uint4 &w0 = pwb[f][0], &w1 = pwb[f][LB - 1];
                prep_pair<KB>(PI ? make_pair(w0.z, w0.w) : make_pair(w0.x, w0.y), PI ? make_pair(w1.z, w1.w) : make_pair(w1.x, w1.y), ppb[f]);
            } else {
                const uint4 &w0 = pwa[f][0], &w1 = pwa[f][LA - 1];
                prep_pair<KA>(PI ? make_pair(w0.z, w0.w) : make_pair(w0.x, w0.y), PI ? make_pair(w1.z, w1.w) : make_pair(w1.x, w1.y), ppa[f]);
            }
        };
        auto exp_task = [&](auto ec) {
            constexpr int e = decltype(ec)::value;
            if constexpr (e < FM * EA) {
                constexpr int f = e / EA, task = e % EA;
                expand_task<KA, E, task>(word_of(xwa[f][0], XST), word_of(xwa[f][LA - 1], XST), ppa[f], tta[f], km, na[f]);
            } else {
                constexpr int f = (e - FM * EA) / EB, task = (e - FM * EA) % EB;
                expand_task<KB, E, task>(word_of(xwb[f][0], XST), word_of(xwb[f][LB - 1], XST), ppb[f], ttb[f], km, nb[f]);
            }
        };
        static_for<NMI>([&](auto qc) {
            constexpr int q = decltype(qc)::value, i = q / FN, j = q % FN;
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], acc[i][j], 4, 4, 0, sa, 0, sb);
            static_for<T *(q + 1) / NMI - T * q / NMI>([&](auto tc) {
                constexpr int t = T * q / NMI + decltype(tc)::value;
                if constexpr (ODD) {            // preps first: the expansions of this step use them
                    if constexpr (t < T_PREP) prep_task(std::integral_constant<int, t>{});
                    else exp_task(std::integral_constant<int, t - T_PREP>{});
                } else {                        // preps last: they replace what the expansions of this step still read
                    if constexpr (t < T_EXP) exp_task(std::integral_constant<int, t>{});
                    else prep_task(std::integral_constant<int, t - T_EXP>{});
                }
            });
            hook(qc);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto no_hook = [](auto) {};

    // The digit weights 4^da, 4^db enter as the block scales of the instruction
    // (biased exponents 127 + 2 da, 127 + 2 db in every byte), together with the power
    // of two that undoes the halved two-plane codes (out_scale): every digit pair
    // accumulates with its weight of Eq. 1 and the accumulators hold the final integers.
    const int log2_out = p.out_scale == 4.0f ? 2 : p.out_scale == 2.0f ? 1 : 0;

    // Digit pairs in any order (their weights travel with the instruction); all
    // bookkeeping below is branch-free so that the loop body stays one basic block.
    const int total_it = p.DA * p.DB * p.nk;
    int fda = 0, fdb = 0, fk = 0;                       // digit pair / chunk being fetched
    int cda = 0, cdb = 0, ck = 0;                       // digit pair / chunk being computed
    auto advance = [&](int &da, int &db, int &k) {
        ++k;
        const bool wk = k == p.nk;
        k = wk ? 0 : k;
        db += wk ? 1 : 0;
        const bool wb = db == p.DB;
        db = wb ? 0 : db;
        da += wb ? 1 : 0;
    };

    // Pipeline over chunk c (8 steps, words w0 = steps 0-3, w1 = steps 4-7, LDS buffer c & 1):
    //   step 0   reads w1 of chunk c
    //   step 5|6 chunk c + 1 has landed in the other buffer (issued a whole chunk earlier); barrier
    //   step 6   reads w0 of chunk c + 1 and issues the loads of chunk c + 2 into buffer c & 1,
    //            which nobody reads any more
    //   step 7   expands step 0 of chunk c + 1
    uint4 wa0[FM][LA], wb0[FN][LB], wa1[FM][LA], wb1[FN][LB];
    v8i_t ea0[FM], eb0[FN], ea1[FM], eb1[FN];
    FetchState fs;
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    fetch_begin(fs, fda, fdb, fk, total_it > 0);
    static_for<A_SLOTS + B_SLOTS>([&](auto uc) { fetch_one(fs, 0, uc); });
    advance(fda, fdb, fk);
    fetch_begin(fs, fda, fdb, fk, total_it > 1);
    static_for<A_SLOTS + B_SLOTS>([&](auto uc) { fetch_one(fs, 1, uc); });
    advance(fda, fdb, fk);
    __builtin_amdgcn_s_waitcnt(VMCNT0);                 // (waits for chunk 1 as well; only once)
    __syncthreads();
    static_for<NREAD>([&](auto rc) { read_one(0, I0{}, rc, wa0, wb0); });
    // fragments of step 0 of the first chunk
    static_for<FM>([&](auto fc) {
        constexpr int f = decltype(fc)::value;
        prep_pair<KA>(make_pair(wa0[f][0].x, wa0[f][0].y), make_pair(wa0[f][LA - 1].x, wa0[f][LA - 1].y), ppa[f]);
        static_for<EA>([&](auto tc) {
            expand_task<KA, 0, decltype(tc)::value>(wa0[f][0].x, wa0[f][LA - 1].x, ppa[f], tta[f], km, ea0[f]);
        });
    });
    static_for<FN>([&](auto fc) {
        constexpr int f = decltype(fc)::value;
        prep_pair<KB>(make_pair(wb0[f][0].x, wb0[f][0].y), make_pair(wb0[f][LB - 1].x, wb0[f][LB - 1].y), ppb[f]);
        static_for<EB>([&](auto tc) {
            expand_task<KB, 0, decltype(tc)::value>(wb0[f][0].x, wb0[f][LB - 1].x, ppb[f], ttb[f], km, eb0[f]);
        });
    });

#ifdef APNN_BIG_TIMING
    const unsigned long long tt1 = wall_clock64();
#endif
    for (int it = 0; it < total_it; ++it) {
        const int buf = it & 1;
        int sa = 0x7f7f7f7f + 0x02020202 * cda + 0x01010101 * log2_out, sb = 0x7f7f7f7f + 0x02020202 * cdb;
        asm volatile("" : "+v"(sa), "+v"(sb));          // in vector registers before the first portion
        __builtin_amdgcn_sched_barrier(0);
        //   multiply step | expand step (words, index) into | prepare pair (words, which) | memory
        step(I0{}, ea0, eb0, sa, sb, wa0, wb0, I1{}, ea1, eb1, wa0, wb0, I1{}, [&](auto qc) { reads_of(buf, I1{}, qc, wa1, wb1); });
        step(I1{}, ea1, eb1, sa, sb, wa0, wb0, I2{}, ea0, eb0, wa0, wb0, I1{}, no_hook);
        step(I0{}, ea0, eb0, sa, sb, wa0, wb0, I3{}, ea1, eb1, wa1, wb1, I0{}, no_hook);
        step(I1{}, ea1, eb1, sa, sb, wa1, wb1, I0{}, ea0, eb0, wa1, wb1, I0{}, no_hook);
        step(I0{}, ea0, eb0, sa, sb, wa1, wb1, I1{}, ea1, eb1, wa1, wb1, I1{}, no_hook);
        step(I1{}, ea1, eb1, sa, sb, wa1, wb1, I2{}, ea0, eb0, wa1, wb1, I1{}, no_hook);
        __builtin_amdgcn_s_waitcnt(VMCNT0);             // this wave's part of chunk it + 1 is in LDS
        __syncthreads();
        fetch_begin(fs, fda, fdb, fk, it + 2 < total_it);   // beyond the last chunk: zeros, never read
        advance(fda, fdb, fk);
        __builtin_amdgcn_sched_barrier(0);
        step(I0{}, ea0, eb0, sa, sb, wa1, wb1, I3{}, ea1, eb1, wa0, wb0, I0{}, [&](auto qc) {
            reads_of(buf ^ 1, I0{}, qc, wa0, wb0);      // (the A reads come first; prep A of this step, last, uses them)
            loads_of(fs, buf, qc);
        });
        step(I1{}, ea1, eb1, sa, sb, wa0, wb0, I0{}, ea0, eb0, wa0, wb0, I0{}, no_hook);
        advance(cda, cdb, ck);
    }
    __builtin_amdgcn_s_waitcnt(VMCNT0);                 // the loads issued for chunks beyond the last one have landed
#ifdef APNN_BIG_TIMING
    const unsigned long long tt2 = wall_clock64();
#endif

    // ---- epilogue
    if (p.Y && !p.scale) {
        // Plain int32 output, straight from the accumulators: register r of tile (i, j)
        // is row 8 (r / 4) + 4 lh + r % 4, column lr, so one store instruction writes two
        // whole 128-byte row segments.  Buffer stores with the whole byte offset (row and
        // column) in the per-lane offset, the only part the hardware checks against the
        // descriptor's size: rows beyond M land beyond the M x N bytes and are dropped,
        // columns beyond N are sent out of range explicitly; no branches, no waits, the
        // stores stream out behind the conversions.  The host guarantees (M + BM) N 4 < 2^31,
        // so adding a row offset never carries into the out-of-range bit.
        const __amdgpu_buffer_rsrc_t rsrcY =
            __builtin_amdgcn_make_buffer_rsrc(p.Y, 0, 4u * static_cast<uint32_t>(p.M) * p.N, 0x00020000);
        const int gn0 = n0 + wn * FN * 32 + lr;
        const uint32_t vbase = 4u * (static_cast<uint32_t>(m0 + wm * FM * 32 + 4 * lh) * p.N + gn0);
        uint32_t voffY[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j) voffY[j] = (vbase + 128u * j) | (gn0 + 32 * j < p.N ? 0u : OUT_OF_RANGE);
        static_for<FM * FN * 16>([&](auto c) {
            // (the FN tiles of a row one after the other: FN x 128 contiguous bytes of a row leave together)
            constexpr int i = decltype(c)::value / (FN * 16), r = decltype(c)::value / FN % 16, j = decltype(c)::value % FN;
            constexpr int row = i * 32 + 8 * (r >> 2) + (r & 3);
            __builtin_amdgcn_raw_buffer_store_b32(static_cast<int>(acc[i][j][r]) + p.c0, rsrcY,
                                                  voffY[j] + 4u * row * static_cast<uint32_t>(p.N), 0, 0);
        });
#ifdef APNN_BIG_TIMING
        // Instrumented build only (-DAPNN_BIG_TIMING, `python bench.py --phases`): every wave leaves the time stamps
        // of its entry, the start and the end of its main loop, its last store instruction and the acknowledgement
        // of its stores in the buffer that p.T points at (8 x 64 bits per wave; apnn_gemm takes the address from
        // the environment variable APNN_DBG_PTR in such a build).
        {
            const unsigned long long tt3 = wall_clock64();
            __builtin_amdgcn_s_waitcnt(0);              // all stores of this wave have been acknowledged
            const unsigned long long tt4 = wall_clock64();
            if (lane == 0 && p.T) {
                unsigned long long *d = reinterpret_cast<unsigned long long *>(p.T) + (static_cast<size_t>(blockIdx.x) * NW + wave) * 8;
                d[0] = tt0; d[1] = tt1; d[2] = tt2; d[3] = tt3; d[4] = tt4;
            }
        }
#endif
        return;
    }
    MfmaParams pe = p;                                  // the scale is already in the accumulators
    pe.out_scale = 1.0f;
    static_for<FN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int gn = n0 + wn * FN * 32 + j * 32 + lr;
        float sc = 0.0f, bi = 0.0f;
        if (p.scale && gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
        static_for<FM * 4>([&](auto ikc) {
            constexpr int i = decltype(ikc)::value / 4, k = decltype(ikc)::value % 4;
            const int row0 = m0 + wm * FM * 32 + i * 32 + 8 * k;
            const float v4[4] = {acc[i][j][4 * k], acc[i][j][4 * k + 1], acc[i][j][4 * k + 2], acc[i][j][4 * k + 3]};
            finish_rows8(pe, v4, row0, gn, sc, bi, load_res_rows8(pe, row0, gn >> 5, lane), lane, lr, lh);
        });
    });
}

}  // namespace apnn
