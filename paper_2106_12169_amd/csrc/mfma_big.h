// Matrix-core kernel for large matrix-layout products (block tile 256 x 256).
//
// Same arithmetic, operand encodings, digit passes and epilogue as
// mfma_fp4_kernel; what differs is the schedule of the main loop, which at this
// size decides the run time:
//   - every wave owns FM x FN = 4 x 4 matrix-instruction tiles (128 x 128 outputs),
//     so one expansion of a plane word into FP4 codes feeds four matrix
//     instructions; the 256 accumulator registers per lane live in the
//     accumulation half of the unified register file (one wave per SIMD);
//   - the loader addresses global memory as a uniform base plus a 32-bit lane
//     offset (operands larger than 4 GiB are left to the other kernels by the
//     host) and clamps rows beyond M / N to the last row instead of predicating;
//   - the LDS words of the second half of a chunk are read while the first half is
//     multiplied, and the next chunk is written to the other LDS buffer between the
//     two halves, so that only the first read after the barrier is exposed;
//   - the expansion uses the K order "nibble i of dword r holds the element at bit
//     4 i + rho(r)", rho = (0, 2, 1, 3), which lets a two-plane digit be interleaved
//     pairwise first (10 instead of 14 instructions per 32 values).
#pragma once
#include "mfma_kernel.h"

namespace apnn {

struct Fp4Masks2 { uint32_t m2, m3, m5, m8; };

// 32 K positions of one operand row -> 4 dwords of 8 FP4 codes; nibble i of dword
// r holds the element at bit 4 i + rho(r), rho = (0, 2, 1, 3), of the plane words.
// HALF selects dwords 0-1 or 2-3, so that the work can be dealt out in small
// portions between matrix instructions (3 to 5 vector instructions per half).
template <int KIND, int HALF> __device__ __forceinline__ void expand_fp4_half(uint32_t x0, uint32_t x1, const Fp4Masks2 &k, v8i_t &out)
{
    if (KIND == OPK_U1) {                       // 0 -> 0000 (0.0), 1 -> 0010 (1.0)
        if (HALF == 0) { out[0] = (x0 << 1) & k.m2; out[1] = (x0 >> 1) & k.m2; }
        else           { out[2] = x0 & k.m2;        out[3] = (x0 >> 2) & k.m2; }
    } else if (KIND == OPK_PM1) {               // 1 -> 0010 (+1.0), 0 -> 1010 (-1.0)
        if (HALF == 0) { out[0] = (~(x0 << 3) & k.m8) | k.m2; out[1] = (~(x0 << 1) & k.m8) | k.m2; }
        else           { out[2] = (~(x0 << 2) & k.m8) | k.m2; out[3] = (~x0 & k.m8) | k.m2; }
    } else {                                    // code = x1 x0 = value / 2
        // (a & m5) | (b & ~m5) as one three-input bit operation (truth table a:0xF0, b:0xCC, mask:0xAA)
        constexpr int SEL = (0xF0 & 0xAA) | (0xCC & 0x55);
        if (HALF == 0) {
            const uint32_t ze = __builtin_amdgcn_bitop3_b32(x0, x1 << 1, k.m5, SEL);     // pairs of the even positions
            out[0] = ze & k.m3;
            out[1] = (ze >> 2) & k.m3;
        } else {
            const uint32_t zo = __builtin_amdgcn_bitop3_b32(x0 >> 1, x1, k.m5, SEL);     // pairs of the odd positions
            out[2] = zo & k.m3;
            out[3] = (zo >> 2) & k.m3;
        }
    }
    if (HALF == 1) out[4] = out[5] = out[6] = out[7] = 0;
}

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int i)
{
    return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

template <int KA, int KB, int NWM, int NWN, int FM, int FN>
__global__ __launch_bounds__(64 * NWM * NWN, 1) void mfma_big_kernel(const MfmaParams p)
{
    constexpr int KC = 16;                              // words per chunk = 8 matrix-instruction steps = 2 groups of 4
    constexpr int NT = 64 * NWM * NWN;
    constexpr int LA = DigitPlanes<KA>::value, LB = DigitPlanes<KB>::value;
    constexpr int BM = NWM * FM * 32, BN = NWN * FN * 32;
    constexpr int RSA = LA * KC + 4, RSB = LB * KC + 4; // padded LDS row strides (words)
    constexpr int A_VECS = BM * LA * (KC / 4), B_VECS = BN * LB * (KC / 4);
    static_assert(A_VECS % NT == 0 && B_VECS % NT == 0, "every loader slot is full");
    static_assert(NT % (4 * LA) == 0 && NT % (4 * LB) == 0, "all slots of a thread share piece and plane");
    constexpr int A_SLOTS = A_VECS / NT, B_SLOTS = B_VECS / NT;

    constexpr int TILE_WORDS = 2 * BM * RSA + 2 * BN * RSB;
    __shared__ __attribute__((aligned(16))) uint32_t smem[TILE_WORDS];
    uint32_t (*sA)[BM * RSA] = reinterpret_cast<uint32_t (*)[BM * RSA]>(smem);
    uint32_t (*sB)[BN * RSB] = reinterpret_cast<uint32_t (*)[BN * RSB]>(smem + 2 * BM * RSA);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave % NWN;
    const int lr = lane & 31, lh = lane >> 5;

    const int tilesN = (p.N + BN - 1) / BN;
    const int m0 = (blockIdx.x / tilesN) * BM, n0 = (blockIdx.x % tilesN) * BN;

    Fp4Masks2 km;
    km.m2 = reg_const(0x22222222u); km.m3 = reg_const(0x33333333u);
    km.m5 = reg_const(0x55555555u); km.m8 = reg_const(0x88888888u);

    // ---- loader: slot u of thread tid covers vector v = tid + NT u = (row * L + plane) * 4 + piece.
    // Buffer loads: descriptor base (scalar) + per-lane byte offset (constant over the
    // whole loop) + scalar offset of (digit plane, chunk); a lane whose piece or plane
    // does not exist uses an offset beyond the descriptor's range and receives zeros.
    const uint32_t bytesA = 4u * static_cast<uint32_t>(p.M) * p.PA * p.ldwA, bytesB = 4u * static_cast<uint32_t>(p.N) * p.PB * p.ldwB;
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.A), 0, bytesA, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.B), 0, bytesB, 0x00020000);
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;      // operands are smaller than 2 GiB (host check)
    uint32_t offA[A_SLOTS], offB[B_SLOTS];              // byte offsets of (row, plane of digit 0, piece) in chunk 0
#pragma unroll
    for (int u = 0; u < A_SLOTS; ++u) {
        const int v = tid + NT * u, c = v % 4, rp = v / 4;
        const int gm = min(m0 + rp / LA, p.M - 1);
        offA[u] = 4u * ((static_cast<uint32_t>(gm) * p.PA + rp % LA) * p.ldwA + 4 * c);
    }
#pragma unroll
    for (int u = 0; u < B_SLOTS; ++u) {
        const int v = tid + NT * u, c = v % 4, rp = v / 4;
        const int gn = min(n0 + rp / LB, p.N - 1);
        offB[u] = 4u * ((static_cast<uint32_t>(gn) * p.PB + rp % LB) * p.ldwB + 4 * c);
    }
    typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));
    v4u_t ra[A_SLOTS], rb[B_SLOTS];
    // piece and plane of a slot are the same for all slots of a thread (NT is a multiple of 4 L)
    const int my_c4 = 4 * (tid % 4), my_plA = (tid / 4) % LA, my_plB = (tid / 4) % LB;
    struct FetchState { int soffA, soffB; uint32_t badA, badB; };
    auto fetch_begin = [&](FetchState &fs, int da, int db, int kc, bool live) {
        const int pa0 = LA == 2 ? 2 * da : da, pb0 = LB == 2 ? 2 * db : db;       // first plane of the digit
        fs.soffA = 4 * (pa0 * p.ldwA + kc * KC);
        fs.soffB = 4 * (pb0 * p.ldwB + kc * KC);
        const int okK = static_cast<int>(live) & static_cast<int>(my_c4 < p.Kw - kc * KC);
        fs.badA = (okK & static_cast<int>(my_plA < p.PA - pa0)) ? 0u : OUT_OF_RANGE;
        fs.badB = (okK & static_cast<int>(my_plB < p.PB - pb0)) ? 0u : OUT_OF_RANGE;
    };
    auto fetch_one = [&](const FetchState &fs, auto uc) {        // slot u: A slots first, then B slots
        constexpr int u = decltype(uc)::value;
        if constexpr (u < A_SLOTS) ra[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, offA[u] | fs.badA, fs.soffA, 0);
        else rb[u - A_SLOTS] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, offB[u - A_SLOTS] | fs.badB, fs.soffB, 0);
    };
    auto stage_one = [&](int buf, auto uc) {
        constexpr int u = decltype(uc)::value;
        if constexpr (u < A_SLOTS) {
            const int v = tid + NT * u, c = v % 4, rp = v / 4;
            *reinterpret_cast<v4u_t *>(&sA[buf][(rp / LA) * RSA + (rp % LA) * KC + 4 * c]) = ra[u];
        } else {
            const int v = tid + NT * (u - A_SLOTS), c = v % 4, rp = v / 4;
            *reinterpret_cast<v4u_t *>(&sB[buf][(rp / LB) * RSB + (rp % LB) * KC + 4 * c]) = rb[u - A_SLOTS];
        }
    };

    v16f_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // ---- one step = FM x FN matrix instructions on the FP4 fragments of 64 K positions.
    // The fragments of step s + 1 are expanded while the matrix instructions of step s
    // run.  A lone wave per SIMD only overlaps the two if they alternate finely in its
    // instruction stream (measured: about 4 vector instructions hide behind each matrix
    // instruction, a longer run of vector work stalls the matrix pipe), so the step is
    // written as FM FN portions "one matrix instruction, a half-fragment expansion, at
    // most one memory instruction", each fenced against instruction scheduling.
    // The digit weights 4^da, 4^db enter as the block scales of the instruction
    // (biased exponents 127 + 2 da, 127 + 2 db in every byte): every digit pair
    // accumulates with its weight of Eq. 1 and the accumulators are never touched by
    // anything but the matrix unit until the epilogue.  The power of two that undoes
    // the halved two-plane codes (out_scale) is folded into the A-side scale as well,
    // so the accumulators hold the final integers.
    const int log2_out = p.out_scale == 4.0f ? 2 : p.out_scale == 2.0f ? 1 : 0;
    constexpr int NMI = FM * FN, NHALF = 2 * (FM + FN);
    auto step = [&](const v8i_t (&fa)[FM], const v8i_t (&fb)[FN], int sa, int sb,            // fragments of this step
                    const uint4 (&wa)[FM][LA], const uint4 (&wb)[FN][LB], auto stc,         // words / step index of the next one
                    v8i_t (&na)[FM], v8i_t (&nb)[FN], auto &&hook) {
        constexpr int st = decltype(stc)::value;
        static_for<NMI>([&](auto qc) {
            constexpr int q = decltype(qc)::value, i = q / FN, j = q % FN;
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], acc[i][j], 4, 4, 0, sa, 0, sb);
            static_for<NHALF *(q + 1) / NMI - NHALF * q / NMI>([&](auto hc) {
                constexpr int h = NHALF * q / NMI + decltype(hc)::value, fr = h / 2, half = h % 2;
                if constexpr (fr < FM) expand_fp4_half<KA, half>(word_of(wa[fr][0], st), word_of(wa[fr][LA - 1], st), km, na[fr]);
                else expand_fp4_half<KB, half>(word_of(wb[fr - FM][0], st), word_of(wb[fr - FM][LB - 1], st), km, nb[fr - FM]);
            });
            hook(qc);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto no_hook = [](auto) {};

    // one LDS read of a group per portion: read r covers (fragment row f, plane pl) of A, then of B
    auto read_one = [&](int buf, int g, auto rc, uint4 (&wa)[FM][LA], uint4 (&wb)[FN][LB]) {
        constexpr int r = decltype(rc)::value;
        if constexpr (r < FM * LA) {
            constexpr int f = r / LA, pl = r % LA;
            wa[f][pl] = *reinterpret_cast<const uint4 *>(&sA[buf][(wm * FM * 32 + f * 32 + lr) * RSA + pl * KC + 8 * lh + 4 * g]);
        } else if constexpr (r < FM * LA + FN * LB) {
            constexpr int f = (r - FM * LA) / LB, pl = (r - FM * LA) % LB;
            wb[f][pl] = *reinterpret_cast<const uint4 *>(&sB[buf][(wn * FN * 32 + f * 32 + lr) * RSB + pl * KC + 8 * lh + 4 * g]);
        }
    };
    constexpr int NREAD = FM * LA + FN * LB;
    static_assert(NREAD <= NMI && A_SLOTS + B_SLOTS <= NMI, "one memory instruction of each kind per portion");

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
    //   step 3   writes chunk c + 1 (registers -> other LDS buffer) and fetches chunk c + 2 into the registers
    //   step 5|6 barrier
    //   step 6   reads w0 of chunk c + 1
    //   step 7   expands step 0 of chunk c + 1
    uint4 wa0[FM][LA], wb0[FN][LB], wa1[FM][LA], wb1[FN][LB];
    v8i_t ea0[FM], eb0[FN], ea1[FM], eb1[FN];
    FetchState fs;
    fetch_begin(fs, fda, fdb, fk, total_it > 0);
    static_for<A_SLOTS + B_SLOTS>([&](auto uc) { fetch_one(fs, uc); });
    advance(fda, fdb, fk);
    static_for<A_SLOTS + B_SLOTS>([&](auto uc) { stage_one(0, uc); });
    fetch_begin(fs, fda, fdb, fk, total_it > 1);
    static_for<A_SLOTS + B_SLOTS>([&](auto uc) { fetch_one(fs, uc); });
    advance(fda, fdb, fk);
    __syncthreads();
    static_for<NREAD>([&](auto rc) { read_one(0, 0, rc, wa0, wb0); });
    static_for<FM>([&](auto fc) {
        constexpr int f = decltype(fc)::value;
        expand_fp4_half<KA, 0>(wa0[f][0].x, wa0[f][LA - 1].x, km, ea0[f]);
        expand_fp4_half<KA, 1>(wa0[f][0].x, wa0[f][LA - 1].x, km, ea0[f]);
    });
    static_for<FN>([&](auto fc) {
        constexpr int f = decltype(fc)::value;
        expand_fp4_half<KB, 0>(wb0[f][0].x, wb0[f][LB - 1].x, km, eb0[f]);
        expand_fp4_half<KB, 1>(wb0[f][0].x, wb0[f][LB - 1].x, km, eb0[f]);
    });

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    for (int it = 0; it < total_it; ++it) {
        const int buf = it & 1;
        int sa = 0x7f7f7f7f + 0x02020202 * cda + 0x01010101 * log2_out, sb = 0x7f7f7f7f + 0x02020202 * cdb;
        asm volatile("" : "+v"(sa), "+v"(sb));          // in vector registers before the first portion
        __builtin_amdgcn_sched_barrier(0);
        step(ea0, eb0, sa, sb, wa0, wb0, I1{}, ea1, eb1, [&](auto qc) { read_one(buf, 1, qc, wa1, wb1); });
        step(ea1, eb1, sa, sb, wa0, wb0, I2{}, ea0, eb0, no_hook);
        step(ea0, eb0, sa, sb, wa0, wb0, I3{}, ea1, eb1, no_hook);
        fetch_begin(fs, fda, fdb, fk, it + 2 < total_it);   // beyond the last chunk: zeros, staged but never read
        advance(fda, fdb, fk);
        __builtin_amdgcn_sched_barrier(0);
        step(ea1, eb1, sa, sb, wa1, wb1, I0{}, ea0, eb0, [&](auto qc) {
            if constexpr (decltype(qc)::value < A_SLOTS + B_SLOTS) {
                stage_one(buf ^ 1, qc);                 // that buffer was last read before the previous barrier
                fetch_one(fs, qc);
            }
        });
        step(ea0, eb0, sa, sb, wa1, wb1, I1{}, ea1, eb1, no_hook);
        step(ea1, eb1, sa, sb, wa1, wb1, I2{}, ea0, eb0, no_hook);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        step(ea0, eb0, sa, sb, wa1, wb1, I3{}, ea1, eb1, [&](auto qc) { read_one(buf ^ 1, 0, qc, wa0, wb0); });
        step(ea1, eb1, sa, sb, wa0, wb0, I0{}, ea0, eb0, no_hook);
        advance(cda, cdb, ck);
    }

    // ---- epilogue
    constexpr int WN = FN * 32;                         // columns of a wave tile
    constexpr int SLAB_STRIDE = WN + 4;                 // words; the pad keeps the two lane halves on different banks
    static_assert(NWM * NWN * 32 * SLAB_STRIDE <= TILE_WORDS, "the output slabs reuse the operand tiles");
    if (p.Y && !p.scale && (p.N & 3) == 0) {
        // Plain int32 output.  A lane's accumulators are 128-byte row fragments
        // scattered over 16 rows per tile; every wave transposes them through an LDS
        // slab of its own (32 rows x WN columns at a time; the operand tiles are dead),
        // so that the stores leave as whole WN-column row segments, 16 bytes per lane.
        // A wave's LDS accesses are served in order, so no barrier is needed between
        // its writes and reads, and the waves of a block drain independently.
        __syncthreads();                                // every wave is done with the operand tiles
        int32_t *slab = reinterpret_cast<int32_t *>(smem) + wave * 32 * SLAB_STRIDE;
        const int row_l = lane / (WN / 4), c4_l = (lane % (WN / 4)) * 4;       // this lane's (row, column) in a 64-vector sweep
        constexpr int ROWS_PER_SWEEP = 64 / (WN / 4), SWEEPS = 32 / ROWS_PER_SWEEP;
        // Buffer stores: rows beyond M fall outside the descriptor and are dropped by
        // the hardware; columns beyond N are sent out of range explicitly.  The host
        // guarantees (M + BM) N 4 < 2^31.
        const __amdgpu_buffer_rsrc_t rsrcY =
            __builtin_amdgcn_make_buffer_rsrc(p.Y, 0, 4u * static_cast<uint32_t>(p.M) * p.N, 0x00020000);
        const int gn = n0 + wn * WN + c4_l;
        const uint32_t voffY = (4u * (static_cast<uint32_t>(m0 + wm * FM * 32 + row_l) * p.N + gn)) | (gn < p.N ? 0u : OUT_OF_RANGE);
        static_for<FM>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            static_for<FN * 16>([&](auto jrc) {
                constexpr int j = decltype(jrc)::value / 16, r = decltype(jrc)::value % 16;
                slab[(8 * (r >> 2) + 4 * lh + (r & 3)) * SLAB_STRIDE + j * 32 + lr] = static_cast<int>(acc[i][j][r]) + p.c0;
            });
            v4u_t rows[SWEEPS];
            static_for<SWEEPS>([&](auto sc) {
                constexpr int sw = decltype(sc)::value;
                rows[sw] = *reinterpret_cast<const v4u_t *>(&slab[(sw * ROWS_PER_SWEEP + row_l) * SLAB_STRIDE + c4_l]);
            });
            static_for<SWEEPS>([&](auto sc) {
                constexpr int sw = decltype(sc)::value;
                __builtin_amdgcn_raw_buffer_store_b128(rows[sw], rsrcY, voffY, 4 * (i * 32 + sw * ROWS_PER_SWEEP) * p.N, 0);
            });
        });
        return;
    }
    MfmaParams pe = p;                                  // the scale is already in the accumulators
    pe.out_scale = 1.0f;
    static_for<FN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int gn = n0 + wn * FN * 32 + j * 32 + lr;
        float sc = 0.0f, bi = 0.0f;
        if (p.scale && gn < p.N) { sc = p.scale[gn]; bi = p.bias[gn]; }
        static_for<FM * 16>([&](auto irc) {
            constexpr int i = decltype(irc)::value / 16, r = decltype(irc)::value % 16;
            finish_value(pe, acc[i][j][r], m0 + wm * FM * 32 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3), gn, sc, bi, false, 0u, lr, lh);
        });
    });
}

}  // namespace apnn
