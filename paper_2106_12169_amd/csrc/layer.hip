// Host side of apnn_gemm / apnn_conv2d / apnn_layer: argument validation,
// encoding recovery constants (Sec. 3.2), tile choice (Sec. 4.3) and launch.
#include <atomic>
#include <cstdlib>
#include <cstring>

#include "../../include/apnn_debug.h"
#include "common.h"
#include "mfma_launch.h"
#include "tile_launch.h"

namespace apnn {

// Kernel-choice overrides (tests, experiments).  Each is read from the process
// environment once, the first time any of them is asked for, and can afterwards be
// set or cleared through apnn_debug_force; the dispatch itself only loads an int.
enum Override { OV_MFMA, OV_TILE, OV_MFMA_TILE, OV_MFMA_SHORTK, OV_MFMA_SMALL, OV_MFMA_NSPLIT, OV_MFMA_FN, OV_INT8, OV_COUNT };
static const char *const kOverrideNames[OV_COUNT] = {"MFMA", "TILE", "MFMA_TILE", "MFMA_SHORTK", "MFMA_SMALL",
                                                     "MFMA_NSPLIT", "MFMA_FN", "INT8"};
static std::atomic<int> g_override[OV_COUNT];

static void overrides_from_env()
{
    for (int i = 0; i < OV_COUNT; ++i) {
        char name[40] = "APNN_";
        std::strncat(name, kOverrideNames[i], sizeof(name) - 6);
        const char *e = std::getenv(name);
        g_override[i].store(e && *e ? std::atoi(e) : -1, std::memory_order_relaxed);
    }
}

// Value of an override, -1 when it is not set.
static int ov(Override which)
{
    static const bool once = (overrides_from_env(), true);
    (void)once;
    return g_override[which].load(std::memory_order_relaxed);
}

// Tile choice, the two-step heuristic of Sec. 4.3.  Candidates are ranked by thread-level parallelism (Eq. 3; here
// the number of blocks: plane pairs are batched in time, not space, so p q does not multiply it).  If even the most
// parallel candidate stays below its threshold it is taken; otherwise the candidate of the highest compute intensity
// (Eq. 4, 2 bm bn / (bm + bn)) whose parallelism still reaches its threshold.  The paper uses one threshold, T = 64,
// for its 82 multiprocessors; here each candidate carries the block count from which it measured faster on the 256
// compute units of MI355X, and the share of its area that must be real output (ragged edges).
struct TileCandidate { int edge; int64_t min_blocks; double min_useful; };

static int rank_tiles(const TileCandidate *cand, int n, int64_t M, int64_t N)
{
    int best = cand[0].edge;                    // the head of the priority queue: highest parallelism
    double best_ci = 0.0;
    for (int i = 0; i < n; ++i) {
        const int64_t e = cand[i].edge, blocks = ceil_div(M, e) * ceil_div(N, e);
        const double useful = static_cast<double>(M) * N / (static_cast<double>(blocks) * e * e);
        const double ci = 2.0 * e * e / (e + e);
        if (i > 0 && (blocks < cand[i].min_blocks || useful < cand[i].min_useful)) continue;
        if (ci > best_ci) { best_ci = ci; best = cand[i].edge; }
    }
    return best;
}

// AND+popcount kernel.  Measured: the 64 x 64 tile (4 waves per SIMD) matches or beats the 128 x 128 tile (2 waves per
// SIMD) from 1024^2 outputs up, because the extra resident waves cover block start-up and drain, so 128 is no
// candidate; below one block per compute unit the 32 x 32 tile recovers parallelism.
// The TILE override (8, 4 or 2: the per-thread edge) replaces the choice (experiments, tests).
static int pick_tile(int64_t M, int64_t N)
{
    if (const int r = ov(OV_TILE); r == 8 || r == 4 || r == 2) return r;
    static const TileCandidate cand[] = {{32, 0, 0.0}, {64, 256, 0.0}};
    return rank_tiles(cand, 2, M, N) / 16;
}

struct Problem {
    const char *who;
    bool conv;
    int64_t M, N, Ktotal;      // rows, columns, logical reduction length
    int PA, PB;
    apnn_encoding encA, encB;
};

// ---- FP4 matrix-core path --------------------------------------------------------
// Applies when every partial sum stays an exact fp32 integer
// (K max|a| max|b| < 2^24), the encodings are ones the kernel has a digit kind
// for, and (convolution) the channel count allows 8-byte loader vectors.
// The MFMA override set to 0 forces the AND+popcount kernel (the literal AP-Bit emulation).
static bool mfma_kind(int planes, apnn_encoding enc, int &kind, int &digits, int64_t &maxabs)
{
    if (enc == APNN_ENC_PM1) { kind = OPK_PM1; digits = 1; maxabs = 1; return planes == 1; }
    kind = planes == 1 ? OPK_U1 : OPK_U2;
    digits = (planes + 1) / 2;
    maxabs = (int64_t(1) << planes) - 1;
    return true;
}

static int pick_mfma_tile(int64_t M, int64_t N, bool conv)
{
    if (const int t = ov(OV_MFMA_TILE); t == 32 || t == 64 || t == 128 || (t == 256 && !conv)) return t;
    // Convolutions: the lane-private small-layer kernel at every size.  Measured on the ResNet-18 shapes at batch
    // 128 it matches or beats the LDS-staged 64 x 64 and 128 x 128 tiles layer by layer (stage 1: 59 - 73 us against
    // 70 - 87; stage 2: 25 - 42 against 27 - 59), because their gather through registers and LDS costs more
    // instructions than the matrix instructions it feeds.
    if (conv) return 32;
    // Matrices: 32 (one wave tile per block, K split over its waves) is the head of the queue; larger tiles need most
    // of the 256 compute units to get a block and at most a quarter of their area wasted on ragged edges.
    static const TileCandidate cand[] = {{32, 0, 0.0}, {64, 1024, 0.0}, {128, 192, 0.75}, {256, 192, 0.75}};
    return rank_tiles(cand, 4, M, N);
}

// ---- 8-bit integer matrix path (matrix operands) -------------------------------------
// One pass over K whatever p and q are (the FP4 form needs ceil(p/2) ceil(q/2)), exact for every K the int32
// result allows.  Its cost is the transposition of plane words into bytes, which grows with the plane counts, so it
// is taken where it measured faster on 2048^3 ... 4096^3 products: five or more FP4 passes; four with both operands
// above two bits (w3a5 24 against 37 us, w4a4 21 against 27 at 2048^3); four with a narrow operand (w2a8, w1a7) only up
// to one 128 x 128 tile per compute unit (2048^3: 24.7 against 27.0 us; 3072^3: 89 against 81, 4096^3: 144 against
// 117, where the FP4 form runs its 256 x 256 tiles) -- given enough tiles to occupy the chip, and whenever the FP4
// form could not be exact (w8a8, K = 2048: 40 us against 1040 us of the AND+popcount kernel).  Override INT8: 0 never, 1 whenever it applies, 2 and 3
// the same with the kernel that shares out the outputs / K among the waves.
struct I8Operand { int cls; int alpha, off, flipped, pad; uint32_t flip; };

static I8Operand i8_operand(int planes, apnn_encoding enc)
{
    I8Operand o{};
    o.cls = planes <= 2 ? 0 : planes <= 4 ? 1 : 2;
    if (enc == APNN_ENC_PM1) {            // the stored bit b stands for 2 b - 1
        o.alpha = 2; o.off = -1;
    } else if (planes == 8) {             // the byte is value - 128 (top plane inverted)
        o.alpha = 1; o.off = 128; o.flipped = 128; o.pad = -128; o.flip = ~0u;
    } else {
        o.alpha = 1;
    }
    return o;
}

static bool try_int8(const Problem &pr, MfmaParams &mp, bool fp4_exact, void *stream, int &rc)
{
    const int force = ov(OV_INT8);
    if (force == 0 || ov(OV_MFMA) == 0 || pr.conv || pr.Ktotal <= 0) return false;
    const int64_t tiles = ceil_div(pr.M, 128) * ceil_div(pr.N, 128);
    if (force < 1) {
        const int passes = ((pr.PA + 1) / 2) * ((pr.PB + 1) / 2);
        const bool faster = passes >= 5 || (passes == 4 && ((pr.PA > 2 && pr.PB > 2) || tiles <= 256));
        if (fp4_exact && (!faster || tiles < 64)) return false;
    }
    const int64_t lim = int64_t(1) << 31;       // operands and output are addressed with 31-bit byte offsets
    if (4 * pr.M * pr.PA * mp.ldwA >= lim || 4 * pr.N * pr.PB * mp.ldwB >= lim || 4 * (pr.M + 128) * pr.N >= lim) return false;
    if (tiles > 0x7FFFFFFF) return false;
    const I8Operand a = i8_operand(pr.PA, pr.encA), b = i8_operand(pr.PB, pr.encB);
    mp.PA = pr.PA; mp.PB = pr.PB;
    mp.nk = static_cast<int>(round_up(ceil_div(mp.Kw, 4), 4));       // chunks of 4 words; the kernel takes four per loop pass
    const int64_t K = pr.Ktotal, npad = static_cast<int64_t>(mp.nk) * 128 - K;
    mp.flipA = a.flip; mp.flipB = b.flip;
    mp.accmul = a.alpha * b.alpha;
    mp.mulA = a.alpha * b.off;
    mp.mulB = b.alpha * a.off;
    // (wrapping 32-bit arithmetic, as in the kernel: the terms cancel to a result that fits)
    mp.c0 = static_cast<int>(static_cast<uint32_t>(-static_cast<int64_t>(a.alpha) * b.alpha * npad * a.pad * b.pad
                                                   - static_cast<int64_t>(a.alpha) * b.off * a.flipped * K
                                                   - static_cast<int64_t>(b.alpha) * a.off * b.flipped * K
                                                   + K * a.off * b.off));
    mp.out_scale = 1.0f;
    mp.xcd_regions = (ceil_div(pr.M, 128) % 2 == 0 && ceil_div(pr.N, 128) % 4 == 0) ? 1 : 0;
    // K shared out among the waves of a block (half the transposition work per matrix instruction, but one wave per
    // SIMD and four partial results to add): measured faster from K of about 3000 up (2048 x 2048 outputs, w4a4:
    // K = 2048 22.1 against 20.8 us, 4096 30.8 against 32.1, 8192 49.4 against 56.5; w3a5 4096^3 128 against 136).
    // Override INT8 = 2: never, 3: whenever the planes fit its LDS.
    const bool wide = force != 2 && pr.PA + pr.PB <= 10 && !(a.cls == 2 && b.cls == 2) && (force == 3 || K >= 3072);
    if (!(wide && launch_mfma_i8_wide(mp, a.cls, b.cls, static_cast<unsigned>(tiles), as_stream(stream))) &&
        !launch_mfma_i8(mp, a.cls, b.cls, static_cast<unsigned>(tiles), as_stream(stream)))
        return false;
    rc = check_launch(pr.who);
    return true;
}

// What the dispatch decided for a layer that takes the small-layer convolution kernel with K split over the
// waves of a block: filled in instead of launching when a caller wants to put two such layers into one launch.
struct SmallPlan {
    bool ok;
    MfmaParams mp;
    int kA, kB, vw, gmax;
    unsigned grid;
};

// Returns true if the launch was issued (status in rc), false if the path does not apply.  With a plan, nothing is
// launched: the plan is filled in if the layer takes the small-layer convolution kernel, and left not ok otherwise.
static bool try_mfma(const Problem &pr, MfmaParams &mp, void *stream, int &rc, SmallPlan *plan)
{
    if (ov(OV_MFMA) == 0) return false;
    int kA, kB;
    int64_t maxA, maxB;
    if (!mfma_kind(pr.PA, pr.encA, kA, mp.DA, maxA) || !mfma_kind(pr.PB, pr.encB, kB, mp.DB, maxB)) return false;
    // (a pooled sum adds four results before the conversion to an integer)
    const bool fp4_exact = pr.Ktotal > 0 && round_up(pr.Ktotal, 1024) * maxA * maxB * (mp.pool == 2 ? 4 : 1) < (int64_t(1) << 24);
    if (!plan && try_int8(pr, mp, fp4_exact, stream, rc)) return true;
    if (!fp4_exact) return false;
    if (pr.conv && mp.Cw % 2 != 0) return false;
    if (pr.conv && kA == OPK_PM1) kA = OPK_PM1Z;         // -1/+1 features: taps outside the frame must contribute 0
    mp.PA = pr.PA; mp.PB = pr.PB;
    mp.out_scale = (kA == OPK_U2 ? 2.0f : 1.0f) * (kB == OPK_U2 ? 2.0f : 1.0f);
    // 0 pad bits of two -1/+1 operands multiply to +1 at every padded K position
    int t = pick_mfma_tile(pr.M, pr.N, pr.conv);
    if (kA == OPK_PM1Z && t == 128) t = 64;              // instantiated for the 64-tile and the small-layer kernel
    if ((t == 256 || t == 128) && !pr.conv) {   // the pipelined kernel addresses operands and output with 31-bit byte offsets
        const int64_t lim = int64_t(1) << 31;
        if (4 * pr.M * pr.PA * mp.ldwA >= lim || 4 * pr.N * pr.PB * mp.ldwB >= lim || 4 * (pr.M + 256) * pr.N >= lim) t = 64;
    }
    // 8-word chunks: no step multiplies padding (override 0: no special case for short K)
    const bool short_k = !pr.conv && mp.Kw <= 8 && t <= 64 && ov(OV_MFMA_SHORTK) != 0;
    if (short_k) t = 64;
    const int kc = short_k ? 8 : mfma_chunk_words(t);
    mp.nk = static_cast<int>(ceil_div(mp.Kw, kc));
    mp.c0 = (kA == OPK_PM1 && kB == OPK_PM1) ? -static_cast<int>(static_cast<int64_t>(mp.nk) * kc * 32 - pr.Ktotal) : 0;
    const int64_t tiles = ceil_div(pr.M, t) * ceil_div(pr.N, t);
    if (tiles > 0x7FFFFFFF) return false;
    const unsigned grid = static_cast<unsigned>(tiles);
    bool ok;
    if (t == 32 && ov(OV_MFMA_SMALL) != 0) {                           // small layer: lane-private loads, no LDS staging (0: chunked kernel)
        int nsplit = tiles <= 4096 ? 4 : 1;                            // measured: the split wins up to a few thousand tiles
        if (const int en = ov(OV_MFMA_NSPLIT); en == 1 || en == 4) nsplit = en;
        const int64_t nse = round_up(ceil_div(mp.Kw, 2), 4);          // steps of the small-layer kernel (groups of four)
        mp.nk = 1;
        mp.c0 = (kA == OPK_PM1 && kB == OPK_PM1) ? -static_cast<int>(nse * 64 - pr.Ktotal) : 0;
        // Large convolution layers (one wave tile per wave): 32 x 64 wave tiles, so that the row operand is loaded,
        // decoded and expanded once for 64 output channels.
        int fn = 1;
        if (pr.conv && nsplit == 1) fn = pr.N % 64 == 0 ? 2 : 1;
        if (const int f = ov(OV_MFMA_FN); f == 1 || (f == 2 && pr.conv && nsplit == 1)) fn = f;   // (tests, experiments)
        const int64_t wave_tiles = ceil_div(pr.M, 32) * ceil_div(pr.N, 32 * fn);
        const unsigned g = static_cast<unsigned>(nsplit == 1 ? ceil_div(wave_tiles, 4) : tiles);
        const int gmax = static_cast<int>(ceil_div(nse / 4, nsplit));  // most groups of four steps a wave has
        if (plan) {
            if (pr.conv && nsplit == 4) {
                plan->ok = true; plan->mp = mp; plan->kA = kA; plan->kB = kB;
                plan->vw = mp.Cw % 4 == 0 ? 4 : 2; plan->gmax = gmax; plan->grid = g;
            }
            rc = APNN_OK;
            return true;
        }
        const int vw = mp.Cw % 4 == 0 ? 4 : 2;
        ok = !pr.conv ? launch_mfma_small_matrix(mp, kA, kB, nsplit, g, as_stream(stream))
             : fn > 1 ? launch_mfma_small_conv_wide(mp, kA, kB, vw, fn, g, as_stream(stream))
                      : launch_mfma_small_conv(mp, kA, kB, vw, nsplit, gmax, g, as_stream(stream));
        if (!ok) return false;
        rc = check_launch(pr.who);
        return true;
    }
    if (plan) { rc = APNN_OK; return true; }
    if ((t == 256 || t == 128) && !pr.conv)
        mp.xcd_regions = (ceil_div(pr.M, t) % 2 == 0 && ceil_div(pr.N, t) % 4 == 0) ? 1 : 0;
    switch (t) {
        case 256: ok = launch_mfma256(mp, kA, kB, pr.conv, grid, as_stream(stream)); break;
        case 128: ok = launch_mfma128(mp, kA, kB, pr.conv, grid, as_stream(stream)); break;
        case 64: ok = short_k ? launch_mfma64_k8(mp, kA, kB, grid, as_stream(stream))
                              : launch_mfma64(mp, kA, kB, pr.conv, grid, as_stream(stream)); break;
        default: ok = launch_mfma32(mp, kA, kB, pr.conv, grid, as_stream(stream)); break;
    }
    if (!ok) return false;
    rc = check_launch(pr.who);
    return true;
}

static int run_tile(const Problem &pr, TileParams &p, int vw, void *stream)
{
    bool use_xor = false;
    p.alpha = 1; p.uA = 0; p.uB = 0; p.c0 = 0;
    const bool a_pm = pr.encA == APNN_ENC_PM1, b_pm = pr.encB == APNN_ENC_PM1;
    // -1/+1 features whose zero bits would be read as -1 where they must contribute 0 (taps outside the frame):
    // the kernel gives the feature operand a validity plane that counts negatively (Sec. 4.2 (b), tile_kernel.h).
    const bool pmz = pr.conv && a_pm && (b_pm || p.pad > 0);
    int r = pick_tile(pr.M, pr.N);
    if (pr.conv && vw == 2 && r == 8) r = 4;     // instantiated register tiles per loader width
    if (pr.conv && vw == 1) r = 2;
    if (pmz) {
        // words of K a pass walks (whole LDS read groups), each of which the validity passes count as 32 too many
        const int64_t nk = ceil_div(p.Kw, kTileKC);
        const int64_t walked = (nk - 1) * kTileKC + round_up(p.Kw - (nk - 1) * kTileKC, kTileLV);
        const int64_t weights = (int64_t(1) << pr.PB) - 1;              // sum of the plane weights of the column operand
        if (3 * 32 * walked * weights >= (int64_t(1) << 31))
            return fail(APNN_ERR_OVERFLOW, "%s: K too long for the validity-plane form of -1/+1 features", pr.who);
        p.PA = 2;
        if (b_pm) {                     // sum (2 a - V)(2 b - 1) = 2 [2 popc(a b) - popc(V b)] + popc(V) - 2 popc(a)
            p.alpha = 2; p.uA = 1; p.c0 = static_cast<int>(-64 * walked);
        } else {                        // sum (2 a - V) B_t = 2 popc(a B_t) - popc(V B_t), planes weighted by 2^t
            p.alpha = 1; p.c0 = static_cast<int>(-32 * walked * weights);
        }
    } else if (a_pm && b_pm) {          // Case II:  K - 2 popc(XOR)
        use_xor = true; p.alpha = -2; p.c0 = static_cast<int>(pr.Ktotal);
    } else if (a_pm) {                  // Case III: 2 What X - J X, J X = row sum of the 0/1 operand
        p.alpha = 2; p.uB = -1;
    } else if (b_pm) {
        p.alpha = 2; p.uA = -1;
    }
    if (p.pool == APNN_POOL_SUM2) {     // the sum of a grid must fit the int32 result as well
        const int64_t ma = a_pm ? 1 : (int64_t(1) << pr.PA) - 1, mb = b_pm ? 1 : (int64_t(1) << pr.PB) - 1;
        if (4 * pr.Ktotal * ma * mb >= (int64_t(1) << 31))
            return fail(APNN_ERR_OVERFLOW, "%s: the pooled sum of four results may exceed int32", pr.who);
    }
    const int64_t tiles = ceil_div(pr.M, 16 * r) * ceil_div(pr.N, 16 * r);
    if (tiles > 0x7FFFFFFF) return fail(APNN_ERR_INVALID_ARG, "%s: problem too large for one launch", pr.who);
    // XCD-aware tile order: among the factorizations of 8 that divide the tile
    // grid, take the one with the smallest per-XCD operand footprint.
    p.xm = p.xn = 0;
    {
        const int64_t tM = ceil_div(pr.M, 16 * r), tN = ceil_div(pr.N, 16 * r);
        double best = 0.0;
        for (int xm = 1; xm <= 8; xm *= 2) {
            const int xn = 8 / xm;
            if (tM % xm != 0 || tN % xn != 0) continue;
            const double foot = static_cast<double>(tM / xm) * pr.PA + static_cast<double>(tN / xn) * pr.PB;
            if (p.xm == 0 || foot < best) { best = foot; p.xm = xm; p.xn = xn; }
        }
    }
    p.nk = static_cast<int>(ceil_div(p.Kw, kTileKC));
    const unsigned grid = static_cast<unsigned>(tiles);
    bool ok = false;
    switch (r) {
        case 8: ok = launch_tile8(p, pr.conv, vw, use_xor, pmz, grid, as_stream(stream)); break;
        case 4: ok = launch_tile4(p, pr.conv, vw, use_xor, pmz, grid, as_stream(stream)); break;
        default: ok = launch_tile2(p, pr.conv, vw, use_xor, pmz, grid, as_stream(stream)); break;
    }
    if (!ok) return fail(APNN_ERR_UNSUPPORTED, "%s: no kernel instance for this configuration", pr.who);
    return check_launch(pr.who);
}

// Matrix-core kernel when it applies, AND+popcount kernel otherwise; both read the
// same operands and write the same outputs.
static int run_either(const Problem &pr, TileParams &p, int vw, void *stream, SmallPlan *plan)
{
    MfmaParams mp{};
    mp.A = p.A; mp.B = p.B; mp.M = p.M; mp.N = p.N;
    mp.ldwA = p.ldwA; mp.ldwB = p.ldwB; mp.Kw = p.Kw;
    mp.H = p.H; mp.W = p.W; mp.Cw = p.Cw; mp.R = p.R; mp.S = p.S; mp.stride = p.stride; mp.pad = p.pad;
    mp.pool = p.pool; mp.Hp = p.Hp; mp.Wp = p.Wp;
    if (pr.conv) {
        mp.invS = 1.0f / static_cast<float>(p.S);
        mp.invWo = 1.0f / static_cast<float>(p.Wo);
        mp.invHoWo = 1.0f / (static_cast<float>(p.Ho) * static_cast<float>(p.Wo));
        mp.invWp = 1.0f / static_cast<float>(p.Wp > 0 ? p.Wp : 1);
        mp.invHpWp = 1.0f / (static_cast<float>(p.Hp > 0 ? p.Hp : 1) * static_cast<float>(p.Wp > 0 ? p.Wp : 1));
        mp.fastdiv = (pr.M + 256 < (int64_t(1) << 21)) ? 1 : 0;      // row indices, tile overhang included, stay below 2^21
    }
    mp.Ho = p.Ho; mp.Wo = p.Wo; mp.invCw = p.invCw;
    mp.Y = p.Y; mp.T = p.T; mp.scale = p.scale; mp.bias = p.bias;
    mp.res = p.res; mp.q_res = p.q_res; mp.res_scale = p.res_scale;
    mp.out = p.out; mp.q_out = p.q_out; mp.NW = p.NW;
    int rc = APNN_OK;
    if (try_mfma(pr, mp, stream, rc, plan)) return rc;
    if (plan) return APNN_OK;
    return run_tile(pr, p, vw, stream);
}

static int check_desc(const char *who, const apnn_conv_desc &d, bool is_gemm)
{
    if (int rc = check_bits_enc(who, "weight", d.p, d.encW)) return rc;
    if (int rc = check_bits_enc(who, "activation", d.q, d.encX)) return rc;
    if (d.N < 0 || d.Cin < 0 || d.Cout < 0) return fail(APNN_ERR_INVALID_ARG, "%s: negative size", who);
    if (is_gemm) {
        if (d.H != 1 || d.W != 1 || d.R != 1 || d.S != 1 || d.stride != 1 || d.pad != 0)
            return fail(APNN_ERR_INVALID_ARG, "%s: is_gemm needs H = W = R = S = stride = 1, pad = 0", who);
        return check_int32_range(who, d.Cin, d.p, d.q);
    }
    if (d.H < 1 || d.W < 1 || d.R < 1 || d.S < 1 || d.stride < 1 || d.pad < 0)
        return fail(APNN_ERR_INVALID_ARG, "%s: bad convolution geometry", who);
    if (d.H + 2 * d.pad < d.R || d.W + 2 * d.pad < d.S)
        return fail(APNN_ERR_INVALID_ARG, "%s: kernel larger than the padded frame", who);
    if (d.Cin % 32 != 0 || d.Cin == 0)
        return fail(APNN_ERR_INVALID_ARG, "%s: Cin = %lld must be a positive multiple of 32 for packed features", who, (long long)d.Cin);
    return check_int32_range(who, d.Cin * d.R * d.S, d.p, d.q);
}

// With a plan: validation and dispatch only, nothing is launched (see SmallPlan).
static int layer_impl(const char *who, const apnn_layer_desc &L, const uint32_t *W_dev, const uint32_t *X_dev,
                      uint32_t *out_packed, void *stream, SmallPlan *plan = nullptr)
{
    const apnn_conv_desc &d = L.conv;
    const bool is_gemm = L.is_gemm != 0;
    if (int rc = check_desc(who, d, is_gemm)) return rc;
    if (L.q_out < 0 || L.q_out > 8) return fail(APNN_ERR_UNSUPPORTED, "%s: q_out = %d, supported 0..8", who, L.q_out);
    const bool want_float = L.q_out > 0 || L.float_out_dev != nullptr;
    if (want_float && (!L.scale_dev || !L.bias_dev)) return fail(APNN_ERR_INVALID_ARG, "%s: scale_dev/bias_dev required", who);
    if (L.q_out > 0 && !out_packed) return fail(APNN_ERR_INVALID_ARG, "%s: out_packed_dev is null but q_out > 0", who);
    if (L.q_out > 0 && d.Cout % 32 != 0)
        return fail(APNN_ERR_INVALID_ARG, "%s: Cout = %lld must be a multiple of 32 for packed output", who, (long long)d.Cout);
    if (L.q_out == 0 && !L.acc_out_dev && !L.float_out_dev) return fail(APNN_ERR_INVALID_ARG, "%s: no output requested", who);
    if (L.residual_dev) {
        if (!want_float) return fail(APNN_ERR_INVALID_ARG, "%s: residual needs the scale/bias epilogue", who);
        if (L.q_res < 1 || L.q_res > 8) return fail(APNN_ERR_UNSUPPORTED, "%s: q_res = %d, supported 1..8", who, L.q_res);
        if (d.Cout % 32 != 0) return fail(APNN_ERR_INVALID_ARG, "%s: residual needs Cout multiple of 32", who);
        if (!aligned16(L.residual_dev)) return fail(APNN_ERR_ALIGNMENT, "%s: residual_dev not 16-byte aligned", who);
    }
    int Ho = 1, Wo = 1;
    if (!is_gemm) {
        Ho = static_cast<int>((d.H + 2 * d.pad - d.R) / d.stride + 1);
        Wo = static_cast<int>((d.W + 2 * d.pad - d.S) / d.stride + 1);
    }
    if (L.pool != APNN_POOL_NONE && L.pool != APNN_POOL_MAX2 && L.pool != APNN_POOL_SUM2)
        return fail(APNN_ERR_INVALID_ARG, "%s: pool = %d is not an apnn_pool value", who, L.pool);
    if (L.pool && is_gemm) return fail(APNN_ERR_INVALID_ARG, "%s: pooling applies to convolutions only", who);
    // with pooling the kernel enumerates 4 rows per pooled pixel (the grid), incomplete grids are dropped
    const int64_t M = L.pool ? d.N * (Ho / 2) * (Wo / 2) * 4 : d.N * Ho * Wo, N = d.Cout;
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || d.N * d.H * d.W > 0x7FFFFFFF)
        return fail(APNN_ERR_INVALID_ARG, "%s: dimension exceeds 2^31", who);
    if (M == 0 || N == 0) return APNN_OK;
    if (d.Cin > 0 && (!W_dev || !X_dev)) return fail(APNN_ERR_INVALID_ARG, "%s: null operand", who);
    if (!aligned16(W_dev) || !aligned16(X_dev)) return fail(APNN_ERR_ALIGNMENT, "%s: packed operands must be 16-byte aligned", who);
    if ((out_packed && !aligned16(out_packed)) || (L.acc_out_dev && !aligned16(L.acc_out_dev)))
        return fail(APNN_ERR_ALIGNMENT, "%s: outputs must be 16-byte aligned", who);

    TileParams p{};
    p.A = X_dev; p.B = W_dev;                 // activations supply the rows, weights the columns
    p.M = static_cast<int>(M); p.N = static_cast<int>(N);
    p.PA = d.q; p.PB = d.p;
    int vw = 4;
    if (is_gemm) {
        p.Kw = static_cast<int>(apnn_row_words(d.Cin));
        p.ldwA = p.ldwB = p.Kw;
    } else {
        const int64_t Cw = d.Cin / 32, Kw = Cw * d.R * d.S;
        if (Kw > 0x7FFFFFFF) return fail(APNN_ERR_INVALID_ARG, "%s: K too large", who);
        p.Cw = static_cast<int>(Cw); p.Kw = static_cast<int>(Kw);
        p.ldwA = 0; p.ldwB = p.Kw;
        p.H = static_cast<int>(d.H); p.W = static_cast<int>(d.W); p.R = d.R; p.S = d.S;
        p.stride = d.stride; p.pad = d.pad; p.Ho = Ho; p.Wo = Wo;
        p.pool = L.pool; p.Hp = Ho / 2; p.Wp = Wo / 2;
        p.invCw = 1.0f / static_cast<float>(Cw);
        vw = (Cw % 4 == 0) ? 4 : (Cw % 2 == 0) ? 2 : 1;
    }
    p.Y = L.acc_out_dev;
    if (want_float) {
        p.scale = L.scale_dev; p.bias = L.bias_dev; p.T = L.float_out_dev;
        p.res = L.residual_dev; p.q_res = L.q_res; p.res_scale = L.res_scale;
        p.out = L.q_out > 0 ? out_packed : nullptr; p.q_out = L.q_out;
    }
    p.NW = static_cast<int>(N / 32);
    Problem pr{who, !is_gemm, M, N, is_gemm ? d.Cin : d.Cin * d.R * d.S, p.PA, p.PB, d.encX, d.encW};
    return run_either(pr, p, vw, stream, plan);
}

}  // namespace apnn

using namespace apnn;

extern "C" int apnn_gemm(const uint32_t *W_dev, const uint32_t *X_dev, int32_t *Y_dev, int64_t M, int64_t N,
                         int64_t K, int p, int q, apnn_encoding encW, apnn_encoding encX, void *stream)
{
    clear_error();
    if (int rc = check_bits_enc("apnn_gemm", "weight", p, encW)) return rc;
    if (int rc = check_bits_enc("apnn_gemm", "activation", q, encX)) return rc;
    if (M < 0 || N < 0 || K < 0) return fail(APNN_ERR_INVALID_ARG, "apnn_gemm: negative size");
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || apnn_row_words(K) > 0x7FFFFFFF)
        return fail(APNN_ERR_INVALID_ARG, "apnn_gemm: dimension exceeds 2^31");
    if (int rc = check_int32_range("apnn_gemm", K, p, q)) return rc;
    if (M == 0 || N == 0) return APNN_OK;
    if (!Y_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_gemm: Y_dev is null");
    if (K > 0 && (!W_dev || !X_dev)) return fail(APNN_ERR_INVALID_ARG, "apnn_gemm: null operand");
    if (!aligned16(W_dev) || !aligned16(X_dev) || !aligned16(Y_dev))
        return fail(APNN_ERR_ALIGNMENT, "apnn_gemm: buffers must be 16-byte aligned");
    TileParams t{};
    t.A = W_dev; t.B = X_dev;                 // weights supply the rows of Y (W is M x K, Sec. 4.1)
    t.M = static_cast<int>(M); t.N = static_cast<int>(N);
    t.PA = p; t.PB = q;
    t.Kw = static_cast<int>(apnn_row_words(K));
    t.ldwA = t.ldwB = t.Kw;
    t.Y = Y_dev;
#ifdef APNN_BIG_TIMING                              // instrumented build: where mfma_big_kernel leaves its time stamps (mfma_big.h)
    if (const char *e = std::getenv("APNN_DBG_PTR")) t.T = reinterpret_cast<float *>(std::strtoull(e, nullptr, 0));
#endif
    t.NW = static_cast<int>(N / 32);
    Problem pr{"apnn_gemm", false, M, N, K, p, q, encW, encX};
    return run_either(pr, t, 4, stream, nullptr);
}

extern "C" int apnn_conv2d(const apnn_conv_desc *desc, const uint32_t *W_dev, const uint32_t *X_dev, int32_t *Y_dev,
                           void *stream)
{
    clear_error();
    if (!desc) return fail(APNN_ERR_INVALID_ARG, "apnn_conv2d: desc is null");
    if (!Y_dev) return fail(APNN_ERR_INVALID_ARG, "apnn_conv2d: Y_dev is null");
    apnn_layer_desc L{};
    L.conv = *desc;
    L.acc_out_dev = Y_dev;
    return layer_impl("apnn_conv2d", L, W_dev, X_dev, nullptr, stream);
}

extern "C" int apnn_layer(const apnn_layer_desc *desc, const uint32_t *W_dev, const uint32_t *X_dev,
                          uint32_t *out_packed_dev, void *stream)
{
    clear_error();
    if (!desc) return fail(APNN_ERR_INVALID_ARG, "apnn_layer: desc is null");
    return layer_impl("apnn_layer", *desc, W_dev, X_dev, out_packed_dev, stream);
}

extern "C" int apnn_layer_pair(const apnn_layer_desc *descA, const uint32_t *WA_dev, const uint32_t *XA_dev,
                               uint32_t *outA_packed_dev, const apnn_layer_desc *descB, const uint32_t *WB_dev,
                               const uint32_t *XB_dev, uint32_t *outB_packed_dev, void *stream)
{
    clear_error();
    const char *who = "apnn_layer_pair";
    if (!descA || !descB) return fail(APNN_ERR_INVALID_ARG, "%s: desc is null", who);
    SmallPlan a{}, b{};
    if (int rc = layer_impl(who, *descA, WA_dev, XA_dev, outA_packed_dev, stream, &a)) return rc;
    if (int rc = layer_impl(who, *descB, WB_dev, XB_dev, outB_packed_dev, stream, &b)) return rc;
    // (sharing pays while the layers are bound by launch and drain: up to a few blocks per compute unit)
    if (a.ok && b.ok && a.kA == b.kA && a.kB == b.kB && a.vw == b.vw &&
        static_cast<uint64_t>(a.grid) + b.grid <= 2048u) {
        const int gmax = (a.gmax <= 1 && b.gmax <= 1) ? 1 : 5;
        if (launch_mfma_small_conv_pair(a.mp, a.grid, b.mp, b.grid, a.kA, a.kB, a.vw, gmax, as_stream(stream)))
            return check_launch(who);
    }
    if (int rc = layer_impl(who, *descA, WA_dev, XA_dev, outA_packed_dev, stream)) return rc;
    return layer_impl(who, *descB, WB_dev, XB_dev, outB_packed_dev, stream);
}

extern "C" int apnn_debug_force(const char *name, int value)
{
    clear_error();
    if (!name) return fail(APNN_ERR_INVALID_ARG, "apnn_debug_force: name is null");
    (void)ov(OV_MFMA);                                   // the environment is read before the first explicit setting
    for (int i = 0; i < OV_COUNT; ++i)
        if (std::strcmp(name, kOverrideNames[i]) == 0) {
            g_override[i].store(value < 0 ? -1 : value, std::memory_order_relaxed);
            return APNN_OK;
        }
    return fail(APNN_ERR_INVALID_ARG, "apnn_debug_force: unknown override '%s'", name);
}

extern "C" int apnn_debug_tile_choice(int64_t M, int64_t N, int is_conv, int matrix_form)
{
    if (M <= 0 || N <= 0) return 0;
    return matrix_form ? pick_mfma_tile(M, N, is_conv != 0) : 16 * pick_tile(M, N);
}

extern "C" void apnn_debug_reset(void)
{
    (void)ov(OV_MFMA);
    overrides_from_env();
}

extern "C" size_t apnn_workspace_bytes(const apnn_layer_desc *desc)
{
    (void)desc;
    return 0;
}
