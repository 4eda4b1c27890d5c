// Host side of the C-ABI library under -fsanitize=address,undefined: size helpers, the batch-norm fold, the
// override table, the tile choice, every argument check, and the dispatch itself.  The sources with the host logic
// (layer.hip, pack.hip, pool.hip, input_layer.hip, common.cpp) are linked with the stand-ins below in place of the
// kernel-instance launchers, which record what the dispatch asked for and launch nothing; so the whole decision path
// of apnn_gemm / apnn_layer runs without a GPU and its constants can be checked.  Device pointers are fakes that host
// code never dereferences.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/apnn.h"
#include "../../include/apnn_debug.h"
#include "../../paper_2106_12169_amd/csrc/mfma_launch.h"
#include "../../paper_2106_12169_amd/csrc/tile_launch.h"

// ---- stand-ins for the kernel-instance launchers -------------------------------------------------------------
static std::string g_kernel;          // which launcher the last dispatch chose
static apnn::MfmaParams g_mp;
static apnn::TileParams g_tp;
static unsigned g_grid;
static int g_pmz;

namespace apnn {
static bool took(const char *name, const MfmaParams &p, unsigned grid) { g_kernel = name; g_mp = p; g_grid = grid; return true; }
bool launch_mfma256(const MfmaParams &p, int, int, bool, unsigned grid, hipStream_t) { return took("mfma256", p, grid); }
bool launch_mfma128(const MfmaParams &p, int, int, bool, unsigned grid, hipStream_t) { return took("mfma128", p, grid); }
bool launch_mfma64(const MfmaParams &p, int, int, bool, unsigned grid, hipStream_t) { return took("mfma64", p, grid); }
bool launch_mfma64_k8(const MfmaParams &p, int, int, unsigned grid, hipStream_t) { return took("mfma64_k8", p, grid); }
bool launch_mfma32(const MfmaParams &p, int, int, bool, unsigned grid, hipStream_t) { return took("mfma32", p, grid); }
bool launch_mfma_small_conv(const MfmaParams &p, int, int, int, int, int, unsigned grid, hipStream_t) { return took("small_conv", p, grid); }
bool launch_mfma_small_conv_wide(const MfmaParams &p, int, int, int, int, unsigned grid, hipStream_t) { return took("small_conv_wide", p, grid); }
bool launch_mfma_small_conv_pair(const MfmaParams &p0, unsigned grid0, const MfmaParams &, unsigned grid1, int, int, int, int, hipStream_t)
{
    return took("small_conv_pair", p0, grid0 + grid1);
}
bool launch_mfma_small_matrix(const MfmaParams &p, int, int, int, unsigned grid, hipStream_t) { return took("small_matrix", p, grid); }
bool launch_mfma_i8(const MfmaParams &p, int, int, unsigned grid, hipStream_t) { return took("i8", p, grid); }
bool launch_mfma_i8_wide(const MfmaParams &p, int, int, unsigned grid, hipStream_t) { return took("i8_wide", p, grid); }
static bool took_tile(const char *name, const TileParams &p, bool pmz, unsigned grid) { g_kernel = name; g_tp = p; g_pmz = pmz; g_grid = grid; return true; }
bool launch_tile8(const TileParams &p, bool conv, int vw, bool, bool pmz, unsigned grid, hipStream_t) { return conv && vw != 4 ? false : took_tile("tile8", p, pmz, grid); }
bool launch_tile4(const TileParams &p, bool conv, int vw, bool, bool pmz, unsigned grid, hipStream_t) { return conv && vw == 1 ? false : took_tile("tile4", p, pmz, grid); }
bool launch_tile2(const TileParams &p, bool, int, bool, bool pmz, unsigned grid, hipStream_t) { return took_tile("tile2", p, pmz, grid); }
}  // namespace apnn

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("line %d: %s (last error: %s)\n", __LINE__, #cond, apnn_last_error()); ++failures; } } while (0)

int main()
{
    void *fake = reinterpret_cast<void *>(uintptr_t(1) << 20);        // 16-byte aligned, never dereferenced
    const uint32_t *fw = static_cast<const uint32_t *>(fake);
    EXPECT(apnn_row_words(129) == 8 && apnn_packed_words(4096, 4096, 2) == size_t(4096) * 2 * 128);
    EXPECT(apnn_fmap_words(6272, 128, 2) == size_t(6272) * 2 * 4);
    EXPECT(apnn_input_weight_bytes(64, 3, 7, 7) > 0 && apnn_input_weight_bytes(64, 3, 11, 11) > apnn_input_weight_bytes(64, 3, 7, 7));
    EXPECT(apnn_workspace_bytes(nullptr) == 0);

    for (int C : {1, 7, 64, 1000}) {
        std::vector<double> g(C, 1.5), b(C, 0.25), m(C, 0.1), v(C, 2.0);
        std::vector<float> sc(C), bi(C);
        EXPECT(apnn_fold_bn(g.data(), b.data(), m.data(), v.data(), 1e-5, 0.5, 0.25, C, sc.data(), bi.data()) == APNN_OK);
        EXPECT(sc[C - 1] > 0.0f);
    }
    EXPECT(apnn_fold_bn(nullptr, nullptr, nullptr, nullptr, 1e-5, 0.0, 1.0, 4, nullptr, nullptr) == APNN_ERR_INVALID_ARG);

    EXPECT(apnn_debug_force("MFMA", 0) == APNN_OK && apnn_debug_force("INT8", 1) == APNN_OK);
    EXPECT(apnn_debug_force("NOT_A_SWITCH", 1) == APNN_ERR_INVALID_ARG && std::strlen(apnn_last_error()) > 0);
    EXPECT(apnn_debug_force(nullptr, 1) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_debug_force("A_NAME_THAT_IS_MUCH_LONGER_THAN_ANY_SWITCH_OF_THE_LIBRARY_AND_THEN_SOME", 1) == APNN_ERR_INVALID_ARG);
    apnn_debug_reset();
    EXPECT(apnn_debug_tile_choice(4096, 4096, 0, 1) == 256 && apnn_debug_tile_choice(64, 64, 0, 0) == 32);
    EXPECT(apnn_debug_tile_choice(0, 0, 0, 1) == 0);

    // argument checks of the compute entry points (each returns before any launch)
    EXPECT(apnn_gemm(fw, fw, nullptr, 4, 4, 64, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_gemm(fw, fw, static_cast<int32_t *>(fake), 4, 4, 64, 9, 2, APNN_ENC_UNSIGNED, APNN_ENC_UNSIGNED, nullptr) == APNN_ERR_UNSUPPORTED);
    EXPECT(apnn_gemm(fw, fw, static_cast<int32_t *>(fake), 4, 4, 64, 2, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr) == APNN_ERR_UNSUPPORTED);
    EXPECT(apnn_gemm(fw, fw, static_cast<int32_t *>(fake), -1, 4, 64, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_gemm(fw, fw, static_cast<int32_t *>(fake), 4, 4, int64_t(1) << 40, 8, 8, APNN_ENC_UNSIGNED, APNN_ENC_UNSIGNED, nullptr) != APNN_OK);
    EXPECT(apnn_gemm(reinterpret_cast<const uint32_t *>(uintptr_t(fake) + 4), fw, static_cast<int32_t *>(fake), 4, 4, 64, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr) == APNN_ERR_ALIGNMENT);
    EXPECT(apnn_gemm(fw, fw, static_cast<int32_t *>(fake), 0, 4, 64, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr) == APNN_OK);   // empty

    apnn_layer_desc L{};
    L.conv = apnn_conv_desc{8, 28, 28, 128, 128, 3, 3, 1, 1, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED};
    L.q_out = 2;
    EXPECT(apnn_layer(&L, fw, fw, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);      // no scale / bias
    L.scale_dev = L.bias_dev = static_cast<const float *>(fake);
    L.pool = 3;
    EXPECT(apnn_layer(&L, fw, fw, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);
    L.pool = 0; L.q_out = 9;
    EXPECT(apnn_layer(&L, fw, fw, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_UNSUPPORTED);
    L.q_out = 2; L.conv.Cin = 100;
    EXPECT(apnn_layer(&L, fw, fw, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);
    L.conv.Cin = 128; L.conv.N = 0;
    EXPECT(apnn_layer(&L, fw, fw, static_cast<uint32_t *>(fake), nullptr) == APNN_OK);                   // empty batch
    EXPECT(apnn_layer(nullptr, fw, fw, nullptr, nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_layer_pair(nullptr, fw, fw, nullptr, nullptr, fw, fw, nullptr, nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_conv2d(nullptr, fw, fw, static_cast<int32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_input_layer(nullptr, fake, static_cast<const uint8_t *>(fake), static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);

    EXPECT(apnn_pack(fake, 4, 64, 9, APNN_ENC_UNSIGNED, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_UNSUPPORTED);
    EXPECT(apnn_pack(fake, 0, 64, 2, APNN_ENC_UNSIGNED, static_cast<uint32_t *>(fake), nullptr) == APNN_OK);
    EXPECT(apnn_quantize(static_cast<const float *>(fake), 4, 64, 0.0f, 0.0f, 2, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_sumpool(fw, 1, 7, 7, 64, 2, 7, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_OVERFLOW);
    EXPECT(apnn_maxpool(fw, 1, 8, 8, 64, 2, 3, 2, 3, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_INVALID_ARG);
    EXPECT(apnn_pack_patches(static_cast<const uint8_t *>(fake), 1, 3, 8, 8, 7, 12, 2, 3, 8, static_cast<uint32_t *>(fake), nullptr) == APNN_ERR_UNSUPPORTED);

    // ---- the dispatch (a launcher stand-in answers; the status is that of the runtime's last-error query, which
    // without a GPU may be a launch error: only the choice and its constants are looked at)
    int32_t *fy = static_cast<int32_t *>(fake);
    apnn_debug_reset();
    g_kernel.clear();
    (void)apnn_gemm(fw, fw, fy, 4096, 4096, 4096, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr);       // the headline product
    EXPECT(g_kernel == "mfma256" && g_grid == 256 && g_mp.out_scale == 2.0f && g_mp.c0 == 0 && g_mp.xcd_regions == 1);
    (void)apnn_gemm(fw, fw, fy, 2048, 2048, 2048, 3, 5, APNN_ENC_UNSIGNED, APNN_ENC_UNSIGNED, nullptr);  // 6 FP4 passes: one int8 pass
    EXPECT(g_kernel == "i8" && g_grid == 256 && g_mp.accmul == 1 && g_mp.mulA == 0 && g_mp.mulB == 0 && g_mp.c0 == 0);
    (void)apnn_gemm(fw, fw, fy, 2048, 2048, 4096, 3, 5, APNN_ENC_UNSIGNED, APNN_ENC_UNSIGNED, nullptr);  // long K: shared out among the waves
    EXPECT(g_kernel == "i8_wide" && g_grid == 256 && g_mp.nk % 4 == 0);
    (void)apnn_gemm(fw, fw, fy, 2048, 2048, 4096, 5, 6, APNN_ENC_UNSIGNED, APNN_ENC_UNSIGNED, nullptr);  // 11 planes: more than its LDS holds
    EXPECT(g_kernel == "i8");
    (void)apnn_gemm(fw, fw, fy, 20, 20, 4000, 8, 8, APNN_ENC_UNSIGNED, APNN_ENC_UNSIGNED, nullptr);      // beyond the exact range of FP4
    // bytes are value - 128 on both sides: Y = acc + 128 RA + 128 RB + c0, c0 = -npad 128^2 - 2 * 128 * 128 K + 128^2 K
    EXPECT(g_kernel == "i8" && g_mp.mulA == 128 && g_mp.mulB == 128 && g_mp.flipA == ~0u);
    EXPECT(g_mp.c0 == static_cast<int>(-(int64_t(g_mp.nk) * 128 - 4000) * 16384 - 16384 * int64_t(4000)));
    (void)apnn_gemm(fw, fw, fy, 64, 1024, 1024, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr);         // a paper-sized fully connected layer
    EXPECT(g_kernel == "small_matrix");
    (void)apnn_gemm(fw, fw, fy, 512, 512, 100, 1, 1, APNN_ENC_PM1, APNN_ENC_PM1, nullptr);               // Case II: pad positions multiply to +1
    EXPECT(g_mp.c0 < 0);
    EXPECT(apnn_debug_force("MFMA", 0) == APNN_OK);
    (void)apnn_gemm(fw, fw, fy, 4096, 4096, 4096, 1, 2, APNN_ENC_PM1, APNN_ENC_UNSIGNED, nullptr);
    EXPECT(g_kernel == "tile4" && g_grid == 4096 && g_tp.alpha == 2 && g_tp.uB == -1 && g_tp.uA == 0 && g_tp.c0 == 0
           && g_tp.xm * g_tp.xn == 8);
    (void)apnn_gemm(fw, fw, fy, 100, 100, 777, 1, 1, APNN_ENC_PM1, APNN_ENC_PM1, nullptr);               // Case II: K - 2 popc(xor)
    EXPECT(g_kernel == "tile2" && g_tp.alpha == -2 && g_tp.c0 == 777);
    // -1/+1 features with padding on the popcount kernel: validity plane, c0 = -32 (walked words) (plane weights)
    apnn_layer_desc P{};
    P.conv = apnn_conv_desc{2, 9, 9, 96, 64, 3, 3, 1, 1, 3, 1, APNN_ENC_UNSIGNED, APNN_ENC_PM1};
    P.acc_out_dev = fy;
    (void)apnn_layer(&P, fw, fw, nullptr, nullptr);
    EXPECT(g_pmz == 1 && g_tp.PA == 2 && g_tp.alpha == 1 && g_tp.Kw == 27 && g_tp.c0 == -32 * 28 * 7);
    P.conv.p = 1; P.conv.encW = APNN_ENC_PM1;
    (void)apnn_layer(&P, fw, fw, nullptr, nullptr);
    EXPECT(g_pmz == 1 && g_tp.alpha == 2 && g_tp.uA == 1 && g_tp.c0 == -64 * 28);
    P.pool = APNN_POOL_SUM2;
    (void)apnn_layer(&P, fw, fw, nullptr, nullptr);
    EXPECT(g_tp.pool == 2 && g_tp.M == 2 * 4 * 4 * 4 && g_tp.Hp == 4);
    apnn_debug_reset();
    P.conv.Cin = 128;                                                                                       // matrix-core shape again
    (void)apnn_layer(&P, fw, fw, nullptr, nullptr);
    EXPECT(g_kernel == "small_conv" && g_mp.pool == 2);

    if (failures == 0) std::puts("abi host sanitizer run ok");
    return failures != 0;
}
