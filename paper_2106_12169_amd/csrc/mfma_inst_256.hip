// Dispatchers of the large-product matrix-core kernels: the FP4 form (256 x 256 block
// tile, 4 waves of 128 x 128) and the 8-bit integer form (128 x 128); the instances
// live in one translation unit per A-operand kind so that they compile in parallel.
#include "mfma_launch.h"

namespace apnn {

bool launch_mfma256_u1(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st);
bool launch_mfma256_u2(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st);
bool launch_mfma256_pm1(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st);

bool launch_mfma256(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st)
{
    if (conv) return false;              // instantiated for matrix operands only
    switch (kindA) {
        case OPK_U1: return launch_mfma256_u1(p, kindB, grid, st);
        case OPK_U2: return launch_mfma256_u2(p, kindB, grid, st);
        case OPK_PM1: return launch_mfma256_pm1(p, kindB, grid, st);
        default: return false;
    }
}

bool launch_mfma_i8_c2(const MfmaParams &p, int classB, int group, unsigned grid, hipStream_t st);
bool launch_mfma_i8_c4(const MfmaParams &p, int classB, int group, unsigned grid, hipStream_t st);
bool launch_mfma_i8_c8(const MfmaParams &p, int classB, int group, unsigned grid, hipStream_t st);

bool launch_mfma_i8(const MfmaParams &p, int classA, int classB, unsigned grid, hipStream_t st)
{
    // chunks fetched together: four (64 bytes of every plane row) while two group buffers fit the LDS, else two
    const int group = (p.PA + p.PB) <= 9 ? 4 : 2;
    switch (classA) {
        case 0: return launch_mfma_i8_c2(p, classB, group, grid, st);
        case 1: return launch_mfma_i8_c4(p, classB, group, grid, st);
        case 2: return launch_mfma_i8_c8(p, classB, group, grid, st);
        default: return false;
    }
}

bool launch_mfma_i8_wide_c2(const MfmaParams &p, int classB, unsigned grid, hipStream_t st);
bool launch_mfma_i8_wide_c4(const MfmaParams &p, int classB, unsigned grid, hipStream_t st);
bool launch_mfma_i8_wide_c8(const MfmaParams &p, int classB, unsigned grid, hipStream_t st);

bool launch_mfma_i8_wide(const MfmaParams &p, int classA, int classB, unsigned grid, hipStream_t st)
{
    if (p.PA + p.PB > 10) return false;                 // two group buffers of four chunks must fit the 160 KB of LDS
    switch (classA) {
        case 0: return launch_mfma_i8_wide_c2(p, classB, grid, st);
        case 1: return launch_mfma_i8_wide_c4(p, classB, grid, st);
        case 2: return launch_mfma_i8_wide_c8(p, classB, grid, st);
        default: return false;
    }
}

}  // namespace apnn
