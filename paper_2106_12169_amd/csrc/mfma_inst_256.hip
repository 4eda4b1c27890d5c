// Dispatcher of the large-product matrix-core kernel (256 x 256 block tile, 4 waves
// of 128 x 128); the instances live in one translation unit per A-operand kind so
// that they compile in parallel.
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

}  // namespace apnn
