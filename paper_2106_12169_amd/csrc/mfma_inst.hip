// Instances and launcher of the FP4 matrix-core kernel (operands of <= 2 bits).
#include "mfma_kernel.h"
#include "tile_launch.h"

namespace apnn {

template <int KA, int KB> static void go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_fp4_kernel<KA, KB>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma_fp4(const MfmaParams &p, int kindA, int kindB, unsigned grid, hipStream_t st)
{
    switch (kindA * 3 + kindB) {
        case 0: go<0, 0>(p, grid, st); return true;
        case 1: go<0, 1>(p, grid, st); return true;
        case 2: go<0, 2>(p, grid, st); return true;
        case 3: go<1, 0>(p, grid, st); return true;
        case 4: go<1, 1>(p, grid, st); return true;
        case 5: go<1, 2>(p, grid, st); return true;
        case 6: go<2, 0>(p, grid, st); return true;
        case 7: go<2, 1>(p, grid, st); return true;
        case 8: go<2, 2>(p, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
