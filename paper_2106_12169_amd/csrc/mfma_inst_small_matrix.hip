// Matrix-operand instances of the small-layer matrix-core kernel (lane-private
// operand loads, 32 x 32 tiles): one tile per wave or K split over four waves.
#include "mfma_launch.h"
#include "mfma_small.h"

namespace apnn {

template <int KA, int KB> static void go(const MfmaParams &p, int nsplit, unsigned grid, hipStream_t st)
{
    if (nsplit == 1) hipLaunchKernelGGL((mfma_small_kernel<KA, KB, 4, false, 1>), dim3(grid), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((mfma_small_kernel<KA, KB, 4, false, 4>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma_small_matrix(const MfmaParams &p, int kindA, int kindB, int nsplit, unsigned grid, hipStream_t st)
{
    switch (kindA * 3 + kindB) {
        case 0: go<0, 0>(p, nsplit, grid, st); return true;
        case 1: go<0, 1>(p, nsplit, grid, st); return true;
        case 2: go<0, 2>(p, nsplit, grid, st); return true;
        case 3: go<1, 0>(p, nsplit, grid, st); return true;
        case 4: go<1, 1>(p, nsplit, grid, st); return true;
        case 5: go<1, 2>(p, nsplit, grid, st); return true;
        case 6: go<2, 0>(p, nsplit, grid, st); return true;
        case 7: go<2, 1>(p, nsplit, grid, st); return true;
        case 8: go<2, 2>(p, nsplit, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
