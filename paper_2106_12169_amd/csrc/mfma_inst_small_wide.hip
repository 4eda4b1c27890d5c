// Convolution instances of the small-layer matrix-core kernel for large layers: one wave tile per wave
// (no K split), 32 x 64 outputs per wave tile.
#include "mfma_launch.h"
#include "mfma_small_wide.h"

namespace apnn {

template <int KA, int KB> static void go(const MfmaParams &p, int vw, int fn, unsigned grid, hipStream_t st)
{
    (void)fn;                             // 2: the only width instantiated (4 measured slower)
    if (vw == 4) hipLaunchKernelGGL((mfma_small_wide_kernel<KA, KB, 4, 2>), dim3(grid), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((mfma_small_wide_kernel<KA, KB, 2, 2>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma_small_conv_wide(const MfmaParams &p, int kindA, int kindB, int vw, int fn, unsigned grid, hipStream_t st)
{
    if (fn != 2) return false;
    switch (kindA * 3 + kindB) {          // features: 0/1 planes, or -1/+1 with the loader's validity word
        case 9: go<3, 0>(p, vw, fn, grid, st); return true;
        case 10: go<3, 1>(p, vw, fn, grid, st); return true;
        case 11: go<3, 2>(p, vw, fn, grid, st); return true;
        case 0: go<0, 0>(p, vw, fn, grid, st); return true;
        case 1: go<0, 1>(p, vw, fn, grid, st); return true;
        case 2: go<0, 2>(p, vw, fn, grid, st); return true;
        case 3: go<1, 0>(p, vw, fn, grid, st); return true;
        case 4: go<1, 1>(p, vw, fn, grid, st); return true;
        case 5: go<1, 2>(p, vw, fn, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
