// Convolution instances of the small-layer matrix-core kernel (lane-private
// operand loads, 32 x 32 tiles): loader vector width 4 or 2 words, one tile per
// wave or one tile per block with K split over its four waves.
#include "mfma_launch.h"
#include "mfma_small.h"

namespace apnn {

template <int KA, int KB, int VW> static void go_vw(const MfmaParams &p, int nsplit, int gmax, unsigned grid, hipStream_t st)
{
    if (nsplit == 1) hipLaunchKernelGGL((mfma_small_kernel<KA, KB, VW, true, 1>), dim3(grid), dim3(256), 0, st, p);
    else if (gmax == 1) hipLaunchKernelGGL((mfma_small_kernel<KA, KB, VW, true, 4, 1>), dim3(grid), dim3(256), 0, st, p);
    else if (gmax == 2) hipLaunchKernelGGL((mfma_small_kernel<KA, KB, VW, true, 4, 2>), dim3(grid), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((mfma_small_kernel<KA, KB, VW, true, 4>), dim3(grid), dim3(256), 0, st, p);
}

// gmax: most groups of four steps a wave of a K-split block has (1, 2, or more)
template <int KA, int KB> static void go(const MfmaParams &p, int vw, int nsplit, int gmax, unsigned grid, hipStream_t st)
{
    if (vw == 4) go_vw<KA, KB, 4>(p, nsplit, gmax, grid, st);
    else go_vw<KA, KB, 2>(p, nsplit, gmax, grid, st);
}

bool launch_mfma_small_conv(const MfmaParams &p, int kindA, int kindB, int vw, int nsplit, int gmax, unsigned grid,
                            hipStream_t st)
{
    switch (kindA * 3 + kindB) {          // features: 0/1 planes, or -1/+1 with the loader's validity word
        case 9: go<3, 0>(p, vw, nsplit, gmax, grid, st); return true;
        case 10: go<3, 1>(p, vw, nsplit, gmax, grid, st); return true;
        case 11: go<3, 2>(p, vw, nsplit, gmax, grid, st); return true;
        case 0: go<0, 0>(p, vw, nsplit, gmax, grid, st); return true;
        case 1: go<0, 1>(p, vw, nsplit, gmax, grid, st); return true;
        case 2: go<0, 2>(p, vw, nsplit, gmax, grid, st); return true;
        case 3: go<1, 0>(p, vw, nsplit, gmax, grid, st); return true;
        case 4: go<1, 1>(p, vw, nsplit, gmax, grid, st); return true;
        case 5: go<1, 2>(p, vw, nsplit, gmax, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
