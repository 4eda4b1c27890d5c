// Pair instances of the small-layer matrix-core kernel: two independent
// convolution layers of the same operand kinds and loader width in one launch.
#include "mfma_launch.h"
#include "mfma_small.h"

namespace apnn {

template <int KA, int KB> static void go(const MfmaPairParams &pp, int vw, int gmax, unsigned grid, hipStream_t st)
{
    if (vw == 4 && gmax == 1) hipLaunchKernelGGL((mfma_small_pair_kernel<KA, KB, 4, 1>), dim3(grid), dim3(256), 0, st, pp);
    else if (vw == 4) hipLaunchKernelGGL((mfma_small_pair_kernel<KA, KB, 4, 5>), dim3(grid), dim3(256), 0, st, pp);
    else if (gmax == 1) hipLaunchKernelGGL((mfma_small_pair_kernel<KA, KB, 2, 1>), dim3(grid), dim3(256), 0, st, pp);
    else hipLaunchKernelGGL((mfma_small_pair_kernel<KA, KB, 2, 5>), dim3(grid), dim3(256), 0, st, pp);
}

bool launch_mfma_small_conv_pair(const MfmaParams &p0, unsigned grid0, const MfmaParams &p1, unsigned grid1, int kindA,
                                 int kindB, int vw, int gmax, hipStream_t st)
{
    MfmaPairParams pp;
    pp.p[0] = p0; pp.p[1] = p1;
    pp.blocks0 = static_cast<int>(grid0);
    const unsigned grid = grid0 + grid1;
    switch (kindA * 3 + kindB) {          // features: 0/1 planes, or -1/+1 with the loader's validity word
        case 9: go<3, 0>(pp, vw, gmax, grid, st); return true;
        case 10: go<3, 1>(pp, vw, gmax, grid, st); return true;
        case 11: go<3, 2>(pp, vw, gmax, grid, st); return true;
        case 0: go<0, 0>(pp, vw, gmax, grid, st); return true;
        case 1: go<0, 1>(pp, vw, gmax, grid, st); return true;
        case 2: go<0, 2>(pp, vw, gmax, grid, st); return true;
        case 3: go<1, 0>(pp, vw, gmax, grid, st); return true;
        case 4: go<1, 1>(pp, vw, gmax, grid, st); return true;
        case 5: go<1, 2>(pp, vw, gmax, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
