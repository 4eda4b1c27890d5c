// Matrix-operand instances of the LDS-resident small-layer matrix-core kernel (32 x 32 tile,
// whole K on chip): K of at most 32, 64, 96 or 160 words per plane.
#include "mfma_launch.h"
#include "mfma_small.h"

namespace apnn {

template <int KA, int KB, bool CONV> static void go(const MfmaParams &p, int kcmax, unsigned grid, hipStream_t st)
{
    switch (kcmax) {
        case 32: hipLaunchKernelGGL((mfma_small_kernel<KA, KB, 32, CONV>), dim3(grid), dim3(256), 0, st, p); break;
        case 64: hipLaunchKernelGGL((mfma_small_kernel<KA, KB, 64, CONV>), dim3(grid), dim3(256), 0, st, p); break;
        case 96: hipLaunchKernelGGL((mfma_small_kernel<KA, KB, 96, CONV>), dim3(grid), dim3(256), 0, st, p); break;
        default: hipLaunchKernelGGL((mfma_small_kernel<KA, KB, 160, CONV>), dim3(grid), dim3(256), 0, st, p); break;
    }
}

bool launch_mfma_small_matrix(const MfmaParams &p, int kindA, int kindB, int kcmax, unsigned grid, hipStream_t st)
{
    switch (kindA * 3 + kindB) {
        case 0: go<0, 0, false>(p, kcmax, grid, st); return true;
        case 1: go<0, 1, false>(p, kcmax, grid, st); return true;
        case 2: go<0, 2, false>(p, kcmax, grid, st); return true;
        case 3: go<1, 0, false>(p, kcmax, grid, st); return true;
        case 4: go<1, 1, false>(p, kcmax, grid, st); return true;
        case 5: go<1, 2, false>(p, kcmax, grid, st); return true;
        case 6: go<2, 0, false>(p, kcmax, grid, st); return true;
        case 7: go<2, 1, false>(p, kcmax, grid, st); return true;
        case 8: go<2, 2, false>(p, kcmax, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
