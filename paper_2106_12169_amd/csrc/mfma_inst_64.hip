// Instances of the FP4 matrix-core kernel with a 64 x 64 block tile.
#include "mfma_launch.h"

namespace apnn {

template <int KA, int KB, bool CONV> static void go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_fp4_kernel<KA, KB, 2, 2, 1, 1, 1, 32, (CONV ? 2 : 4), CONV>), dim3(grid), dim3(256), 0, st, p);
}

// Short-K matrix operands (K <= 256, e.g. the receptive-field-packed input layer):
// 8-word chunks, so that no matrix-instruction step multiplies padding.
template <int KA, int KB> static void go_k8(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_fp4_kernel<KA, KB, 2, 2, 1, 1, 1, 8, 4, false>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma64_k8(const MfmaParams &p, int kindA, int kindB, unsigned grid, hipStream_t st)
{
    switch (kindA * 3 + kindB) {
        case 0: go_k8<0, 0>(p, grid, st); return true;
        case 1: go_k8<0, 1>(p, grid, st); return true;
        case 2: go_k8<0, 2>(p, grid, st); return true;
        case 3: go_k8<1, 0>(p, grid, st); return true;
        case 4: go_k8<1, 1>(p, grid, st); return true;
        case 5: go_k8<1, 2>(p, grid, st); return true;
        case 6: go_k8<2, 0>(p, grid, st); return true;
        case 7: go_k8<2, 1>(p, grid, st); return true;
        case 8: go_k8<2, 2>(p, grid, st); return true;
        default: return false;
    }
}

bool launch_mfma64(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st)
{
    if (!conv) {
        switch (kindA * 3 + kindB) {
            case 0: go<0, 0, false>(p, grid, st); return true;
            case 1: go<0, 1, false>(p, grid, st); return true;
            case 2: go<0, 2, false>(p, grid, st); return true;
            case 3: go<1, 0, false>(p, grid, st); return true;
            case 4: go<1, 1, false>(p, grid, st); return true;
            case 5: go<1, 2, false>(p, grid, st); return true;
            case 6: go<2, 0, false>(p, grid, st); return true;
            case 7: go<2, 1, false>(p, grid, st); return true;
            case 8: go<2, 2, false>(p, grid, st); return true;
            default: return false;
        }
    }
    switch (kindA * 3 + kindB) {          // features: 0/1 planes, or -1/+1 with the loader's validity word
        case 9: go<3, 0, true>(p, grid, st); return true;
        case 10: go<3, 1, true>(p, grid, st); return true;
        case 11: go<3, 2, true>(p, grid, st); return true;
        case 0: go<0, 0, true>(p, grid, st); return true;
        case 1: go<0, 1, true>(p, grid, st); return true;
        case 2: go<0, 2, true>(p, grid, st); return true;
        case 3: go<1, 0, true>(p, grid, st); return true;
        case 4: go<1, 1, true>(p, grid, st); return true;
        case 5: go<1, 2, true>(p, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
