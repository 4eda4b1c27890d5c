// Instances of the large-product matrix-core kernel (256 x 256 block tile, 4 waves of 128 x 128).
#include "mfma_big.h"
#include "mfma_launch.h"

namespace apnn {

template <int KA, int KB, bool CONV> static void go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    static_assert(!CONV, "matrix operands only");
    hipLaunchKernelGGL((mfma_big_kernel<KA, KB, 2, 2, 4, 4>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma256(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st)
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
    return false;                        // large tiles are instantiated for matrix operands only
}

}  // namespace apnn
