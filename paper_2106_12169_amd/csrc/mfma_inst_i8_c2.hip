// Instances of the 8-bit integer matrix kernel (128 x 128 block tile) whose row operand has plane class C2.
#include "mfma_i8.h"
#include "mfma_launch.h"

namespace apnn {

template <int CB> static void go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_i8_kernel<0, CB, 2, 2>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma_i8_c2(const MfmaParams &p, int classB, unsigned grid, hipStream_t st)
{
    switch (classB) {
        case I8_C2: go<I8_C2>(p, grid, st); return true;
        case I8_C4: go<I8_C4>(p, grid, st); return true;
        case I8_C8: go<I8_C8>(p, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
