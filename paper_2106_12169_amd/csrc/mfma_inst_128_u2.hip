// Instances of the pipelined matrix-core kernel with a 128 x 128 block tile (4 waves of 64 x 64) whose A
// operand kind is OPK_U2.
#include "mfma_big.h"
#include "mfma_launch.h"

namespace apnn {

template <int KB> static void go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_big_kernel<OPK_U2, KB, 2, 2, 2, 2>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma128_u2(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st)
{
    switch (kindB) {
        case OPK_U1: go<OPK_U1>(p, grid, st); return true;
        case OPK_U2: go<OPK_U2>(p, grid, st); return true;
        case OPK_PM1: go<OPK_PM1>(p, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
