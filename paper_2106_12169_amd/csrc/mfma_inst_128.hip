// 128 x 128 block tile: convolution instances of the general FP4 matrix-core kernel, and the dispatcher to the
// matrix-operand instances of the pipelined kernel (one translation unit per A-operand kind).
#include "mfma_launch.h"

namespace apnn {

template <int KA, int KB, bool CONV> static void go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((mfma_fp4_kernel<KA, KB, 2, 2, 1, 2, 2, 16, (CONV ? 2 : 4), CONV>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_mfma128_u1(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st);
bool launch_mfma128_u2(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st);
bool launch_mfma128_pm1(const MfmaParams &p, int kindB, unsigned grid, hipStream_t st);

bool launch_mfma128(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st)
{
    if (!conv) {                          // matrix operands: the pipelined kernel with 64 x 64 wave tiles
        switch (kindA) {
            case OPK_U1: return launch_mfma128_u1(p, kindB, grid, st);
            case OPK_U2: return launch_mfma128_u2(p, kindB, grid, st);
            case OPK_PM1: return launch_mfma128_pm1(p, kindB, grid, st);
            default: return false;
        }
    }
    switch (kindA * 3 + kindB) {          // features are 0/1-encoded in convolution mode
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
