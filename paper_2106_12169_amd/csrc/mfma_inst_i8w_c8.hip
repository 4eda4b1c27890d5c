// Instances of the 8-bit integer matrix kernel with K shared out among the waves (mfma_i8_wide.h) whose row operand
// has plane class C8.
#include "mfma_i8_wide.h"
#include "mfma_launch.h"

namespace apnn {

template <int CB> static bool go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    auto kernel = mfma_i8_wide_kernel<I8_C8, CB>;
    const int lds = mfma_i8_wide_lds_bytes(p.PA, p.PB);
    static int granted = 0;                              // most dynamic LDS asked for so far (per instance)
    if (lds > granted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return false;
        granted = lds;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds, st, p);
    return true;
}

bool launch_mfma_i8_wide_c8(const MfmaParams &p, int classB, unsigned grid, hipStream_t st)
{
    switch (classB) {
        case I8_C2: return go<I8_C2>(p, grid, st);
        case I8_C4: return go<I8_C4>(p, grid, st);

        default: return false;                           // (both operands above four planes: more LDS than there is)
    }
}

}  // namespace apnn
