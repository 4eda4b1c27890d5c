// Instances of the 8-bit integer matrix kernel (128 x 128 block tile) whose row operand has plane class C4.
#include "mfma_i8.h"
#include "mfma_launch.h"

namespace apnn {

// Two waves per SIMD (K split over wave pairs) while the registers of a wave hold its plane words twice over;
// the widest class pair runs one wave per SIMD.
template <int CB, int G> static bool go(const MfmaParams &p, unsigned grid, hipStream_t st)
{
    constexpr int NKS = I8Slots<1>::value + I8Slots<CB>::value <= 12 ? 2 : 1;
    auto kernel = mfma_i8_kernel<1, CB, 2, 2, G, NKS>;
    const int lds = mfma_i8_lds_bytes(p.PA, p.PB, G, NKS);
    static int granted = 0;                              // most dynamic LDS asked for so far (per instance)
    if (lds > granted) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return false;
        granted = lds;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256 * NKS), lds, st, p);
    return true;
}

bool launch_mfma_i8_c4(const MfmaParams &p, int classB, int group, unsigned grid, hipStream_t st)
{
    switch (classB * 8 + group) {
        case I8_C2 * 8 + 4: return go<I8_C2, 4>(p, grid, st);
        case I8_C4 * 8 + 4: return go<I8_C4, 4>(p, grid, st);
        case I8_C8 * 8 + 4: return go<I8_C8, 4>(p, grid, st);
        case I8_C2 * 8 + 2: return go<I8_C2, 2>(p, grid, st);
        case I8_C4 * 8 + 2: return go<I8_C4, 2>(p, grid, st);
        case I8_C8 * 8 + 2: return go<I8_C8, 2>(p, grid, st);
        default: return false;
    }
}

}  // namespace apnn
