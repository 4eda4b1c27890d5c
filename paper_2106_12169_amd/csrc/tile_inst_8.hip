// Instances of the tile kernel with a 8 x 8 register tile per thread.
#include "tile_launch.h"

namespace apnn {

template <int VW, bool CONV, bool XOR, bool PMZ = false>
static void go(const TileParams &p, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((tile_kernel<8, 8, kTileKC, VW, kTileLV, CONV, XOR, PMZ>), dim3(grid), dim3(256), 0, st, p);
}

bool launch_tile8(const TileParams &p, bool conv, int vw, bool use_xor, bool pmz, unsigned grid, hipStream_t st)
{
    if (!conv) {
        if (vw != 4 || pmz) return false;
        if (use_xor) go<4, false, true>(p, grid, st); else go<4, false, false>(p, grid, st);
        return true;
    }
    if (use_xor) return false;
    // narrower loader vectors need more loader slots than the 8 x 8 register budget allows
    switch (vw) {
        case 4: if (pmz) go<4, true, false, true>(p, grid, st); else go<4, true, false>(p, grid, st); return true;
        default: return false;
    }
}

}  // namespace apnn
