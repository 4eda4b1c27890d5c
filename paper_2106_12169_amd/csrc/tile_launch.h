// Launchers of the tile kernel instances; each tile size lives in its own
// translation unit so the instances compile in parallel.
#pragma once
#include "tile_kernel.h"

namespace apnn {

// r = per-thread tile edge (8, 4 or 2); block tile is (16 r) x (16 r).
// vw = loader vector width in words (matrix mode: 4; conv mode: 4, 2 or 1).
// pmz = convolution over -1/+1 features with a validity plane (tile_kernel.h).
// Returns false if the combination is not instantiated.
bool launch_tile8(const TileParams &p, bool conv, int vw, bool use_xor, bool pmz, unsigned grid, hipStream_t st);
bool launch_tile4(const TileParams &p, bool conv, int vw, bool use_xor, bool pmz, unsigned grid, hipStream_t st);
bool launch_tile2(const TileParams &p, bool conv, int vw, bool use_xor, bool pmz, unsigned grid, hipStream_t st);

constexpr int kTileKC = 16;   // K words staged per chunk
#ifndef APNN_TILE_LV
#define APNN_TILE_LV 4
#endif
constexpr int kTileLV = APNN_TILE_LV;   // words per LDS read (2: ds_read_b64, 4: ds_read_b128)

}  // namespace apnn
