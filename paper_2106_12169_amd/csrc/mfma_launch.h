// Launchers of the FP4 matrix-core kernel instances (one translation unit per
// block-tile size so they compile in parallel).
#pragma once
#include "mfma_kernel.h"

namespace apnn {

// tile: 256 (256 x 256 block, 4 waves, mfma_big_kernel), 128 (128 x 128, 4 waves), 64 (64 x 64, 4 waves),
// 32 (32 x 32, 4 waves splitting K).
// Returns false if the combination is not instantiated.
bool launch_mfma256(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st);
bool launch_mfma128(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st);
bool launch_mfma64(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st);
bool launch_mfma64_k8(const MfmaParams &p, int kindA, int kindB, unsigned grid, hipStream_t st);   // K <= 8 words
bool launch_mfma32(const MfmaParams &p, int kindA, int kindB, bool conv, unsigned grid, hipStream_t st);

// Small-layer kernel (lane-private operand loads, 32 x 32 tiles); nsplit = 1: one
// tile per wave (grid = ceil(tiles / 4)), nsplit = 4: one tile per block, K split
// over its waves (grid = tiles).  vw: conv loader vector width in words (4 or 2).
bool launch_mfma_small_conv(const MfmaParams &p, int kindA, int kindB, int vw, int nsplit, int gmax, unsigned grid,
                            hipStream_t st);
// One wave tile of 32 x 32 fn outputs per wave, no K split (fn = 2; grid = ceil(row tiles x ceil(N / (32 fn)) / 4)).
bool launch_mfma_small_conv_wide(const MfmaParams &p, int kindA, int kindB, int vw, int fn, unsigned grid, hipStream_t st);
// Two convolution layers in one launch (nsplit = 4 both; gmax: the larger of the two, rounded to an instance).
bool launch_mfma_small_conv_pair(const MfmaParams &p0, unsigned grid0, const MfmaParams &p1, unsigned grid1, int kindA,
                                 int kindB, int vw, int gmax, hipStream_t st);
bool launch_mfma_small_matrix(const MfmaParams &p, int kindA, int kindB, int nsplit, unsigned grid, hipStream_t st);

// 8-bit integer matrix form (matrix operands, 128 x 128 block tile); class: 0, 1, 2 for up to 2, 4, 8 planes.
bool launch_mfma_i8(const MfmaParams &p, int classA, int classB, unsigned grid, hipStream_t st);
// The same with K, not the outputs, shared out among the four waves of a block (up to 10 planes in all, not both
// operands above four); false if there is no such instance.
bool launch_mfma_i8_wide(const MfmaParams &p, int classA, int classB, unsigned grid, hipStream_t st);

// K words per chunk of each tile size (must match the instances).
constexpr int mfma_chunk_words(int tile) { return tile == 256 ? 16 : tile == 128 ? 16 : 32; }

}  // namespace apnn
