/*
 * apnn_debug.h -- test and experiment hooks of libapnn.so.  Nothing here is
 * needed to use the library: results are the same whatever is forced, only the
 * kernel that computes them changes.
 *
 * The library chooses between its AND/XOR + popcount kernel and its
 * matrix-instruction kernels, and among their tile sizes, from the problem
 * shape (the thread-level-parallelism / compute-intensity trade-off of
 * Sec. 4.3).  Tests force each choice in turn so that every kernel is compared
 * with the oracle; measurements force one to time it.
 *
 * Each override starts from the environment variable APNN_<name>, read once per
 * process (when the first dispatching call or the first call below is made),
 * and is unset (-1) when that variable is absent.
 *
 *   name          values
 *   MFMA          0: plane-pair AND/XOR + popcount kernel only
 *   INT8          0: never the 8-bit integer matrix form; 1: whenever it applies
 *   TILE          8 | 4 | 2: per-thread register tile edge of the popcount kernel
 *   MFMA_TILE     256 | 128 | 64 | 32: block tile of the matrix-instruction kernels
 *   MFMA_SMALL    0: chunked K loop also for 32 x 32 tiles
 *   MFMA_NSPLIT   1 | 4: waves of a block that split K of a 32 x 32 tile
 *   MFMA_FN       1 | 2: 32 x 32 or 32 x 64 wave tiles of the small-layer kernel
 *   MFMA_SHORTK   0: no special case for K <= 256
 * A forced value the dispatch cannot honour for a call is ignored for that call.
 */
#ifndef APNN_DEBUG_H
#define APNN_DEBUG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Sets override `name` to `value` (value < 0: unset).  Host only; affects the
 * calls made after it, on every thread.  Returns APNN_OK, or
 * APNN_ERR_INVALID_ARG for an unknown name. */
int apnn_debug_force(const char *name, int value);

/* Every override back to what the process environment says. */
void apnn_debug_reset(void);

/* The block tile edge (square tiles: 32, 64, 128 or 256 output rows and
 * columns) the dispatch would take for an M x N output: the two-step heuristic
 * of Sec. 4.3 -- rank the candidates by thread-level parallelism (Eq. 3), keep
 * the most parallel one if even it stays below its threshold, else take the
 * highest compute intensity (Eq. 4) whose parallelism reaches its threshold.
 * matrix_form != 0: the matrix-instruction kernels, else the popcount kernel;
 * is_conv != 0: convolution operands.  Overrides in force are honoured.
 * Host only, launches nothing; 0 for an empty output. */
int apnn_debug_tile_choice(int64_t M, int64_t N, int is_conv, int matrix_form);

#ifdef __cplusplus
}
#endif
#endif /* APNN_DEBUG_H */
