/*
 * apnn_bench.h -- measurement helpers, built into a library of their own
 * (libapnn_bench.so): the benchmark uses them to measure the sustained rates
 * its roofline figures are quoted against.  They compute nothing of the method
 * and libapnn.so does not contain them.
 *
 * Same conventions as apnn.h: *_dev pointers are caller-owned device memory,
 * `stream` is the caller's hipStream_t as void*, calls enqueue and return, the
 * return value is 0 on success and nonzero on a bad argument or a failed launch.
 */
#ifndef APNN_BENCH_H
#define APNN_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Register-only AND + popcount-accumulate chain (the inner operation of the
 * plane-pair product, Sec. 3.1): every lane of `blocks` x 256 threads issues
 * 128 * iters lane-operations; the per-lane checksums go to out_dev
 * (blocks * 256 words).  *lane_ops receives the lane-operation count of the
 * launch.  Measures the sustained bitwise + popcount issue rate. */
int apnn_probe_valu(int blocks, int iters, uint32_t *out_dev, double *lane_ops, void *stream);

/* Plain 16-byte-per-lane copy of `bytes` (a multiple of 16; both pointers
 * 16-byte aligned) from src_dev to dst_dev: the known-size kernel that the
 * memory-traffic counters are scaled by. */
int apnn_probe_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream);

/* Issue-rate probe: 256 blocks (one per compute unit) of 4 or 8 waves
 * (waves_per_simd 1 or 2) run `iters` rounds of four slots, a slot being one
 * FP4 matrix instruction (32 x 32 x 64; left out if with_matrix is 0) followed
 * by vector_per_matrix (0, 4, 8 or 16) independent vector instructions, all on
 * registers.  Device time / (4 iters waves_per_simd) is the time a SIMD needs
 * per slot: it shows how many vector instructions run underneath a matrix
 * instruction, which is what the kernels' schedules are built around.
 * out_dev: 256 * 256 * waves_per_simd words of checksums. */
int apnn_probe_issue(int vector_per_matrix, int with_matrix, int waves_per_simd, int iters, uint32_t *out_dev,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* APNN_BENCH_H */
