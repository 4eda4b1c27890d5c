// Measurement probes (libapnn_bench.so): a register-only AND + popcount chain for the
// sustained issue rate of the plane-pair inner operation (Sec. 3.1), and a plain copy
// of known size for scaling the memory-traffic counters, and a loop of one matrix
// instruction followed by a given number of independent vector instructions, run with
// one or two waves per SIMD, for the rate at which a SIMD issues them together.
// Nothing of the method is computed here.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/apnn_bench.h"

namespace {

// Register-only AND + popcount-accumulate chain on an 8 x 8 accumulator tile.
__global__ __launch_bounds__(256) void probe_valu_kernel(uint32_t *__restrict__ out, int iters)
{
    uint32_t a[8], b[8], acc[8][8];
    const uint32_t seed = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = seed * 2654435761u + i * 40503u;
        b[i] = ~seed * 2246822519u + i * 9176u;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
            asm volatile(
                "v_and_b32 %0, %16, %17\n\tv_and_b32 %1, %16, %18\n\tv_and_b32 %2, %16, %19\n\tv_and_b32 %3, %16, %20\n\t"
                "v_and_b32 %4, %16, %21\n\tv_and_b32 %5, %16, %22\n\tv_and_b32 %6, %16, %23\n\tv_and_b32 %7, %16, %24\n\t"
                "v_bcnt_u32_b32 %8, %0, %8\n\tv_bcnt_u32_b32 %9, %1, %9\n\tv_bcnt_u32_b32 %10, %2, %10\n\t"
                "v_bcnt_u32_b32 %11, %3, %11\n\tv_bcnt_u32_b32 %12, %4, %12\n\tv_bcnt_u32_b32 %13, %5, %13\n\t"
                "v_bcnt_u32_b32 %14, %6, %14\n\tv_bcnt_u32_b32 %15, %7, %15"
                : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7),
                  "+v"(acc[i][0]), "+v"(acc[i][1]), "+v"(acc[i][2]), "+v"(acc[i][3]), "+v"(acc[i][4]),
                  "+v"(acc[i][5]), "+v"(acc[i][6]), "+v"(acc[i][7])
                : "v"(a[i]), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "v"(b[4]), "v"(b[5]), "v"(b[6]), "v"(b[7]));
        }
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * 256;
    for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}


typedef int v8i_probe_t __attribute__((ext_vector_type(8)));
typedef float v16f_probe_t __attribute__((ext_vector_type(16)));

// Four accumulator tiles in turn: [FP4 matrix instruction (32 x 32 x 64)] + NV independent vector instructions each.
template <int NV, bool MFMA> __global__ __launch_bounds__(512) void probe_issue_kernel(uint32_t *__restrict__ out, int iters)
{
    v16f_probe_t acc[4];
    v8i_probe_t a[4], b;
    for (int j = 0; j < 4; ++j) {
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
        for (int r = 0; r < 8; ++r) a[j][r] = 0x22222222 + 0x01010101 * ((threadIdx.x + j + r) & 1);
    }
    for (int r = 0; r < 8; ++r) b[r] = 0x22222222;
    uint32_t x0 = threadIdx.x, x1 = threadIdx.x * 3, x2 = threadIdx.x * 5, x3 = threadIdx.x * 7;
    const uint32_t m = 0x33333333u + blockIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (MFMA) acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j], b, acc[j], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if ((v & 3) == 0) asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(x0) : "v"(m), "v"(x1));
                if ((v & 3) == 1) asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(x1) : "v"(m), "v"(x2));
                if ((v & 3) == 2) asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(x2) : "v"(m), "v"(x3));
                if ((v & 3) == 3) asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(x3) : "v"(m), "v"(x0));
            }
        }
    }
    float s = 0.0f;
    for (int j = 0; j < 4; ++j)
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = static_cast<uint32_t>(s) + (x0 ^ x1 ^ x2 ^ x3);
}

template <bool MFMA> bool launch_issue(int nv, dim3 grid, dim3 block, hipStream_t st, uint32_t *out, int iters)
{
    switch (nv) {
        case 0: hipLaunchKernelGGL((probe_issue_kernel<0, MFMA>), grid, block, 0, st, out, iters); return true;
        case 4: hipLaunchKernelGGL((probe_issue_kernel<4, MFMA>), grid, block, 0, st, out, iters); return true;
        case 8: hipLaunchKernelGGL((probe_issue_kernel<8, MFMA>), grid, block, 0, st, out, iters); return true;
        case 16: hipLaunchKernelGGL((probe_issue_kernel<16, MFMA>), grid, block, 0, st, out, iters); return true;
        default: return false;
    }
}

int launch_status()
{
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

}  // namespace

extern "C" int apnn_probe_valu(int blocks, int iters, uint32_t *out_dev, double *lane_ops, void *stream)
{
    if (blocks < 1 || iters < 1 || !out_dev) return 1;
    hipLaunchKernelGGL(probe_valu_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), out_dev, iters);
    if (lane_ops) *lane_ops = 128.0 * iters * 256.0 * blocks;   // 64 AND + 64 popcount-accumulate per iteration
    return launch_status();
}

extern "C" int apnn_probe_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream)
{
    if (!src_dev || !dst_dev || bytes % 16 != 0) return 1;
    if ((reinterpret_cast<uintptr_t>(src_dev) | reinterpret_cast<uintptr_t>(dst_dev)) & 15u) return 4;
    if (bytes == 0) return 0;
    const size_t n = bytes / 16;
    const unsigned grid = static_cast<unsigned>(n / 256 + 1 < 8192 ? n / 256 + 1 : 8192);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src_dev), static_cast<uint4 *>(dst_dev), n);
    return launch_status();
}

extern "C" int apnn_probe_issue(int vector_per_matrix, int with_matrix, int waves_per_simd, int iters, uint32_t *out_dev,
                                void *stream)
{
    if ((waves_per_simd != 1 && waves_per_simd != 2) || iters < 1 || !out_dev) return 1;
    if (!with_matrix && vector_per_matrix == 0) return 1;
    const dim3 grid(256), block(256 * waves_per_simd);   // one block per compute unit: 4 or 8 waves on its 4 SIMDs
    const bool ok = with_matrix ? launch_issue<true>(vector_per_matrix, grid, block, static_cast<hipStream_t>(stream), out_dev, iters)
                                : launch_issue<false>(vector_per_matrix, grid, block, static_cast<hipStream_t>(stream), out_dev, iters);
    if (!ok) return 1;
    return launch_status();
}
