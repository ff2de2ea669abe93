// Measurement probes of the benchmark (a shared object of their own, loaded by bench.py only - not part of liblrq):
// a pure int8 MFMA loop and a plain copy kernel.  They give the sustained matrix rate and the copy bandwidth of the
// device the benchmark runs on, next to which the published peaks (and the fractions of them that the real kernels
// reach) can be read, and the copy calibrates the byte counters of rocprofv3.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned mix(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// Every wave issues iters x 65536 x 8 int8 multiply-accumulates as independent matrix instructions - 16 of
// v_mfma_i32_16x16x64_i8 per trip (WIDE = false: the GEMM's instruction) or 8 of v_mfma_i32_32x32x32_i8 (WIDE = true);
// nothing else competes for the pipe.
// random = 0: every operand byte is 1 (no data toggling); 1: pseudo-random operand bytes, four different A and four
// different B register sets in rotation (the matrix pipe's power draw, and with it the sustained clock, depends on
// how many operand bits toggle - and on the instruction: the 16 x 16 x 64 shape sustains the higher rate).
template <bool WIDE>
__global__ __launch_bounds__(256, 2) void mfma_i8_probe_kernel(int iters, int random, int* __restrict__ out) {
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned seed = (threadIdx.x * 16u + i * 4u + c) * 2654435761u + blockIdx.x;
            a[i][c] = random ? (int)mix(seed) : 0x01010101;
            b[i][c] = random ? (int)mix(seed ^ 0x9e3779b9u) : 0x01010101;
        }
    int s = 0;
    if constexpr (WIDE) {
        v16i acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i % 4], b[(i / 2) % 4], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
    } else {
        v4i acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i % 4], b[(i / 2) % 4], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][3];
    }
    if (s == 0x7fffffff) out[0] = s;   // keeps the loop alive; practically never taken
}

// One 16-byte element per thread, one workgroup per 4 KiB, streaming (non-temporal) accesses: workgroups are
// dispatched in order, so the chip sweeps both buffers as one compact moving window.  Measured faster than a
// persistent grid-stride loop (whose workgroups touch pages far apart) by 20 - 40 %.
typedef unsigned v4u __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_probe_kernel(const v4u* __restrict__ src, v4u* __restrict__ dst, size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

}  // namespace

extern "C" {

// `blocks` workgroups of 4 waves, each wave issuing iters x 8 x 65536 int8 operations; pattern 0 = all operand bytes 1,
// 1 = pseudo-random operand bytes, both with v_mfma_i32_16x16x64_i8; 2 and 3 = the same two with v_mfma_i32_32x32x32_i8.
// *ops_per_launch (host, may be NULL) receives the int8 operations one launch performs (2 per multiply-accumulate).
// out: int[1] device scratch.  Returns 0 or -1.
__attribute__((visibility("default"))) int bench_probe_mfma_i8(void* stream, int blocks, int iters, int pattern, int* out,
                                                                double* ops_per_launch) {
    if (blocks <= 0 || iters <= 0 || !out || pattern < 0 || pattern > 3) return -1;
    if (ops_per_launch) *ops_per_launch = 2.0 * 32 * 32 * 32 * 8.0 * iters * 4.0 * blocks;
    if (pattern < 2)
        hipLaunchKernelGGL(mfma_i8_probe_kernel<false>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, pattern, out);
    else
        hipLaunchKernelGGL(mfma_i8_probe_kernel<true>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), iters, pattern - 2, out);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Plain 16-byte-per-lane device copy of `bytes` (multiple of 16) from src to dst.  Returns 0 or -1.
__attribute__((visibility("default"))) int bench_probe_copy(void* stream, const void* src, void* dst, size_t bytes) {
    if (!src || !dst || bytes < 16) return -1;
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4u*>(src), static_cast<v4u*>(dst), n16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
