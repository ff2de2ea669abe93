// Adaptive Rotation Scheme + per-token activation quantizer (gfx950).
//
// Every kernel here works in fp64 on the exact values of the bf16 inputs: the Hadamard butterflies
// (Preliminaries, Eq. hadamard, unnormalised +-1 form) are then exact additions, and the rounding
// decision q = rint(u * (qmax / amax)) is one division and one multiplication in IEEE fp64, so the
// integer codes do not depend on the order in which a kernel schedules its work.
#include "lrq_internal.h"

namespace lrq {
namespace {

constexpr int kWave = 64;

__device__ __forceinline__ void load8_bf16(const uint16_t* __restrict__ p, double v[8]) {
    const uint4 raw = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = (double)__uint_as_float(w[i] << 16);
        v[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
}

// n-point butterfly network on v[0..n), ascending strides, (a, b) -> (a + b, a - b).
template <int N>
__device__ __forceinline__ void butterflies(double* v, int stages) {
#pragma unroll
    for (int s = 0, st = 1; st < N; ++s, st <<= 1) {
        if (s < stages) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                if ((i & st) == 0) {
                    const double a = v[i], b = v[i + st];
                    v[i] = a + b;
                    v[i + st] = a - b;
                }
            }
        }
    }
}

__device__ __forceinline__ double wave_max(double m) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) m = fmax(m, __shfl_xor(m, o, kWave));
    return m;
}

// Block-wide maximum of non-negative doubles; red must hold blockDim.x / 64 doubles.
__device__ __forceinline__ double block_max(double m, double* red) {
    m = wave_max(m);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == 0) red[wave] = m;
    __syncthreads();
    const int nw = (blockDim.x + kWave - 1) / kWave;
    double r = red[0];
    for (int i = 1; i < nw; ++i) r = fmax(r, red[i]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ int quant1(double u, double inv, double qmax) {
    double r = rint(u * inv);
    r = fmin(fmax(r, -qmax), qmax);
    return (int)r;
}

__device__ __forceinline__ void store8_codes(int8_t* __restrict__ dst, const double v[8], double inv, double qmax) {
    unsigned lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        lo |= (unsigned)(quant1(v[i], inv, qmax) & 0xff) << (8 * i);
        hi |= (unsigned)(quant1(v[4 + i], inv, qmax) & 0xff) << (8 * i);
    }
    *reinterpret_cast<uint2*>(dst) = make_uint2(lo, hi);
}

// One workgroup per token row.  The row lives in LDS as doubles; the first three butterfly stages
// run in registers on each 8-element chunk, the remaining ones as radix-8 passes over LDS.
__global__ void hadamard_quant_generic_kernel(const uint16_t* __restrict__ X, int K, int log2h, double qmax,
                                              double norm, int8_t* __restrict__ q, float* __restrict__ scale) {
    extern __shared__ double lds[];
    double* row = lds;
    double* red = lds + K;
    const int t = threadIdx.x, nt = blockDim.x;
    const size_t base = (size_t)blockIdx.x * K;
    const int nchunks = K >> 3;
    const int s0 = log2h < 3 ? log2h : 3;
    for (int c = t; c < nchunks; c += nt) {
        double v[8];
        load8_bf16(X + base + (size_t)c * 8, v);
        butterflies<8>(v, s0);
#pragma unroll
        for (int i = 0; i < 8; ++i) row[c * 8 + i] = v[i];
    }
    __syncthreads();
    for (int pb = 3; pb < log2h; pb += 3) {
        const int nb = (log2h - pb) < 3 ? (log2h - pb) : 3;
        const int S = 1 << pb, n = 1 << nb;
        const int ngroups = K >> nb;
        for (int g = t; g < ngroups; g += nt) {
            const int idx0 = ((g >> pb) << (pb + nb)) | (g & (S - 1));
            double v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (j < n) ? row[idx0 + j * S] : 0.0;
            butterflies<8>(v, nb);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < n) row[idx0 + j * S] = v[j];
        }
        __syncthreads();
    }
    double m = 0.0;
    for (int i = t; i < K; i += nt) m = fmax(m, fabs(row[i]));
    const double amax = block_max(m, red);
    const double inv = amax > 0.0 ? qmax / amax : 0.0;
    for (int c = t; c < nchunks; c += nt) {
        double v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = row[c * 8 + i];
        store8_codes(q + base + (size_t)c * 8, v, inv, qmax);
    }
    if (t == 0) scale[blockIdx.x] = (float)(amax / norm);
}

// ---------------------------------------------------------------- dense rotation, fp64, k ascending
constexpr int DT = 64;   // output tile (rows x cols) of one workgroup
constexpr int DK = 16;   // K step

__global__ __launch_bounds__(256) void dense_rotate_f64_kernel(const uint16_t* __restrict__ X,
                                                                const uint16_t* __restrict__ R, int M, int K,
                                                                double* __restrict__ U) {
    __shared__ double Xs[DK][DT + 1];
    __shared__ double Rs[DK][DT];
    const int t = threadIdx.x;
    const int row0 = blockIdx.y * DT, col0 = blockIdx.x * DT;
    const int ty = t / 16, tx = t % 16;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    const int xr = t / 4, xk = (t % 4) * 4;      // X tile: 64 rows x 16 k, 4 bf16 per thread
    const int rk = t / 16, rc = (t % 16) * 4;    // R tile: 16 k x 64 cols, 4 bf16 per thread
    int xrow = row0 + xr;
    if (xrow >= M) xrow = M - 1;
    for (int k0 = 0; k0 < K; k0 += DK) {
        const uint2 xa = *reinterpret_cast<const uint2*>(X + (size_t)xrow * K + k0 + xk);
        const uint2 ra = *reinterpret_cast<const uint2*>(R + (size_t)(k0 + rk) * K + col0 + rc);
        Xs[xk + 0][xr] = (double)__uint_as_float(xa.x << 16);
        Xs[xk + 1][xr] = (double)__uint_as_float(xa.x & 0xffff0000u);
        Xs[xk + 2][xr] = (double)__uint_as_float(xa.y << 16);
        Xs[xk + 3][xr] = (double)__uint_as_float(xa.y & 0xffff0000u);
        Rs[rk][rc + 0] = (double)__uint_as_float(ra.x << 16);
        Rs[rk][rc + 1] = (double)__uint_as_float(ra.x & 0xffff0000u);
        Rs[rk][rc + 2] = (double)__uint_as_float(ra.y << 16);
        Rs[rk][rc + 3] = (double)__uint_as_float(ra.y & 0xffff0000u);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < DK; ++kk) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Xs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Rs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = row0 + ty * 4 + i;
        if (r < M) {
            double* dst = U + (size_t)r * K + col0 + tx * 4;
            *reinterpret_cast<double2*>(dst) = make_double2(acc[i][0], acc[i][1]);
            *reinterpret_cast<double2*>(dst + 2) = make_double2(acc[i][2], acc[i][3]);
        }
    }
}

// One workgroup per row: absmax and codes from fp64 U.
__global__ void quant_from_f64_kernel(const double* __restrict__ U, int K, double qmax, double norm,
                                      int8_t* __restrict__ q, float* __restrict__ scale) {
    __shared__ double red[16];
    const int t = threadIdx.x, nt = blockDim.x;
    const size_t base = (size_t)blockIdx.x * K;
    double m = 0.0;
    for (int i = t; i < K; i += nt) m = fmax(m, fabs(U[base + i]));
    const double amax = block_max(m, red);
    const double inv = amax > 0.0 ? qmax / amax : 0.0;
    for (int c = t; c < (K >> 3); c += nt) {
        double v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = U[base + (size_t)c * 8 + i];
        store8_codes(q + base + (size_t)c * 8, v, inv, qmax);
    }
    if (t == 0) scale[blockIdx.x] = (float)(amax / norm);
}

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

int threads_for_row(int K) {
    int nt = ((K / 8 + kWave - 1) / kWave) * kWave;
    if (nt > 1024) nt = 1024;
    return nt;
}

}  // namespace

hipError_t launch_hadamard_quant(hipStream_t st, const uint16_t* X, int M, int K, int h, int act_bits,
                                 int8_t* q, float* scale) {
    const double qmax = (double)((1 << (act_bits - 1)) - 1);
    const double norm = qmax * sqrt((double)h);
    const int nt = threads_for_row(K);
    const size_t lds = (size_t)(K + 16) * sizeof(double);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(hadamard_quant_generic_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(hadamard_quant_generic_kernel, dim3(M), dim3(nt), lds, st, X, K, ilog2(h), qmax, norm, q, scale);
    return hipGetLastError();
}

hipError_t launch_plain_quant(hipStream_t st, const uint16_t* X, int M, int K, int act_bits, int8_t* q,
                              float* scale) {
    return launch_hadamard_quant(st, X, M, K, 1, act_bits, q, scale);
}

hipError_t launch_dense_rotate_quant(hipStream_t st, const uint16_t* X, const uint16_t* R, int M, int K,
                                     int act_bits, double* U, int8_t* q, float* scale) {
    const double qmax = (double)((1 << (act_bits - 1)) - 1);
    dim3 grid(K / DT, (M + DT - 1) / DT);
    hipLaunchKernelGGL(dense_rotate_f64_kernel, grid, dim3(256), 0, st, X, R, M, K, U);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(quant_from_f64_kernel, dim3(M), dim3(256), 0, st, U, K, qmax, qmax, q, scale);
    return hipGetLastError();
}

}  // namespace lrq
