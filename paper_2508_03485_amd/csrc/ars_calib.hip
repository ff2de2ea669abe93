// Calibration-time kernels of the Adaptive Rotation Scheme (gfx950), all in fp64:
//   * the greedy outlier-aware rotation builder (Method, equation R^i = E_c* R~ Q E_c*, R^ = prod R^i), block-wise,
//     the staggered channel permutation P and the second rotation;
//   * the fluctuation metric J = ||X||_F / sqrt(B N C) (Method, Eq. J).
// These run once per layer on a few thousand calibration tokens; they are written for reproducibility (every sum
// is taken term by term in a fixed order with separately rounded multiply and add), not for speed.
#include "lrq_internal.h"

namespace lrq {
namespace {

constexpr int RB = 8;     // rows a workgroup multiplies at once

__global__ void bf16_to_f64_kernel(const uint16_t* __restrict__ X, size_t n, double* __restrict__ Y) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        Y[i] = (double)__uint_as_float((unsigned)X[i] << 16);
}

__global__ void block_identity_kernel(double* __restrict__ Rhat, int B, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const size_t e = i % ((size_t)B * B);
        Rhat[i] = (e / B == e % B) ? 1.0 : 0.0;
    }
}

// Per channel: max |y|, max y, min y over the T calibration tokens.  One thread per channel, 256 channels per
// workgroup, rows split over gridDim.y slices and merged with order-independent atomics on monotone keys.
__device__ __forceinline__ unsigned long long okey64(double v) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double okey64_inv(unsigned long long k) {
    return __longlong_as_double((long long)((k >> 63) ? (k & 0x7fffffffffffffffull) : ~k));
}

__global__ void channel_stats_kernel(const double* __restrict__ Y, int T, int K, unsigned long long* __restrict__ stats) {
    // stats[0][c]: key of max |y| (bits of a non-negative double order as integers), stats[1][c]: key of max y,
    // stats[2][c]: key of max (-y); all three must be zeroed before the launch
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    const int per = (T + gridDim.y - 1) / gridDim.y;
    const int t0 = blockIdx.y * per, t1 = min(T, t0 + per);
    if (t0 >= t1) return;
    double a = 0.0, hi = -INFINITY, lo = INFINITY;
    for (int t = t0; t < t1; ++t) {
        const double v = Y[(size_t)t * K + c];
        a = fmax(a, fabs(v));
        hi = fmax(hi, v);
        lo = fmin(lo, v);
    }
    atomicMax(&stats[c], (unsigned long long)__double_as_longlong(a));
    atomicMax(&stats[(size_t)K + c], okey64(hi));
    atomicMax(&stats[2 * (size_t)K + c], okey64(-lo));
}

__global__ void zero_u64_kernel(unsigned long long* __restrict__ p, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0ull;
}

// One greedy step applied to rows of S (the calibration activations, or the running product R^ whose rows are the
// B rows of each block): row <- E . ((row . E) . R~) . Q) with E the exchange of channels 0 and c* of the block;
// c* = first channel of the block with the largest max |y| (absmax: [K] keys from channel_stats_kernel).
// blockDim.x = B; blockIdx.x = block g; blockIdx.y = chunk of RB rows.  In place: a chunk is staged in LDS first.
// S element (row r, block g, channel j): S[g * blk_stride + r * row_stride + j].
__global__ void greedy_step_kernel(double* __restrict__ S, int rows, size_t blk_stride, size_t row_stride, int B,
                                   const unsigned long long* __restrict__ absmax, const double* __restrict__ Rtilde,
                                   const double* __restrict__ Q, size_t q_blk_stride) {
    extern __shared__ __attribute__((aligned(16))) double sm[];
    double* v = sm;                    // [RB][B]
    double* w = sm + RB * B;           // [RB][B]
    __shared__ unsigned long long best_key;
    __shared__ int best_idx;
    const int j = threadIdx.x, g = blockIdx.x;
    if (j == 0) { best_key = 0ull; best_idx = 0x7fffffff; }
    __syncthreads();
    const unsigned long long mine = absmax[(size_t)g * B + j];
    atomicMax(&best_key, mine);
    __syncthreads();
    if (mine == best_key) atomicMin(&best_idx, j);
    __syncthreads();
    const int cs = best_idx;
    const int src_j = j == 0 ? cs : (j == cs ? 0 : j);          // column exchange 0 <-> c*
    const int r0 = blockIdx.y * RB;
    double* base = S + (size_t)g * blk_stride;
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
        const int r = r0 + rr;
        v[rr * B + j] = r < rows ? base[(size_t)r * row_stride + src_j] : 0.0;
    }
    __syncthreads();
    double acc[RB];
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) acc[rr] = 0.0;
    for (int k = 0; k < B; ++k) {
        const double m = Rtilde[(size_t)k * B + j];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) acc[rr] = __dadd_rn(acc[rr], __dmul_rn(v[rr * B + k], m));
    }
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) w[rr * B + j] = acc[rr];
    __syncthreads();
    const double* Qg = Q + (size_t)g * q_blk_stride;
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) acc[rr] = 0.0;
    for (int k = 0; k < B; ++k) {
        const double m = Qg[(size_t)k * B + j];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) acc[rr] = __dadd_rn(acc[rr], __dmul_rn(w[rr * B + k], m));
    }
    // exchange back: output channel src_j takes this thread's value
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
        const int r = r0 + rr;
        if (r < rows) base[(size_t)r * row_stride + src_j] = acc[rr];
    }
}

__global__ void f64_to_bf16_kernel(const double* __restrict__ A, size_t n, uint16_t* __restrict__ out) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        // one rounding, fp64 -> bf16, nearest even: on the 64-bit pattern (bf16 keeps 7 of the 52 fraction bits; the
        // exponent is re-biased afterwards through an exact fp64 -> fp32 conversion of the already rounded value)
        const double a = A[i];
        unsigned long long b = (unsigned long long)__double_as_longlong(a);
        const unsigned long long lsb = (b >> 45) & 1ull;
        b += 0x00000FFFFFFFFFFFull + lsb;
        b &= ~0x00001FFFFFFFFFFFull;
        const float f = (float)__longlong_as_double((long long)b);     // exact: 8 significant bits, |a| well inside fp32 range
        out[i] = (uint16_t)(__float_as_uint(f) >> 16);
    }
}

// Staggered permutation: rank channels by range = max - min (descending, ties by channel index), deal ranks across
// the nb blocks left to right on even rounds and right to left on odd rounds.  perm[new] = old.
__global__ void zigzag_perm_kernel(const unsigned long long* __restrict__ stats, int K, int B, int32_t* __restrict__ perm) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    const unsigned long long* hi = stats + K;
    const unsigned long long* nlo = stats + 2 * (size_t)K;
    const double mine = okey64_inv(hi[c]) + okey64_inv(nlo[c]);         // max - min = max + max(-y): one rounded add
    int rank = 0;
    for (int o = 0; o < K; ++o) {
        const double other = okey64_inv(hi[o]) + okey64_inv(nlo[o]);
        rank += (other > mine) || (other == mine && o < c);
    }
    const int nb = K / B, rnd = rank / nb, pos = rank % nb;
    const int blk = (rnd % 2 == 0) ? pos : nb - 1 - pos;
    perm[blk * B + rnd] = c;
}

__global__ void permute_cols_f64_kernel(const double* __restrict__ in, const int32_t* __restrict__ perm, int T, int K,
                                        double* __restrict__ out) {
    const size_t n = (size_t)T * K, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const size_t t = i / K;
        const int j = (int)(i % K);
        out[i] = in[t * K + perm[j]];
    }
}

// J: sum of squares in fp64.  Each thread accumulates a strided slice, the workgroup reduces in LDS (tree), one
// atomic add of the workgroup's partial per launch slot; partials are summed by a second tiny kernel in slot order,
// so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void sumsq_partial_kernel(const uint16_t* __restrict__ X, size_t n8, double* __restrict__ part) {
    __shared__ double red[256];
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    double s = 0.0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
        const uint4 v = reinterpret_cast<const uint4*>(X)[i];
        const unsigned wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const double a = (double)__uint_as_float(wd[k] << 16), b = (double)__uint_as_float(wd[k] & 0xffff0000u);
            s += a * a;
            s += b * b;
        }
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

__global__ void j_finish_kernel(const double* __restrict__ part, int nparts, double count, double* __restrict__ J) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        double s = 0.0;
        for (int i = 0; i < nparts; ++i) s += part[i];
        J[0] = sqrt(s) / sqrt(count);
    }
}

// Column maxima of |a| for a [rows, K] matrix of bf16 or fp32: keys are the bit patterns of |a| as fp32 (monotone
// for non-negative floats), merged with atomicMax; keys must be zeroed first.  One thread per channel.
template <typename T>
__global__ void col_absmax_kernel(const T* __restrict__ A, int rows, int K, unsigned* __restrict__ keys) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    const int per = (rows + gridDim.y - 1) / gridDim.y;
    const int r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
    unsigned m = 0u;
    for (int r = r0; r < r1; ++r) {
        unsigned b;
        if constexpr (sizeof(T) == 2) b = ((unsigned)A[(size_t)r * K + c] << 16) & 0x7fffffffu;
        else b = __float_as_uint(A[(size_t)r * K + c]) & 0x7fffffffu;
        m = max(m, b);
    }
    if (r0 < r1) atomicMax(&keys[c], m);
}

__global__ void zero_u32_kernel(unsigned* __restrict__ p, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

__global__ void smooth_factor_kernel(const unsigned* __restrict__ akey, const unsigned* __restrict__ wkey, int K,
                                     double alpha, float* __restrict__ s_out, float* __restrict__ inv_out) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    const double a = (double)__uint_as_float(akey[c]), w = (double)__uint_as_float(wkey[c]);
    double s = 1.0;
    if (a > 0.0 && w > 0.0) s = (alpha == 0.5) ? sqrt(a / w) : pow(a, alpha) / pow(w, 1.0 - alpha);
    s_out[c] = (float)s;
    inv_out[c] = (float)(1.0 / s);
}

__global__ void scale_columns_kernel(const float* __restrict__ W, const float* __restrict__ s, size_t n, int K,
                                     float* __restrict__ out) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = W[i] * s[i % K];
}

inline int blocks_for(size_t n, int per = 256, int cap = 4096) {
    const size_t b = (n + per - 1) / per;
    return (int)(b < 1 ? 1 : (b > (size_t)cap ? (size_t)cap : b));
}

}  // namespace

size_t ars_build_workspace_bytes(int T, int K, int B) {
    return 2 * round256((size_t)T * K * sizeof(double)) + round256((size_t)K * B * sizeof(double)) +
           round256(3 * (size_t)K * sizeof(unsigned long long));
}

hipError_t launch_ars_build_rotation(hipStream_t st, const uint16_t* Xcal, int T, int K, int B, int n_steps,
                                     const double* Rtilde, const double* Q1, const double* Q2, uint16_t* R1,
                                     int32_t* perm, uint16_t* R2, void* ws) {
    char* p = static_cast<char*>(ws);
    double* Y = reinterpret_cast<double*>(p);            p += round256((size_t)T * K * sizeof(double));
    double* Yp = reinterpret_cast<double*>(p);           p += round256((size_t)T * K * sizeof(double));
    double* Rhat = reinterpret_cast<double*>(p);         p += round256((size_t)K * B * sizeof(double));
    unsigned long long* stats = reinterpret_cast<unsigned long long*>(p);
    const int nb = K / B;
    const size_t nY = (size_t)T * K, nR = (size_t)K * B;
    const size_t lds = 2 * RB * B * sizeof(double);
    const size_t q_blk = (size_t)n_steps * B * B;
    {
        const hipError_t e = allow_large_lds(reinterpret_cast<const void*>(greedy_step_kernel), 158 * 1024);
        if (e != hipSuccess) return e;
    }
    auto stats_pass = [&](const double* A) {
        hipLaunchKernelGGL(zero_u64_kernel, dim3(blocks_for(3 * (size_t)K)), dim3(256), 0, st, stats, 3 * (size_t)K);
        int slices = T / 64;
        slices = slices < 1 ? 1 : (slices > 64 ? 64 : slices);
        hipLaunchKernelGGL(channel_stats_kernel, dim3((K + 255) / 256, slices), dim3(256), 0, st, A, T, K, stats);
    };
    auto greedy = [&](double* A, const double* Q, uint16_t* Rout) {
        hipLaunchKernelGGL(block_identity_kernel, dim3(blocks_for(nR)), dim3(256), 0, st, Rhat, B, nR);
        for (int i = 0; i < n_steps; ++i) {
            stats_pass(A);
            const double* Qi = Q + (size_t)i * B * B;
            // the running product first (it reads the same c* as the activations: stats stay untouched in between)
            hipLaunchKernelGGL(greedy_step_kernel, dim3(nb, (B + RB - 1) / RB), dim3(B), lds, st, Rhat, B, (size_t)B * B,
                               (size_t)B, B, stats, Rtilde, Qi, q_blk);
            hipLaunchKernelGGL(greedy_step_kernel, dim3(nb, (T + RB - 1) / RB), dim3(B), lds, st, A, T, (size_t)B,
                               (size_t)K, B, stats, Rtilde, Qi, q_blk);
        }
        hipLaunchKernelGGL(f64_to_bf16_kernel, dim3(blocks_for(nR)), dim3(256), 0, st, Rhat, nR, Rout);
    };
    hipLaunchKernelGGL(bf16_to_f64_kernel, dim3(blocks_for(nY)), dim3(256), 0, st, Xcal, nY, Y);
    greedy(Y, Q1, R1);
    stats_pass(Y);
    hipLaunchKernelGGL(zigzag_perm_kernel, dim3((K + 255) / 256), dim3(256), 0, st, stats, K, B, perm);
    hipLaunchKernelGGL(permute_cols_f64_kernel, dim3(blocks_for(nY)), dim3(256), 0, st, Y, perm, T, K, Yp);
    greedy(Yp, Q2, R2);
    return hipGetLastError();
}

size_t smooth_workspace_bytes(int K) { return round256(2 * (size_t)K * sizeof(unsigned)); }

hipError_t launch_smooth_factor(hipStream_t st, const uint16_t* Xcal, int T, const float* W, int N, int K, double alpha,
                                float* s, float* inv_s, float* W_out, void* ws) {
    unsigned* akey = static_cast<unsigned*>(ws);
    unsigned* wkey = akey + K;
    hipLaunchKernelGGL(zero_u32_kernel, dim3(blocks_for(2 * (size_t)K)), dim3(256), 0, st, akey, 2 * (size_t)K);
    auto slices = [](int rows) { const int v = rows / 64; return v < 1 ? 1 : (v > 64 ? 64 : v); };
    hipLaunchKernelGGL((col_absmax_kernel<uint16_t>), dim3((K + 255) / 256, slices(T)), dim3(256), 0, st, Xcal, T, K, akey);
    hipLaunchKernelGGL((col_absmax_kernel<float>), dim3((K + 255) / 256, slices(N)), dim3(256), 0, st, W, N, K, wkey);
    hipLaunchKernelGGL(smooth_factor_kernel, dim3((K + 255) / 256), dim3(256), 0, st, akey, wkey, K, alpha, s, inv_s);
    if (W_out) {
        const size_t n = (size_t)N * K;
        hipLaunchKernelGGL(scale_columns_kernel, dim3(blocks_for(n)), dim3(256), 0, st, W, s, n, K, W_out);
    }
    return hipGetLastError();
}

size_t fluctuation_workspace_bytes() { return round256(1024 * sizeof(double)); }

hipError_t launch_fluctuation_metric(hipStream_t st, const uint16_t* X, size_t n, double* J, void* ws) {
    double* part = static_cast<double*>(ws);
    const int nparts = blocks_for(n / 8, 256 * 8, 1024);
    hipLaunchKernelGGL(sumsq_partial_kernel, dim3(nparts), dim3(256), 0, st, X, n / 8, part);
    hipLaunchKernelGGL(j_finish_kernel, dim3(1), dim3(64), 0, st, part, nparts, (double)n, J);
    return hipGetLastError();
}

}  // namespace lrq
