// Twin-Log Quantization of a weight matrix: calibrate (search-based clipping), encode, build the
// per-channel int8 level table and pack (Method, "Twin-Log Quantization for Weights").  Offline step:
// one workgroup per output channel, fp64 throughout, written for clarity rather than speed.
#include "lrq_internal.h"

namespace lrq {
namespace {

constexpr int NT = 256;
constexpr int kWave = 64;

struct Red4 {
    double pmax, pmin, nmax, nmin;
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ double wave_maxd(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ double wave_mind(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmin(v, __shfl_xor(v, o, kWave));
    return v;
}

// Sum of the workgroup's NT per-thread values in ascending thread order, one fp64 addition after the other (the order
// the search objective is defined in); red must hold NT doubles.  Every thread returns the same bits.
__device__ __forceinline__ double block_sum_ascending(double v, double* red) {
    red[threadIdx.x] = v;
    __syncthreads();
    double r = 0.0;
    for (int i = 0; i < NT; ++i) r = r + red[i];
    __syncthreads();
    return r;
}

__device__ __forceinline__ double block_sum(double v, double* red) {
    v = wave_sum(v);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int i = 0; i < NT / kWave; ++i) r += red[i];
    __syncthreads();
    return r;
}

__device__ __forceinline__ double clampd(double v, double lo, double hi) { return fmin(fmax(v, lo), hi); }

// Grid search of one clip factor for one sign (Eq. hyperparameters clip); all threads return the
// same (s, z, factor).  sgn = +1 scans the positive weights, -1 the negative ones.
// ggrid / ngamma: optional grid of the lower clip factor (extension: s = (c W_max - g W_min) / intervals,
// z = round(g W_min / s)), scanned inside the loop over c; ngamma = 0 is the paper's formula (g = 1).
// The objective of a candidate is summed in a fixed order: thread j adds the terms of k = j, j + NT, j + 2 NT, ...
// one after the other, then the NT partial sums are added in ascending j - so which of two close candidates is the
// smaller one does not depend on the reduction tree.
__device__ void search_side(const float* __restrict__ w, const double* __restrict__ ell, int K, double sgn,
                            bool has, double wmax, double wmin, const float* __restrict__ grid, int ngrid,
                            const float* __restrict__ ggrid, int ngamma,
                            double nint, double qlo, double qhi, double* red, double& s_out, double& z_out,
                            float& c_out, float& g_out, double& err_out) {
    double best_err = INFINITY, best_s = 1.0, best_z = has ? rint(wmin) : 0.0;
    float best_c = 1.0f, best_g = 1.0f;
    const int ng = ngamma > 0 ? ngamma : 1;
    for (int ci = 0; ci < ngrid; ++ci)
    for (int gi = 0; gi < ng; ++gi) {
        const float c32 = grid[ci];
        const float g32 = ngamma > 0 ? ggrid[gi] : 1.0f;
        const double T = (double)c32 * wmax;
        const double B = (double)g32 * wmin;
        if (!(has && T > B)) continue;                       // uniform over the workgroup
        const double s = (T - B) / nint;
        const double z = rint(B / s);
        double err = 0.0;
        for (int k = threadIdx.x; k < K; k += NT) {
            const double wk = (double)w[k];
            if (wk * sgn > 0.0) {
                const double qv = clampd(rint(ell[k] / s) - z, qlo, qhi);
                const double d = exp2(s * (qv + z)) - fabs(wk);
                err = err + d * d;
            }
        }
        err = block_sum_ascending(err, red);
        if (err < best_err) {
            best_err = err;
            best_s = s;
            best_z = z;
            best_c = c32;
            best_g = g32;
        }
    }
    s_out = best_s;
    z_out = best_z;
    c_out = best_c;
    g_out = best_g;
    err_out = best_err;
}

// Round-to-nearest-even bf16 of a double.  The detour over fp32 could round twice only when the fp32 value lands
// exactly on a bf16 midpoint; the sign of what the first rounding dropped then decides the tie.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
    const float f = (float)x;
    unsigned u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);     // inf / nan
    const double d = fabs(x) - fabs((double)f);
    if ((u & 0xffffu) == 0x8000u && d != 0.0) return (uint16_t)((u >> 16) + (d > 0.0 ? 1u : 0u));
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Round-to-nearest-even FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest value
// 448, subnormals in steps of 2^-9) of a double, saturating.
__device__ __forceinline__ uint8_t f64_to_e4m3_rne(double x) {
    const unsigned sgn = x < 0.0 ? 0x80u : 0u;
    const double a = fmin(fabs(x), 448.0);
    if (!(a > 0.0)) return (uint8_t)sgn;
    int e = ilogb(a);
    e = e < -6 ? -6 : e;                                   // below 2^-6 everything shares the subnormal spacing
    double n = rint(ldexp(a, 3 - e));                      // multiples of 2^(e - 3): 8 .. 16 for a normal, 0 .. 8 below
    if (n >= 16.0) { n = 8.0; ++e; }
    if (e > 8 || (e == 8 && n > 14.0)) return (uint8_t)(sgn | 0x7eu);
    if (n < 8.0) return (uint8_t)(sgn | (unsigned)n);      // subnormal (n = 8 at e = -6 is the smallest normal)
    return (uint8_t)(sgn | ((unsigned)(e + 7) << 3) | ((unsigned)n - 8u));
}

__global__ __launch_bounds__(NT) void tlq_quantize_pack_kernel(
    const float* __restrict__ W, int N, int K, int bits, int I, const float* __restrict__ agrid, int na,
    const float* __restrict__ bgrid, int nb, uint8_t* __restrict__ codes_out, double* __restrict__ s_pos,
    double* __restrict__ s_neg, int32_t* __restrict__ z_pos, int32_t* __restrict__ z_neg,
    float* __restrict__ alpha, float* __restrict__ beta, int8_t* __restrict__ lut, float* __restrict__ wscale,
    uint8_t* __restrict__ gemm_codes, int32_t* __restrict__ colsum, const float* __restrict__ ggrid, int ngamma,
    float* __restrict__ gamma_pos, float* __restrict__ gamma_neg, uint16_t* __restrict__ levels,
    double* __restrict__ err_pos, double* __restrict__ err_neg, uint8_t* __restrict__ lut_fp8, float* __restrict__ wscale_fp8) {
    extern __shared__ double sm[];
    double* ell = sm;                                   // K doubles: log2|w|
    double* red = sm + K;                               // NT doubles of reduction scratch
    int8_t* code = reinterpret_cast<int8_t*>(red + NT); // K signed codes
    const int n = blockIdx.x, t = threadIdx.x;
    const float* w = W + (size_t)n * K;
    const int half = 1 << (bits - 1), nlev = 1 << bits;

    // W' = log2|W| and the per-sign extrema over the masked positions
    double pmax = -INFINITY, pmin = INFINITY, nmax = -INFINITY, nmin = INFINITY;
    for (int k = t; k < K; k += NT) {
        const double wk = (double)w[k];
        const double l = wk != 0.0 ? log2(fabs(wk)) : 0.0;
        ell[k] = l;
        if (wk > 0.0) { pmax = fmax(pmax, l); pmin = fmin(pmin, l); }
        if (wk < 0.0) { nmax = fmax(nmax, l); nmin = fmin(nmin, l); }
    }
    pmax = wave_maxd(pmax); pmin = wave_mind(pmin); nmax = wave_maxd(nmax); nmin = wave_mind(nmin);
    Red4* r4 = reinterpret_cast<Red4*>(red);
    if (t % kWave == 0) r4[t / kWave] = Red4{pmax, pmin, nmax, nmin};
    __syncthreads();
    for (int i = 0; i < NT / kWave; ++i) {
        pmax = fmax(pmax, r4[i].pmax); pmin = fmin(pmin, r4[i].pmin);
        nmax = fmax(nmax, r4[i].nmax); nmin = fmin(nmin, r4[i].nmin);
    }
    __syncthreads();
    const bool has_p = pmax >= pmin, has_n = nmax >= nmin;   // +-inf sentinels survive on an empty side
    if (!has_p) pmax = pmin = 0.0;
    if (!has_n) nmax = nmin = 0.0;

    double sp, zp, sn, zn, ep, en;
    float al, be, gp, gn;
    search_side(w, ell, K, 1.0, has_p, pmax, pmin, agrid, na, ggrid, ngamma, (double)(half - 1), 0.0, (double)(half - 1),
                red, sp, zp, al, gp, ep);
    search_side(w, ell, K, -1.0, has_n, nmax, nmin, bgrid, nb, ggrid, ngamma, (double)half, 1.0, (double)half, red, sn, zn,
                be, gn, en);

    if (t == 0) {
        s_pos[n] = sp; s_neg[n] = sn; z_pos[n] = (int32_t)zp; z_neg[n] = (int32_t)zn;
        alpha[n] = al; beta[n] = be;
        if (gamma_pos) gamma_pos[n] = gp;
        if (gamma_neg) gamma_neg[n] = gn;
        if (err_pos) err_pos[n] = ep;
        if (err_neg) err_neg[n] = en;
    }

    // level table: e(c) = s+(c + z+) for c >= 0, s-(-c + z-) for c < 0; exponent split and integerisation
    double v = 0.0;
    if (t < nlev) {
        const int c = t < half ? t : t - nlev;              // signed code whose low bits are t
        const double e = c >= 0 ? sp * ((double)c + zp) : sn * ((double)(-c) + zn);
        double mag;
        if (I < 0) {
            mag = exp2(e);
        } else {
            const double f = floor(e), r = e - f;
            const double mant = rint(exp2(r) * (double)(1 << I));
            mag = ldexp(mant, (int)f - I);
        }
        v = c >= 0 ? mag : -mag;
        red[t] = fabs(v);
    }
    __syncthreads();
    double vmax = 0.0;
    for (int i = 0; i < nlev; ++i) vmax = fmax(vmax, red[i]);
    const float ws = (float)(vmax / 127.0);
    __shared__ int lutv[16];
    if (t < 16) {
        int8_t entry = 0;
        if (t < nlev) entry = (int8_t)(int)clampd(rint(v / (double)ws), -127.0, 127.0);
        lut[(size_t)n * 16 + t] = entry;
        lutv[t] = entry;
        if (levels) levels[(size_t)n * 16 + t] = t < nlev ? f64_to_bf16_rne(v) : (uint16_t)0;
    }
    if (t == 0) wscale[n] = ws;

    // the same levels with I = 3 as FP8 E4M3 operands: divided by the power of two that puts the largest in [128, 256)
    if (lut_fp8 && wscale_fp8) {
        __syncthreads();
        double v3 = 0.0;
        if (t < nlev) {
            const int c = t < half ? t : t - nlev;
            const double e = c >= 0 ? sp * ((double)c + zp) : sn * ((double)(-c) + zn);
            const double f = floor(e), r = e - f;
            const double mag = ldexp(rint(exp2(r) * 8.0), (int)f - 3);
            v3 = c >= 0 ? mag : -mag;
            red[t] = mag;
        }
        __syncthreads();
        double m3 = 0.0;
        for (int i = 0; i < nlev; ++i) m3 = fmax(m3, red[i]);
        const int ex = (m3 > 0.0 ? ilogb(m3) : 0) - 7;
        if (t < 16) lut_fp8[(size_t)n * 16 + t] = t < nlev ? f64_to_e4m3_rne(ldexp(v3, -ex)) : (uint8_t)0;
        if (t == 0) wscale_fp8[n] = ldexpf(1.0f, ex);
        __syncthreads();
    }

    // codes (Eq. log-based quantizer); the negative twin is clamped to [1, 2^(b-1)]
    for (int k = t; k < K; k += NT) {
        const double wk = (double)w[k];
        int c = 0;
        if (wk > 0.0) c = (int)clampd(rint(ell[k] / sp) - zp, 0.0, (double)(half - 1));
        else if (wk < 0.0) c = -(int)clampd(rint(ell[k] / sn) - zn, 1.0, (double)half);
        code[k] = (int8_t)c;
    }
    __syncthreads();

    const unsigned mask = (unsigned)nlev - 1u;
    {   // sum of the channel's decoded levels (exact in fp64: |sum| <= 127 K)
        double part = 0.0;
        for (int k = t; k < K; k += NT) part += (double)lutv[(unsigned)code[k] & mask];
        const double tot = block_sum(part, red);
        if (t == 0) colsum[n] = (int32_t)tot;
    }
    if (bits == 4) {
        // canonical: byte j = code[2j] | code[2j+1] << 4, written 4 bytes at a time
        uint32_t* dst = reinterpret_cast<uint32_t*>(codes_out + (size_t)n * (K / 2));
        for (int g = t; g < K / 8; g += NT) {
            unsigned canon = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) canon |= ((unsigned)code[g * 8 + i] & mask) << (4 * i);
            dst[g] = canon;
        }
    } else {
        // canonical: 8 codes -> 24-bit little-endian group
        uint8_t* dst = codes_out + (size_t)n * (K / 8 * 3);
        for (int g = t; g < K / 8; g += NT) {
            unsigned v24 = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) v24 |= ((unsigned)code[g * 8 + i] & mask) << (3 * i);
            dst[g * 3 + 0] = (uint8_t)(v24 & 255u);
            dst[g * 3 + 1] = (uint8_t)((v24 >> 8) & 255u);
            dst[g * 3 + 2] = (uint8_t)(v24 >> 16);
        }
    }
    // GEMM layout, either bit-width: one nibble per code (a 3-bit code leaves its top bit clear, so that a single
    // AND turns a dword into four byte-permute selectors); byte j of a dword = code[k+j] | code[k+4+j] << 4
    for (int g = t; g < K / 8; g += NT) {
        unsigned tiled = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            tiled |= (((unsigned)code[g * 8 + j] & mask) | (((unsigned)code[g * 8 + 4 + j] & mask) << 4)) << (8 * j);
        // slot (n % 16, 16-k group kq) of the unit; the channel's half of its 32-tile picks the slot's 8-byte half
        const int kb = g / 8, r = g % 8, kq = r / 2, d = r % 2;
        const size_t unit = (size_t)(n / kGemmTileN) * (K / kGemmBlockK) + kb;
        const size_t off = (unit * 64 + (n % 16) + 16 * kq) * 16 + (((n % kGemmTileN) / 16) * 2 + d) * 4;
        *reinterpret_cast<uint32_t*>(gemm_codes + off) = tiled;
    }
}

}  // namespace

hipError_t launch_tlq_quantize_pack(hipStream_t st, const float* W, int N, int K, int bits, int I,
                                    const float* alpha_grid, int n_alpha, const float* beta_grid, int n_beta,
                                    const lrq_tlq_weight& out, const float* gamma_grid, int n_gamma, float* gamma_pos,
                                    float* gamma_neg) {
    const size_t lds = (size_t)K * sizeof(double) + NT * sizeof(double) + (size_t)K;
    {
        const hipError_t e = allow_large_lds(reinterpret_cast<const void*>(tlq_quantize_pack_kernel), 158 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(tlq_quantize_pack_kernel, dim3(N), dim3(NT), lds, st, W, N, K, bits, I, alpha_grid, n_alpha,
                       beta_grid, n_beta, out.codes, out.s_pos, out.s_neg, out.z_pos, out.z_neg, out.alpha, out.beta,
                       out.lut, out.wscale, out.gemm_codes, out.colsum, gamma_grid, n_gamma, gamma_pos, gamma_neg, out.levels,
                       out.err_pos, out.err_neg, out.lut_fp8, out.wscale_fp8);
    return hipGetLastError();
}

}  // namespace lrq
