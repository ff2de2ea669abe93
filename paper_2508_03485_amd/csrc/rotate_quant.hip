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

// v[i] *= ps[i] for 8 consecutive channels: a bf16 value times an fp32 value is exact in fp64.
__device__ __forceinline__ void prescale8(const float* __restrict__ ps, double v[8]) {
    const float4 a = reinterpret_cast<const float4*>(ps)[0], b = reinterpret_cast<const float4*>(ps)[1];
    v[0] *= (double)a.x; v[1] *= (double)a.y; v[2] *= (double)a.z; v[3] *= (double)a.w;
    v[4] *= (double)b.x; v[5] *= (double)b.y; v[6] *= (double)b.z; v[7] *= (double)b.w;
}

// n-point butterfly network on v[0..n), ascending strides first_stride, 2*first_stride, ... for `stages`
// stages, (a, b) -> (a + b, a - b).
template <int N, int FIRST = 1>
__device__ __forceinline__ void butterflies(double* v, int stages) {
#pragma unroll
    for (int s = 0, st = FIRST; st < N; ++s, st <<= 1) {
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

// ---- per-token quantizer ---------------------------------------------------------------------------------
// Symmetric form: amax = max |u|, inv = qmax / amax, code = rint(u * inv), scale = amax / (qmax sqrt(h)).
// Zero-point form (Eq. 1 as printed): range = max u - min u, L = 2^b - 1, inv = L / range, z = rint(min u * inv),
// x_q = clamp(rint(u * inv) - z, 0, L), s = range / L; stored as q = x_q - 2^(b-1) and zero = z + 2^(b-1), so
// that x_f = scale (q + zero), scale = s / sqrt(h).  A constant token takes x_q = 0 and (s, z) = (|c|, sign c).
struct RowQ {
    double inv;     // multiplier of u
    double zsub;    // zero-point form: what is subtracted from rint(u * inv) before the clamp to [-half, half-1]
    float scale;
    int izero;
};

__device__ __forceinline__ RowQ rowq_sym(double amax, const QuantSpec& qs) {
    RowQ r;
    r.inv = amax > 0.0 ? qs.qmax / amax : 0.0;
    r.zsub = 0.0;
    r.scale = (float)(amax / qs.norm);
    r.izero = 0;
    return r;
}

__device__ __forceinline__ RowQ rowq_asym(double vmax, double vmin, const QuantSpec& qs) {
    RowQ r;
    const double rng = vmax - vmin;
    double sc, z;
    if (rng > 0.0) {
        r.inv = qs.L / rng;
        sc = rng / qs.L;
        z = rint(vmin * r.inv);
        r.zsub = z + qs.half;
    } else {
        r.inv = 0.0;
        sc = vmin != 0.0 ? fabs(vmin) : 1.0;
        z = vmin > 0.0 ? 1.0 : (vmin < 0.0 ? -1.0 : 0.0);
        r.zsub = qs.half;                       // every code is x_q = 0, i.e. q = -2^(b-1)
    }
    r.scale = (float)(sc / qs.sqrt_h);
    r.izero = (int)(z + qs.half);
    return r;
}

constexpr double kMagic = 6755399441055744.0;   // 1.5 * 2^52: adding it rounds to an integer, ties to even

// One code (low byte of the result).  The product, the magic sum and the later steps round separately
// (this file is compiled with floating-point contraction off).
template <bool ASYM>
__device__ __forceinline__ unsigned code1(double u, const RowQ& p, double half) {
    if constexpr (!ASYM) {
        return (unsigned)__double2loint(u * p.inv + kMagic);
    } else {
        const double r = (u * p.inv + kMagic) - kMagic;
        const double t = fmin(fmax(r - p.zsub, -half), half - 1.0);
        return (unsigned)__double2loint(t + kMagic);
    }
}

// four codes -> one dword of int8
template <bool ASYM>
__device__ __forceinline__ unsigned pack4(const double* v, const RowQ& p, double half) {
    unsigned b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = code1<ASYM>(v[i], p, half);
    const unsigned lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u);
    return (hi << 16) | lo;
}

// Packed 4-bit codes: eight codes q[0..7] in [-7, 7] make one dword; byte j holds q[j] + 8 in its low nibble and
// q[4 + j] + 8 in its high nibble.  lo4 / hi4: the int8 codes q[0..3] / q[4..7], one per byte.
__device__ __forceinline__ unsigned pack_nibbles8(unsigned lo4, unsigned hi4) {
    return ((lo4 ^ 0x08080808u) & 0x0f0f0f0fu) | (((hi4 ^ 0x08080808u) & 0x0f0f0f0fu) << 4);
}

// Four int8 codes in [-7, 7] (one per byte) -> their FP8 E4M3 bit patterns: two 8-entry byte tables (0 .. 7 and the
// negative values by their low three bits) and a pick by the code's bit 3, which is set exactly for the negative ones.
__device__ __forceinline__ unsigned fp8x4_from_codes(unsigned w) {
    const unsigned idx = w & 0x07070707u;
    const unsigned pick = ((w >> 1) & 0x04040404u) | 0x03020100u;
    const unsigned pos = __builtin_amdgcn_perm(0x4e4c4a48u, 0x44403800u, idx);     // 0, 1, 2, 3 | 4, 5, 6, 7
    const unsigned neg = __builtin_amdgcn_perm(0xb8c0c4c8u, 0xcaccce00u, idx);   // -, -7, -6, -5 | -4, -3, -2, -1
    return __builtin_amdgcn_perm(neg, pos, pick);
}

template <bool ASYM>
__device__ __forceinline__ void store8_codes(int8_t* __restrict__ dst, const double v[8], const RowQ& p, double half) {
    *reinterpret_cast<uint2*>(dst) = make_uint2(pack4<ASYM>(v, p, half), pack4<ASYM>(v + 4, p, half));
}

// order-preserving map of a double onto unsigned 64-bit keys (for LDS atomic max on signed values)
__device__ __forceinline__ unsigned long long okey(double x) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double okey_inv(unsigned long long k) {
    const unsigned long long b = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
    return __longlong_as_double((long long)b);
}

__device__ __forceinline__ double block_min(double m, double* red) { return -block_max(-m, red); }

// One workgroup per token row.  The row lives in LDS as doubles; the first three butterfly stages
// run in registers on each 8-element chunk, the remaining ones as radix-8 passes over LDS.
__global__ void hadamard_quant_generic_kernel(const uint16_t* __restrict__ X, int K, int log2h, QuantSpec qs,
                                              int8_t* __restrict__ q, float* __restrict__ scale) {
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
        if (qs.prescale) prescale8(qs.prescale + c * 8, v);
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
    RowQ p;
    if (!qs.asym) {
        double m = 0.0;
        for (int i = t; i < K; i += nt) m = fmax(m, fabs(row[i]));
        p = rowq_sym(block_max(m, red), qs);
    } else {
        double hi = -INFINITY, lo = INFINITY;
        for (int i = t; i < K; i += nt) { hi = fmax(hi, row[i]); lo = fmin(lo, row[i]); }
        hi = block_max(hi, red);
        lo = block_min(lo, red);
        p = rowq_asym(hi, lo, qs);
    }
    for (int c = t; c < nchunks; c += nt) {
        double v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = row[c * 8 + i];
        if (qs.asym) store8_codes<true>(q + base + (size_t)c * 8, v, p, qs.half);
        else store8_codes<false>(q + base + (size_t)c * 8, v, p, qs.half);
    }
    if (t == 0) {
        scale[blockIdx.x] = p.scale;
        if (qs.asym) qs.zero[blockIdx.x] = p.izero;
    }
}

// ---------------------------------------------------------------- register-resident Hadamard, h <= 128
// Every lane owns 32 contiguous elements of a token row (64 bytes in, 32 bytes out): five butterfly
// stages run in registers, and for h = 64 / 128 the last one or two run across the lanes of a quad with
// DPP moves (a Hadamard block is 2 / 4 adjacent lanes).  A workgroup holds R whole rows, so the only
// exchange through LDS is the per-row maximum (one 64-bit LDS atomic per quad).  All arithmetic is
// fp64 and every stage is taken in ascending stride order, like the definition's recursion.
constexpr int E32 = 32;

template <int CTRL>
__device__ __forceinline__ double quad_swap(double v) {
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(v), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(v), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

template <int LOG2H, bool ASYM>
__global__ __launch_bounds__(640) void hadamard_quant_e32_kernel(const uint16_t* __restrict__ X, int M, int K,
                                                                  int rows_per_wg, QuantSpec qs,
                                                                  int8_t* __restrict__ q, float* __restrict__ scale) {
    __shared__ unsigned long long amax_bits[2][32];          // [0]: max |u| (or key of max u), [1]: key of max -u
    const int lpr = K / E32;                       // lanes per row
    const int t = threadIdx.x;
    const int rw = t / lpr, slot = t % lpr;
    const int row = blockIdx.x * rows_per_wg + rw;
    const bool live = rw < rows_per_wg && row < M;
    if (t < 64) amax_bits[t / 32][t % 32] = 0ull;

    double v[E32];
    {
        const int lrow = live ? row : M - 1;
        const uint16_t* src = X + (size_t)lrow * K + (size_t)slot * E32;
#pragma unroll
        for (int c = 0; c < 4; ++c) load8_bf16(src + c * 8, v + c * 8);
        if (qs.prescale) {
#pragma unroll
            for (int c = 0; c < 4; ++c) prescale8(qs.prescale + slot * E32 + c * 8, v + c * 8);
        }
    }
    constexpr int IN_REG = LOG2H < 5 ? LOG2H : 5;
    butterflies<E32>(v, IN_REG);
    if constexpr (LOG2H >= 6) {
        const double sg = (t & 1) ? -1.0 : 1.0;
#pragma unroll
        for (int i = 0; i < E32; ++i) v[i] = fma(v[i], sg, quad_swap<0xB1>(v[i]));
    }
    if constexpr (LOG2H >= 7) {
        const double sg = (t & 2) ? -1.0 : 1.0;
#pragma unroll
        for (int i = 0; i < E32; ++i) v[i] = fma(v[i], sg, quad_swap<0x4E>(v[i]));
    }
    double m = ASYM ? -INFINITY : 0.0, m2 = -INFINITY;
#pragma unroll
    for (int i = 0; i < E32; ++i) {
        if constexpr (ASYM) { m = fmax(m, v[i]); m2 = fmax(m2, -v[i]); }
        else m = fmax(m, fabs(v[i]));
    }
    m = fmax(m, quad_swap<0xB1>(m));
    m = fmax(m, quad_swap<0x4E>(m));
    if constexpr (ASYM) {
        m2 = fmax(m2, quad_swap<0xB1>(m2));
        m2 = fmax(m2, quad_swap<0x4E>(m2));
    }
    __syncthreads();
    if (live && (t & 3) == 0) {
        if constexpr (ASYM) {
            atomicMax(&amax_bits[0][rw], okey(m));
            atomicMax(&amax_bits[1][rw], okey(m2));
        } else {
            atomicMax(&amax_bits[0][rw], (unsigned long long)__double_as_longlong(m));
        }
    }
    __syncthreads();
    if (!live) return;
    RowQ p;
    if constexpr (ASYM) p = rowq_asym(okey_inv(amax_bits[0][rw]), -okey_inv(amax_bits[1][rw]), qs);
    else p = rowq_sym(__longlong_as_double((long long)amax_bits[0][rw]), qs);
    unsigned out[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) out[g] = pack4<ASYM>(v + 4 * g, p, qs.half);
    if (!ASYM && qs.fp8) {
#pragma unroll
        for (int g = 0; g < 8; ++g) out[g] = fp8x4_from_codes(out[g]);
    }
    if (!ASYM && qs.packed) {
        *reinterpret_cast<uint4*>(q + (size_t)row * (K / 2) + (size_t)slot * (E32 / 2)) =
            make_uint4(pack_nibbles8(out[0], out[1]), pack_nibbles8(out[2], out[3]), pack_nibbles8(out[4], out[5]),
                       pack_nibbles8(out[6], out[7]));
    } else {
        uint4* dst = reinterpret_cast<uint4*>(q + (size_t)row * K + (size_t)slot * E32);
        dst[0] = make_uint4(out[0], out[1], out[2], out[3]);
        dst[1] = make_uint4(out[4], out[5], out[6], out[7]);
    }
    if (slot == 0) {
        scale[row] = p.scale;
        if constexpr (ASYM) qs.zero[row] = p.izero;
    }
}

// ---------------------------------------------------------------- two-pass Hadamard, 256 <= h <= 4096
// Pass 1: every lane owns 32 contiguous elements (stages 0..4 in registers).  Pass 2: the G = h / 32 lanes
// of a block exchange the block transposed through LDS - a lane then owns, for its 32 / G (at least one)
// element offsets e, the values of up to 32 pass-1 lanes g - and runs stages 5..9 in registers; for
// h = 2048 / 4096 the last one / two stages run across a lane pair / quad with DPP moves.  The exchange is
// done in two rounds of 16 element offsets each, which halves the LDS footprint (9 bytes per element in
// flight) and so doubles the resident waves.  Codes return through LDS as bytes so that every lane stores
// 32 contiguous bytes.  LDS rows: 16 doubles + 2 of padding per pass-1 lane and 4 more per 32 lanes (the byte
// buffer: 16 bytes per 32 lanes), which keeps the 16-byte writes of pass 1 and the quad-strided accesses of
// pass 2 on distinct banks.  With PERSIST (used for h = 4096) a workgroup walks over row groups and loads the next
// group's bf16 data while it transforms the current one; where LDS has room for it (ONE) the exchange then runs in a single
// round of 32 element offsets (34 doubles per pass-1 lane) with the code bytes in a region of their own, which leaves three
// workgroup barriers per row group instead of six.
// PAD doubles after every 32 pass-1 lanes: the Q lanes of a pass-2 pair / quad read rows 32 apart in one instruction,
// next to 32 / Q element offsets of other lanes, so 32 / Q doubles of padding put all of them on distinct banks.
template <int PAD, int STRIDE = 18>
__device__ __forceinline__ int lds_row(int slot) { return STRIDE * slot + PAD * (slot >> 5); }
constexpr int lds_pad(int log2h) { return log2h == 12 ? 8 : (log2h == 11 ? 16 : 4); }

template <int LOG2H, bool PERSIST, bool ASYM, bool PRE, bool ONE = false>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(PERSIST || PRE ? 2 : 3, PERSIST || PRE ? 2 : 3)))
void hadamard_quant_2pass_kernel(const uint16_t* __restrict__ X, int M, int K,
                                                                   int rows_per_wg, QuantSpec qs,
                                                                   int8_t* __restrict__ q, float* __restrict__ scale) {
    constexpr int G = 1 << (LOG2H - 5);            // pass-1 lanes per block
    constexpr int NG = G < 32 ? G : 32;            // values per element offset held by a pass-2 lane
    constexpr int EPL = 32 / NG;                   // element offsets per pass-2 lane (4, 2, 1)
    constexpr int Q = G / NG;                      // lanes that share an element offset (1, 2, 4)
    extern __shared__ __attribute__((aligned(16))) double lds[];
    __shared__ unsigned long long amax_bits[2][2][32];       // [parity][max |u| or key of max u / key of max -u][row]
    const int lpr = K / E32;
    static_assert(!ONE || PERSIST, "the single-round exchange is a form of the persistent kernel");
    constexpr int PAD = lds_pad(LOG2H);
    constexpr int NR = ONE ? 1 : 2;                // exchange rounds
    constexpr int EPR = 32 / NR;                   // element offsets per round
    constexpr int STRIDE = EPR + 2;                // doubles per pass-1 lane in LDS
    const int rs = lds_row<PAD, STRIDE>(lpr) + 8;  // doubles per row buffer
    const int t = threadIdx.x;
    const int rw = t / lpr, slot = t % lpr;
    const bool inwg = rw < rows_per_wg;
    double* rowbuf = lds + (size_t)(inwg ? rw : 0) * rs;
    // pass 2 role of this thread: lane j of block b, element offsets e0 .. e0 + EPL - 1, quad position gq
    const int b = slot / G, j = slot % G;
    const int e0 = (j / Q) * EPL, gq = j % Q;
    const int my_round = ONE ? 0 : e0 >> 4;
    const int ngroups = (M + rows_per_wg - 1) / rows_per_wg;
    if (t < 128) amax_bits[t / 64][(t / 32) % 2][t % 32] = 0ull;

    uint4 raw[4];
    {
        int r0 = blockIdx.x * rows_per_wg + rw;
        if (!inwg || r0 >= M) r0 = M - 1;
        const uint4* src = reinterpret_cast<const uint4*>(X + (size_t)r0 * K + (size_t)slot * E32);
#pragma unroll
        for (int c = 0; c < 4; ++c) raw[c] = src[c];
    }
    int par = 0;
    for (int grp = blockIdx.x; grp < ngroups; grp += gridDim.x, par ^= 1) {
        const int row = grp * rows_per_wg + rw;
        const bool live = inwg && row < M;
        double v[E32], w[E32];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned wd[4] = {raw[c].x, raw[c].y, raw[c].z, raw[c].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[c * 8 + 2 * i] = (double)__uint_as_float(wd[i] << 16);
                v[c * 8 + 2 * i + 1] = (double)__uint_as_float(wd[i] & 0xffff0000u);
            }
        }
        if constexpr (PRE) {     // a template flag: as a run-time branch it costs the other variants 80 registers
#pragma unroll
            for (int c = 0; c < 4; ++c) prescale8(qs.prescale + slot * E32 + c * 8, v + c * 8);
        }
        butterflies<E32>(v, 5);
#pragma unroll
        for (int round = 0; round < NR; ++round) {
            // earlier readers of the buffer (first half / previous group) are done; the single-round form needs no such
            // barrier: the previous group's last reads of this buffer precede its barrier after the maxima, and its codes
            // went through a buffer of their own
            if (!ONE && (PERSIST || round == 1)) __syncthreads();
            if (inwg) {
                double2* dst = reinterpret_cast<double2*>(rowbuf + lds_row<PAD, STRIDE>(slot));
#pragma unroll
                for (int i = 0; i < EPR / 2; ++i) dst[i] = make_double2(v[EPR * round + 2 * i], v[EPR * round + 2 * i + 1]);
            }
            if (PERSIST && round == 0 && t < 64) amax_bits[par ^ 1][t / 32][t % 32] = 0ull;   // the other parity's slots, for the next group
            __syncthreads();
            if (my_round == round) {
#pragma unroll
                for (int r = 0; r < NG; ++r) {
                    const double* p = rowbuf + lds_row<PAD, STRIDE>(b * G + r + 32 * gq) + (e0 - EPR * round);
                    if constexpr (EPL == 4) {
                        const double2 a = *reinterpret_cast<const double2*>(p), c = *reinterpret_cast<const double2*>(p + 2);
                        w[r * 4 + 0] = a.x; w[r * 4 + 1] = a.y; w[r * 4 + 2] = c.x; w[r * 4 + 3] = c.y;
                    } else if constexpr (EPL == 2) {
                        const double2 a = *reinterpret_cast<const double2*>(p);
                        w[r * 2 + 0] = a.x; w[r * 2 + 1] = a.y;
                    } else {
                        w[r] = *p;
                    }
                }
            }
        }
        if constexpr (PERSIST) {   // next group's data: in flight while pass 2 runs (pass-1 registers are dead by now)
            int rn = (grp + gridDim.x) * rows_per_wg + rw;
            if (!inwg || rn >= M) rn = M - 1;
            const uint4* src = reinterpret_cast<const uint4*>(X + (size_t)rn * K + (size_t)slot * E32);
#pragma unroll
            for (int c = 0; c < 4; ++c) raw[c] = src[c];
        }
        butterflies<E32, EPL>(w, LOG2H - 5 < 5 ? LOG2H - 5 : 5);
        if constexpr (Q >= 2) {
            const double sg = (t & 1) ? -1.0 : 1.0;
#pragma unroll
            for (int i = 0; i < E32; ++i) w[i] = fma(w[i], sg, quad_swap<0xB1>(w[i]));
        }
        if constexpr (Q >= 4) {
            const double sg = (t & 2) ? -1.0 : 1.0;
#pragma unroll
            for (int i = 0; i < E32; ++i) w[i] = fma(w[i], sg, quad_swap<0x4E>(w[i]));
        }
        double m = ASYM ? -INFINITY : 0.0, m2 = -INFINITY;
#pragma unroll
        for (int i = 0; i < E32; ++i) {
            if constexpr (ASYM) { m = fmax(m, w[i]); m2 = fmax(m2, -w[i]); }
            else m = fmax(m, fabs(w[i]));
        }
        m = fmax(m, quad_swap<0xB1>(m));
        m = fmax(m, quad_swap<0x4E>(m));
        if constexpr (ASYM) {
            m2 = fmax(m2, quad_swap<0xB1>(m2));
            m2 = fmax(m2, quad_swap<0x4E>(m2));
        }
        if (live && (t & 3) == 0) {
            if constexpr (ASYM) {
                atomicMax(&amax_bits[par][0][rw], okey(m));
                atomicMax(&amax_bits[par][1][rw], okey(m2));
            } else {
                atomicMax(&amax_bits[par][0][rw], (unsigned long long)__double_as_longlong(m));
            }
        }
        __syncthreads();          // every pass-2 read is done: the buffer can be reused for the codes

        RowQ p;
        {
            const int rr = inwg ? rw : 0;
            if constexpr (ASYM) {
                // rows beyond M leave the keys at 0; feed finite values then (their codes are never stored)
                const unsigned long long k0 = amax_bits[par][0][rr], k1 = amax_bits[par][1][rr];
                p = rowq_asym(k0 ? okey_inv(k0) : 0.0, k1 ? -okey_inv(k1) : 0.0, qs);
            } else {
                p = rowq_sym(__longlong_as_double((long long)amax_bits[par][0][rr]), qs);
            }
        }
        // byte buffer: 32 bytes per pass-1 lane, 16 bytes of padding per 32 lanes
        // (single-round form: a region of its own behind the row buffers, so that the next group's pass 1 may overwrite the
        // row buffer while slower waves still collect this group's codes)
        unsigned char* cbuf = (ONE ? reinterpret_cast<unsigned char*>(lds + (size_t)rows_per_wg * rs) +
                                         (size_t)(inwg ? rw : 0) * (lpr * 32 + (lpr >> 5) * 16)
                                   : reinterpret_cast<unsigned char*>(rowbuf)) + (size_t)b * (G * 32 + (G >> 5) * 16);
        if (inwg) {
#pragma unroll
            for (int r = 0; r < NG; ++r) {
                unsigned char* dstb = cbuf + (r + 32 * gq) * 32 + gq * 16 + e0;
                if constexpr (EPL == 4) {
                    *reinterpret_cast<unsigned*>(dstb) = pack4<ASYM>(w + 4 * r, p, qs.half);
                } else if constexpr (EPL == 2) {
                    const unsigned c0 = code1<ASYM>(w[2 * r], p, qs.half), c1 = code1<ASYM>(w[2 * r + 1], p, qs.half);
                    *reinterpret_cast<unsigned short*>(dstb) = (unsigned short)((c0 & 0xffu) | (c1 << 8));
                } else {
                    *dstb = (unsigned char)code1<ASYM>(w[r], p, qs.half);
                }
            }
        }
        __syncthreads();
        if (live) {
            const uint4* src = reinterpret_cast<const uint4*>(cbuf + j * 32 + (j >> 5) * 16);
            if (!ASYM && qs.packed) {
                const uint4 a = src[0], c = src[1];
                *reinterpret_cast<uint4*>(q + (size_t)row * (K / 2) + (size_t)slot * (E32 / 2)) =
                    make_uint4(pack_nibbles8(a.x, a.y), pack_nibbles8(a.z, a.w), pack_nibbles8(c.x, c.y), pack_nibbles8(c.z, c.w));
            } else if (!ASYM && qs.fp8) {
                const uint4 a = src[0], c = src[1];
                uint4* dst = reinterpret_cast<uint4*>(q + (size_t)row * K + (size_t)slot * E32);
                dst[0] = make_uint4(fp8x4_from_codes(a.x), fp8x4_from_codes(a.y), fp8x4_from_codes(a.z), fp8x4_from_codes(a.w));
                dst[1] = make_uint4(fp8x4_from_codes(c.x), fp8x4_from_codes(c.y), fp8x4_from_codes(c.z), fp8x4_from_codes(c.w));
            } else {
                uint4* dst = reinterpret_cast<uint4*>(q + (size_t)row * K + (size_t)slot * E32);
                dst[0] = src[0];
                dst[1] = src[1];
            }
            if (slot == 0) {
                scale[row] = p.scale;
                if constexpr (ASYM) qs.zero[row] = p.izero;
            }
        }
    }
}

// ---------------------------------------------------------------- dense rotation, fp64, k ascending
constexpr int DT = 64;   // output tile (rows x cols) of one workgroup
constexpr int DK = 16;   // K step

__global__ __launch_bounds__(256) void dense_rotate_f64_kernel(const uint16_t* __restrict__ X,
                                                                const uint16_t* __restrict__ R, int M, int K,
                                                                double* __restrict__ U, const float* __restrict__ ps) {
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
        if (ps) {
#pragma unroll
            for (int i = 0; i < 4; ++i) Xs[xk + i][xr] *= (double)ps[k0 + xk + i];
        }
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

// Dense rotation of a few token rows (conditioning vectors): a 128-row matrix-core tile would be almost empty and the
// launch a handful of workgroups walking all of K, so here every thread owns one output column of one row and runs the
// same ascending-k chain of fused multiply-adds itself (x row in LDS as doubles, read as broadcasts; R read 128
// contiguous bytes per wave and k).
constexpr int kFewRows = 64;
__global__ __launch_bounds__(128) void dense_rotate_fewrows_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ R,
                                                                   int K, double* __restrict__ U, const float* __restrict__ ps) {
    extern __shared__ double xrow[];
    const int t = threadIdx.x, row = blockIdx.y, col = blockIdx.x * 128 + t;
    for (int k = t; k < K; k += 128) {
        double v = (double)__uint_as_float((unsigned)X[(size_t)row * K + k] << 16);
        if (ps) v *= (double)ps[k];
        xrow[k] = v;
    }
    __syncthreads();
    if (col >= K) return;
    const uint16_t* r = R + col;
    double u = 0.0;
    // 32 loads in flight per batch: the chain itself is short (one FMA per k), the loads' latency is what has to be hidden
    int k = 0;
    for (; k + 32 <= K; k += 32) {
        unsigned short rv[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) rv[i] = r[(size_t)(k + i) * K];
#pragma unroll
        for (int i = 0; i < 32; ++i) u = fma(xrow[k + i], (double)__uint_as_float((unsigned)rv[i] << 16), u);
    }
    for (; k < K; ++k) u = fma(xrow[k], (double)__uint_as_float((unsigned)r[(size_t)k * K] << 16), u);
    U[(size_t)row * K + col] = u;
}

// Block-diagonal product on the fp64 matrix cores: dst[:, block g] = src[:, block g] . R_g with src bf16 [M, K] and
// R [K/B, B, B] bf16 (B = K is the dense rotation, one block).  v_mfma_f64_16x16x4_f64 accumulates its four k in
// ascending order, one fused multiply-add each, so chaining the instructions over ascending k gives the same bits as
// the scalar chain above, and - every product of two bf16 values (times an fp32 pre-scale) being exact in fp64 - the
// same bits as a sum with separately rounded multiply and add (a GPU test compares U with the definition bit for bit).
// Workgroup = 4 waves (2 x 2), tile 128 x 128, wave tile 64 x 64 (16 accumulator tiles); B must be a multiple of
// 128 so that a column tile lies inside one block.
// The operand tiles stay in LDS as bf16 and are widened to fp64 when a fragment is read: a K step holds 64 k per
// barrier, the global -> LDS path is a plain 16-byte copy, and LDS traffic is a quarter of what fp64 tiles would cost.
// Row strides: 144 bytes for the left tile (36 dwords: the 16 rows a fragment read touches land on 16 distinct banks,
// the four k of a read on consecutive ones) and 288 bytes for the R tile (its four k rows 8 banks apart).
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int MT_ = 128;

// MR: rows of the workgroup tile, 128 or 64 (wave tile MR / 2 x 64); the tile rows start at row_begin + blockIdx.y * MR.
template <int MR = MT_>
__global__ __launch_bounds__(256, 2) void blockdiag_rotate_mfma_f64_kernel(const uint16_t* __restrict__ src,
                                                                                 const uint16_t* __restrict__ R, int M, int K,
                                                                                 int B, double* __restrict__ dst,
                                                                                 const float* __restrict__ ps, int row_begin) {
    constexpr int KS = 64;                          // k per step
    constexpr int XS = 144, RS = 288;               // row strides in bytes
    constexpr int XT = MR * XS, RT = KS * RS;       // tile bytes
    static_assert(MR == 128 || MR == 64, "tile loads are written out for 128 or 64 rows");
    constexpr int XL = MR / 32;                     // 16-byte chunks of the left tile per thread (MR rows x 128 bytes)
    constexpr int RI = MR / 32;                     // 16-row accumulator tiles per wave
    constexpr int RL = KS * 16 / 256;               // 16-byte chunks of the R tile per thread (KS rows x 256 bytes)
    __shared__ __attribute__((aligned(16))) unsigned char Xs[2][XT];
    __shared__ __attribute__((aligned(16))) unsigned char Rs[2][RT];
    __shared__ float Ps[2][KS];
    const int t = threadIdx.x, lane = t % 64, wv = t / 64;
    const int wm = wv / 2, wn = wv % 2;
    const int row0 = row_begin + blockIdx.y * MR, col0 = blockIdx.x * MT_;
    const int g = col0 / B, kbase = g * B, cb = col0 - kbase;
    v4d acc[RI][4];
#pragma unroll
    for (int i = 0; i < RI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4d{0.0, 0.0, 0.0, 0.0};
    constexpr int XE = 2;                           // bytes per left element
    constexpr int XCH = 128 / 16;                   // chunks per left-tile row (128 bytes of data)
    const unsigned char* xsrc[XL];
    int xdst[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int c = t + 256 * i, row = c / XCH, cc = c % XCH;
        int grow = row0 + row;
        if (grow >= M) grow = M - 1;
        xsrc[i] = reinterpret_cast<const unsigned char*>(src) + ((size_t)grow * K + kbase) * XE + cc * 16;
        xdst[i] = row * XS + cc * 16;
    }
    const unsigned char* rsrc[RL];
    int rdst[RL];
#pragma unroll
    for (int i = 0; i < RL; ++i) {
        const int c = t + 256 * i, row = c / 16, cc = c % 16;
        rsrc[i] = reinterpret_cast<const unsigned char*>(R + (size_t)g * B * B + (size_t)row * B + cb) + cc * 16;
        rdst[i] = row * RS + cc * 16;
    }
    const int nk = B / KS;
    {
#pragma unroll
        for (int i = 0; i < XL; ++i) *reinterpret_cast<uint4*>(&Xs[0][xdst[i]]) = *reinterpret_cast<const uint4*>(xsrc[i]);
#pragma unroll
        for (int i = 0; i < RL; ++i) *reinterpret_cast<uint4*>(&Rs[0][rdst[i]]) = *reinterpret_cast<const uint4*>(rsrc[i]);
        if (t < KS) Ps[0][t] = ps ? ps[kbase + t] : 1.0f;
    }
    __syncthreads();
    for (int kb = 0; kb < nk; ++kb) {
        const int cur = kb & 1;
        // next tile in flight during this step's MFMAs (the last step re-reads its own tile into the idle buffer:
        // branch-free, and nothing reads that buffer afterwards)
        const int kn = kb + 1 < nk ? kb + 1 : kb;
        uint4 xn0 = *reinterpret_cast<const uint4*>(xsrc[0] + (size_t)kn * KS * XE);
        uint4 xn1 = *reinterpret_cast<const uint4*>(xsrc[1] + (size_t)kn * KS * XE);
        uint4 xn2 = xn0, xn3 = xn0;
        if constexpr (XL == 4) {
            xn2 = *reinterpret_cast<const uint4*>(xsrc[2] + (size_t)kn * KS * XE);
            xn3 = *reinterpret_cast<const uint4*>(xsrc[3] + (size_t)kn * KS * XE);
        }
        uint4 rn0 = *reinterpret_cast<const uint4*>(rsrc[0] + (size_t)kn * KS * B * 2);
        uint4 rn1 = *reinterpret_cast<const uint4*>(rsrc[1] + (size_t)kn * KS * B * 2);
        uint4 rn2 = rn0, rn3 = rn0;
        if constexpr (RL == 4) {
            rn2 = *reinterpret_cast<const uint4*>(rsrc[2] + (size_t)kn * KS * B * 2);
            rn3 = *reinterpret_cast<const uint4*>(rsrc[3] + (size_t)kn * KS * B * 2);
        }
        float pn = 1.0f;
        if (ps && t < KS) pn = ps[kbase + kn * KS + t];
        const unsigned char* xa = &Xs[cur][(wm * (MR / 2) + lane % 16) * XS + (lane / 16) * XE];
        const unsigned char* rb = &Rs[cur][(lane / 16) * RS + (wn * 64 + lane % 16) * 2];
#pragma unroll 2
        for (int ks = 0; ks < KS / 4; ++ks) {
            double a[RI], b[4];
#pragma unroll
            for (int i = 0; i < RI; ++i) {
                a[i] = (double)__uint_as_float((unsigned)*reinterpret_cast<const uint16_t*>(xa + i * 16 * XS + ks * 4 * XE) << 16);
            }
            if (ps) {
                const double pv = (double)Ps[cur][ks * 4 + lane / 16];
#pragma unroll
                for (int i = 0; i < RI; ++i) a[i] *= pv;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[j] = (double)__uint_as_float((unsigned)*reinterpret_cast<const uint16_t*>(rb + ks * 4 * RS + j * 32) << 16);
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        // the other buffer's last readers passed the barrier that closed the previous step
        {
            unsigned char* xw = Xs[cur ^ 1];
            unsigned char* rw = Rs[cur ^ 1];
            *reinterpret_cast<uint4*>(xw + xdst[0]) = xn0;
            *reinterpret_cast<uint4*>(xw + xdst[1]) = xn1;
            if constexpr (XL == 4) {
                *reinterpret_cast<uint4*>(xw + xdst[2]) = xn2;
                *reinterpret_cast<uint4*>(xw + xdst[3]) = xn3;
            }
            *reinterpret_cast<uint4*>(rw + rdst[0]) = rn0;
            *reinterpret_cast<uint4*>(rw + rdst[1]) = rn1;
            if constexpr (RL == 4) {
                *reinterpret_cast<uint4*>(rw + rdst[2]) = rn2;
                *reinterpret_cast<uint4*>(rw + rdst[3]) = rn3;
            }
            if (t < KS) Ps[cur ^ 1][t] = pn;
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < RI; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + wm * (MR / 2) + i * 16 + 4 * r + lane / 16;
            if (row < M) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const size_t o = (size_t)row * K + col0 + wn * 64 + j * 16 + lane % 16;
                    dst[o] = acc[i][j][r];
                }
            }
        }
}

// out[row, j] = in[row, perm[j]] for fp64 rows: the row is staged in LDS so that global reads and writes are both
// contiguous.  Indices are clamped into [0, K) (a malformed perm gives wrong values, never an out-of-range access).
__global__ __launch_bounds__(256) void permute_rows_f64_kernel(const double* __restrict__ in, const int32_t* __restrict__ perm,
                                                                int M, int K, double* __restrict__ out) {
    extern __shared__ __attribute__((aligned(16))) double prow[];
    const int t = threadIdx.x;
    for (int row = blockIdx.x; row < M; row += gridDim.x) {
        const double2* src = reinterpret_cast<const double2*>(in + (size_t)row * K);
        for (int c = t; c < K / 2; c += 256) reinterpret_cast<double2*>(prow)[c] = src[c];
        __syncthreads();
        double2* dst = reinterpret_cast<double2*>(out + (size_t)row * K);
        for (int c = t; c < K / 2; c += 256) {
            const int2 pi = reinterpret_cast<const int2*>(perm)[c];
            const int i0 = min(max(pi.x, 0), K - 1), i1 = min(max(pi.y, 0), K - 1);
            dst[c] = make_double2(prow[i0], prow[i1]);
        }
        __syncthreads();
    }
}

// Second stage of the structured rotation: dst[:, block g] = src[:, block g] . R_g for fp64 src and bf16 R
// [K/B, B, B].  A product of an fp64 value and a bf16 value is not exact in fp64, so here multiply and add round
// separately, term by term in ascending k - the plain sum the definition states - and the fused multiply-adds of the
// matrix cores cannot be used.  64 x 64 output tile per workgroup, 4 x 4 outputs per thread, 16 k per LDS stage.
__global__ __launch_bounds__(256) void blockdiag_rotate_seq_f64_kernel(const double* __restrict__ src,
                                                                        const uint16_t* __restrict__ R, int M, int K, int B,
                                                                        double* __restrict__ dst) {
    __shared__ double Xs[DK][DT + 1];
    __shared__ double Rs[DK][DT];
    const int t = threadIdx.x;
    const int row0 = blockIdx.y * DT, col0 = blockIdx.x * DT;
    const int g = col0 / B, kbase = g * B, cb = col0 - kbase;
    const int ty = t / 16, tx = t % 16;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    const int xr = t / 4, xk = (t % 4) * 4;      // src tile: 64 rows x 16 k, 4 doubles per thread
    const int rk = t / 16, rc = (t % 16) * 4;    // R tile: 16 k x 64 cols, 4 bf16 per thread
    int xrow = row0 + xr;
    if (xrow >= M) xrow = M - 1;
    const uint16_t* Rg = R + (size_t)g * B * B;
    for (int k0 = 0; k0 < B; k0 += DK) {
        const double2 x0 = *reinterpret_cast<const double2*>(src + (size_t)xrow * K + kbase + k0 + xk);
        const double2 x1 = *reinterpret_cast<const double2*>(src + (size_t)xrow * K + kbase + k0 + xk + 2);
        const uint2 ra = *reinterpret_cast<const uint2*>(Rg + (size_t)(k0 + rk) * B + cb + rc);
        Xs[xk + 0][xr] = x0.x;
        Xs[xk + 1][xr] = x0.y;
        Xs[xk + 2][xr] = x1.x;
        Xs[xk + 3][xr] = x1.y;
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
                for (int j = 0; j < 4; ++j) acc[i][j] = __dadd_rn(acc[i][j], __dmul_rn(a[i], b[j]));
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = row0 + ty * 4 + i;
        if (r < M) {
            double* o = dst + (size_t)r * K + col0 + tx * 4;
            *reinterpret_cast<double2*>(o) = make_double2(acc[i][0], acc[i][1]);
            *reinterpret_cast<double2*>(o + 2) = make_double2(acc[i][2], acc[i][3]);
        }
    }
}

// One workgroup per row: absmax and codes from fp64 U.
__global__ void quant_from_f64_kernel(const double* __restrict__ U, int K, QuantSpec qs,
                                      int8_t* __restrict__ q, float* __restrict__ scale) {
    __shared__ double red[16];
    const int t = threadIdx.x, nt = blockDim.x;
    const size_t base = (size_t)blockIdx.x * K;
    RowQ p;
    if (!qs.asym) {
        double m = 0.0;
        for (int i = t; i < K; i += nt) m = fmax(m, fabs(U[base + i]));
        p = rowq_sym(block_max(m, red), qs);
    } else {
        double hi = -INFINITY, lo = INFINITY;
        for (int i = t; i < K; i += nt) { hi = fmax(hi, U[base + i]); lo = fmin(lo, U[base + i]); }
        hi = block_max(hi, red);
        lo = block_min(lo, red);
        p = rowq_asym(hi, lo, qs);
    }
    for (int c = t; c < (K >> 3); c += nt) {
        double v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = U[base + (size_t)c * 8 + i];
        if (qs.asym) store8_codes<true>(q + base + (size_t)c * 8, v, p, qs.half);
        else store8_codes<false>(q + base + (size_t)c * 8, v, p, qs.half);
    }
    if (t == 0) {
        scale[blockIdx.x] = p.scale;
        if (qs.asym) qs.zero[blockIdx.x] = p.izero;
    }
}

// The same for K <= 8192: one 8-element chunk per thread, held in registers between the reduction and the rounding, so
// that U is read once, 16 bytes at a time.
__global__ void quant_from_f64_once_kernel(const double* __restrict__ U, int K, QuantSpec qs, int8_t* __restrict__ q,
                                           float* __restrict__ scale) {
    __shared__ double red[16];
    const int t = threadIdx.x;
    const size_t base = (size_t)blockIdx.x * K;
    const bool have = t < (K >> 3);
    double v[8];
    if (have) {
        const double2* src = reinterpret_cast<const double2*>(U + base + (size_t)t * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double2 d = src[i];
            v[2 * i] = d.x;
            v[2 * i + 1] = d.y;
        }
    }
    RowQ p;
    if (!qs.asym) {
        double m = 0.0;
        if (have) {
#pragma unroll
            for (int i = 0; i < 8; ++i) m = fmax(m, fabs(v[i]));
        }
        p = rowq_sym(block_max(m, red), qs);
    } else {
        double hi = -INFINITY, lo = INFINITY;
        if (have) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { hi = fmax(hi, v[i]); lo = fmin(lo, v[i]); }
        }
        hi = block_max(hi, red);
        lo = block_min(lo, red);
        p = rowq_asym(hi, lo, qs);
    }
    if (have) {
        if (qs.asym) store8_codes<true>(q + base + (size_t)t * 8, v, p, qs.half);
        else store8_codes<false>(q + base + (size_t)t * 8, v, p, qs.half);
    }
    if (t == 0) {
        scale[blockIdx.x] = p.scale;
        if (qs.asym) qs.zero[blockIdx.x] = p.izero;
    }
}

// int8 codes [M, K] -> packed nibbles [M, K / 2], 16 codes per thread (K % 16 == 0)
__global__ __launch_bounds__(256) void pack_nibbles_kernel(const int8_t* __restrict__ q, size_t n16, uint8_t* __restrict__ q4) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 v = reinterpret_cast<const uint4*>(q)[i];
    reinterpret_cast<uint2*>(q4)[i] = make_uint2(pack_nibbles8(v.x, v.y), pack_nibbles8(v.z, v.w));
}

// int8 codes in [-7, 7] -> FP8 E4M3 bit patterns in place, 16 codes per thread
__global__ __launch_bounds__(256) void codes_to_fp8_kernel(int8_t* __restrict__ q, size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 v = reinterpret_cast<const uint4*>(q)[i];
    reinterpret_cast<uint4*>(q)[i] = make_uint4(fp8x4_from_codes(v.x), fp8x4_from_codes(v.y), fp8x4_from_codes(v.z), fp8x4_from_codes(v.w));
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

static void launch_quant_from_f64(hipStream_t st, const double* U, int M, int K, const QuantSpec& qs, int8_t* q, float* scale);

static bool e32_shape(int K, int h) { return h <= 128 && K % 128 == 0 && K / E32 <= 576; }
static bool twopass_shape(int K, int h) { return h >= 256 && h <= 4096 && K % 128 == 0 && K / E32 <= 512; }
bool hadamard_packs_in_kernel(int K, int h) { return e32_shape(K, h) || twopass_shape(K, h); }

hipError_t launch_codes_to_fp8(hipStream_t st, int8_t* q, size_t n) {
    const size_t n16 = n / 16;
    hipLaunchKernelGGL(codes_to_fp8_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, q, n16);
    return hipGetLastError();
}

hipError_t launch_pack_nibbles(hipStream_t st, const int8_t* q, int M, int K, uint8_t* q4) {
    const size_t n16 = (size_t)M * K / 16;
    hipLaunchKernelGGL(pack_nibbles_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, q, n16, q4);
    return hipGetLastError();
}

static QuantSpec make_spec(int act_bits, int h, int32_t* zero, const float* prescale = nullptr) {
    QuantSpec qs;
    qs.asym = zero != nullptr;
    qs.qmax = (double)((1 << (act_bits - 1)) - 1);
    qs.sqrt_h = sqrt((double)h);
    qs.norm = qs.qmax * qs.sqrt_h;
    qs.L = (double)((1 << act_bits) - 1);
    qs.half = (double)(1 << (act_bits - 1));
    qs.zero = zero;
    qs.prescale = prescale;
    qs.packed = 0;
    qs.fp8 = 0;
    return qs;
}

static void launch_quant_from_f64(hipStream_t st, const double* U, int M, int K, const QuantSpec& qs, int8_t* q, float* scale) {
    if (K <= 8192) hipLaunchKernelGGL(quant_from_f64_once_kernel, dim3(M), dim3(threads_for_row(K)), 0, st, U, K, qs, q, scale);
    else hipLaunchKernelGGL(quant_from_f64_kernel, dim3(M), dim3(256), 0, st, U, K, qs, q, scale);
}

hipError_t launch_hadamard_quant(hipStream_t st, const uint16_t* X, int M, int K, int h, int act_bits,
                                 int8_t* q, float* scale, int32_t* zero, const float* prescale, bool packed, bool fp8) {
    QuantSpec qs = make_spec(act_bits, h, zero, prescale);
    if (packed || fp8) {
        if ((packed && fp8) || zero || act_bits != 4 || !hadamard_packs_in_kernel(K, h)) return hipErrorInvalidValue;
        qs.packed = packed;
        qs.fp8 = fp8;
    }
    if (e32_shape(K, h)) {
        // R whole rows per workgroup, at most four waves (finer granularity measured faster than nine; 7 rows of 1152 fill four waves)
        const int lpr = K / E32;
        int R = 256 / lpr;
        if (R < 1) R = 1;
        if (R > 32) R = 32;
        const int nt = ((lpr * R + kWave - 1) / kWave) * kWave;
        const dim3 grid((M + R - 1) / R), block(nt);
#define LRQ_CASE(L)                                                                                              \
    case L:                                                                                                      \
        if (qs.asym) hipLaunchKernelGGL((hadamard_quant_e32_kernel<L, true>), grid, block, 0, st, X, M, K, R, qs, q, scale); \
        else hipLaunchKernelGGL((hadamard_quant_e32_kernel<L, false>), grid, block, 0, st, X, M, K, R, qs, q, scale);        \
        break;
        switch (ilog2(h)) { LRQ_CASE(0) LRQ_CASE(1) LRQ_CASE(2) LRQ_CASE(3) LRQ_CASE(4) LRQ_CASE(5) LRQ_CASE(6) LRQ_CASE(7) }
#undef LRQ_CASE
        return hipGetLastError();
    }
    if (twopass_shape(K, h)) {
        const int lpr = K / E32;
        int R = 256 / lpr;                       // about four waves per workgroup; whole rows only
        if (R < 1) R = 1;
        if (R > 32) R = 32;
        const int nt = ((lpr * R + kWave - 1) / kWave) * kWave;
        const int pad = lds_pad(ilog2(h));
        const size_t ldsb_two = (size_t)R * (18 * lpr + pad * (lpr >> 5) + 8) * sizeof(double);
        // single-round form of the persistent kernel: 34 doubles per pass-1 lane, code bytes behind the row buffers
        const size_t ldsb_one = (size_t)R * ((34 * lpr + pad * (lpr >> 5) + 8) * sizeof(double) + lpr * 32 + (lpr >> 5) * 16);
        bool one = h >= 4096 && ldsb_one <= 150 * 1024;
        size_t ldsb = one ? ldsb_one : ldsb_two;
        // resident workgroups per CU: two waves per SIMD by registers, LDS permitting
        const int groups = (M + R - 1) / R;
        int per_cu = (int)((160 * 1024 - 2048) / (ldsb + 512));
        const int by_waves = 8 / (nt / kWave) > 0 ? 8 / (nt / kWave) : 1;
        if (per_cu > by_waves) per_cu = by_waves;
        if (per_cu < 1) per_cu = 1;
        // the largest block runs as persistent workgroups that load the next row group while transforming the current
        // one (measured: 566 vs 690 us at 35100 x 12288; at h = 2048 the plain form is the faster one, 208 vs 288 us)
        const bool persist = h >= 4096 && groups > 256 * per_cu;
        if (!persist) {
            one = false;
            ldsb = ldsb_two;
        }
        const dim3 grid(persist ? 256 * per_cu : groups), block(nt);
#define LRQ_ATTR(L, P, A, S, O) { hipError_t e = allow_large_lds(reinterpret_cast<const void*>(hadamard_quant_2pass_kernel<L, P, A, S, O>), 158 * 1024); if (e != hipSuccess) return e; }
#define LRQ_ATTR2(L, P, O) { if (qs.asym && qs.prescale) LRQ_ATTR(L, P, true, true, O) else if (qs.asym) LRQ_ATTR(L, P, true, false, O) else if (qs.prescale) LRQ_ATTR(L, P, false, true, O) else LRQ_ATTR(L, P, false, false, O) }
        switch (ilog2(h)) {
            case 8: LRQ_ATTR2(8, false, false) break;
            case 9: LRQ_ATTR2(9, false, false) break;
            case 10: LRQ_ATTR2(10, false, false) break;
            case 11: LRQ_ATTR2(11, false, false) break;
            case 12: if (one) LRQ_ATTR2(12, true, true) else if (persist) LRQ_ATTR2(12, true, false) else LRQ_ATTR2(12, false, false) break;
        }
#undef LRQ_ATTR2
#undef LRQ_ATTR
#define LRQ_GO(L, P, O)                                                                                                   \
    {                                                                                                                     \
        if (qs.asym && qs.prescale) hipLaunchKernelGGL((hadamard_quant_2pass_kernel<L, P, true, true, O>), grid, block, ldsb, st, X, M, K, R, qs, q, scale);   \
        else if (qs.asym) hipLaunchKernelGGL((hadamard_quant_2pass_kernel<L, P, true, false, O>), grid, block, ldsb, st, X, M, K, R, qs, q, scale);       \
        else if (qs.prescale) hipLaunchKernelGGL((hadamard_quant_2pass_kernel<L, P, false, true, O>), grid, block, ldsb, st, X, M, K, R, qs, q, scale);   \
        else hipLaunchKernelGGL((hadamard_quant_2pass_kernel<L, P, false, false, O>), grid, block, ldsb, st, X, M, K, R, qs, q, scale);                   \
    }
        switch (ilog2(h)) {
            case 8: LRQ_GO(8, false, false) break;
            case 9: LRQ_GO(9, false, false) break;
            case 10: LRQ_GO(10, false, false) break;
            case 11: LRQ_GO(11, false, false) break;
            case 12: if (one) LRQ_GO(12, true, true) else if (persist) LRQ_GO(12, true, false) else LRQ_GO(12, false, false) break;
        }
#undef LRQ_GO
        return hipGetLastError();
    }
    const int nt = threads_for_row(K);
    const size_t lds = (size_t)(K + 16) * sizeof(double);
    {
        const hipError_t e = allow_large_lds(reinterpret_cast<const void*>(hadamard_quant_generic_kernel), 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(hadamard_quant_generic_kernel, dim3(M), dim3(nt), lds, st, X, K, ilog2(h), qs, q, scale);
    return hipGetLastError();
}

hipError_t launch_plain_quant(hipStream_t st, const uint16_t* X, int M, int K, int act_bits, int8_t* q,
                              float* scale, int32_t* zero, const float* prescale) {
    return launch_hadamard_quant(st, X, M, K, 1, act_bits, q, scale, zero, prescale);
}

hipError_t launch_dense_rotate_quant(hipStream_t st, const uint16_t* X, const uint16_t* R, int M, int K,
                                     int act_bits, double* U, int8_t* q, float* scale, int32_t* zero,
                                     const float* prescale) {
    if (M <= kFewRows && (size_t)K * sizeof(double) <= 48 * 1024) {
        hipLaunchKernelGGL(dense_rotate_fewrows_kernel, dim3((K + 127) / 128, M), dim3(128), (size_t)K * sizeof(double), st, X, R,
                           K, U, prescale);
    } else if (K % MT_ == 0) {
        // 512 workgroups are resident at a time (two per CU).  When the tiles make a few rounds and the last one would be
        // less than half full, the rows of that last round are cut into 64-row tiles and launched after the full
        // rounds: twice as many workgroups, each alone on its CU (8192 x 1152: 576 tiles = 504 + 144 half tiles).
        const int tiles_n = K / MT_, tiles_m = (M + MT_ - 1) / MT_, resident = 512;
        const long tiles = (long)tiles_n * tiles_m;
        int full_m = tiles_m;
        if (tiles > resident && tiles < 4L * resident && tiles % resident != 0 && tiles % resident < resident / 2)
            full_m = (int)((tiles / resident) * resident / tiles_n);
        hipLaunchKernelGGL((blockdiag_rotate_mfma_f64_kernel<MT_>), dim3(tiles_n, full_m), dim3(256), 0, st, X, R, M, K,
                           K, U, prescale, 0);
        if (full_m < tiles_m) {
            const int row_begin = full_m * MT_;
            hipLaunchKernelGGL((blockdiag_rotate_mfma_f64_kernel<64>), dim3(tiles_n, (M - row_begin + 63) / 64),
                               dim3(256), 0, st, X, R, M, K, K, U, prescale, row_begin);
        }
    } else {
        dim3 grid(K / DT, (M + DT - 1) / DT);
        hipLaunchKernelGGL(dense_rotate_f64_kernel, grid, dim3(256), 0, st, X, R, M, K, U, prescale);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const QuantSpec qs = make_spec(act_bits, 1, zero);
    launch_quant_from_f64(st, U, M, K, qs, q, scale);
    return hipGetLastError();
}

// Structured outlier-aware rotation u = ((x . R1) . P) . R2, fp64 throughout: block-diagonal product on the fp64
// matrix cores into Z (U's storage; its products are exact, so the fused accumulation is the plain sum), row
// permutation into Zp, second block-diagonal product with separately rounded multiply and add back into U, then the
// per-token quantizer.
hipError_t launch_blockperm_rotate_quant(hipStream_t st, const uint16_t* X, int M, int K, int B, const uint16_t* R1,
                                         const int32_t* perm, const uint16_t* R2, int act_bits, double* U, double* Zp,
                                         int8_t* q, float* scale, int32_t* zero, const float* prescale) {
    double* Z = U;
    const dim3 grid(K / MT_, (M + MT_ - 1) / MT_);
    hipLaunchKernelGGL((blockdiag_rotate_mfma_f64_kernel<MT_>), grid, dim3(256), 0, st, X, R1, M, K, B, Z, prescale, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = allow_large_lds(reinterpret_cast<const void*>(permute_rows_f64_kernel), 158 * 1024);
    if (e != hipSuccess) return e;
    const int pgrid = M < 4096 ? M : 4096;
    hipLaunchKernelGGL(permute_rows_f64_kernel, dim3(pgrid), dim3(256), (size_t)K * sizeof(double), st, Z, perm, M, K, Zp);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(blockdiag_rotate_seq_f64_kernel, dim3(K / DT, (M + DT - 1) / DT), dim3(256), 0, st, Zp, R2, M, K, B, U);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const QuantSpec qs = make_spec(act_bits, 1, zero);
    launch_quant_from_f64(st, U, M, K, qs, q, scale);
    return hipGetLastError();
}

}  // namespace lrq
