// Decode + bf16 MFMA GEMM on the TLQ levels themselves (gfx950):
//   Y[t,n] = scale_t * sum_k q[t,k] * v_n(code[n,k])  (+ bias_n)
// with v_n(c) = +-round(2^r 2^I) 2^(f-I), the integerised level of "Hardware Implementation" - no per-channel
// int8 renormalisation of the levels.  For 0 <= I <= 7 a level has at most 8 significant bits and is a bf16 value;
// the activation codes (|q| <= 127) are bf16 values too, so every product is exact in fp32 and only the fp32
// accumulation of v_mfma_f32_32x32x16_bf16 rounds.  This is the fidelity reference of the int8 path: the same
// codes, the paper's value map, half the matrix rate.
//
// Workgroup = 4 waves, tile 128 rows x 256 (or 128) columns; a wave owns 64 (32) columns - NTW 32-column tiles - of all
// 128 rows.
// Activation codes are widened to bf16 once per workgroup on their way into LDS (two buffers); the packed weight
// codes go from global memory into registers (same tiling as the int8 GEMM reads) and are decoded there through a
// per-lane 16-entry table of bf16 levels, held as a high-byte and a low-byte table for byte permutes.
//
// K order inside a 64-wide K block: the lane's two 8-byte pieces of the code tiling give lane half hh (lane / 32) the
// k offsets 32 s + 16 hh + [0, 16) for s = 0, 1.  MFMA step u = 2 s + p therefore contracts the sixteen k
//   { 32 s + 16 hh + 8 p + i : hh = 0, 1; i = 0..7 }
// (an MFMA only needs both operands to agree on which k a lane holds), and a lane reads its eight activation values
// of a step as one 16-byte chunk: chunk index 4 s + 2 hh + p of the row.
#include "lrq_internal.h"

namespace lrq {
namespace {

typedef short v8s __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int BM = 128, MT = BM / 32;
constexpr int BK = kGemmBlockK;                 // 64
constexpr int PLANE = 32 * 16 + 32;             // one (row tile, 8-value chunk) plane: 32 rows x 16 bytes, padded
constexpr int ABUF = MT * 8 * PLANE;            // one A tile as bf16: 128 rows x 64 k
constexpr int EPI_ROW = 32 * 4 + 16;            // one staged output row of a 32-column tile (fp32) + pad
constexpr int EPI_WAVE = 32 * EPI_ROW;
constexpr int UNIT = 64 * 16;                   // bytes of one (32-column tile, K block) unit of the code tiling

__device__ __forceinline__ unsigned perm(unsigned hi, unsigned lo, unsigned sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// the lane's codes of one K block: its channel's two 8-byte pieces of the unit (k = 16 (l / 32) + [0, 16) and 32 more)
__device__ __forceinline__ uint4 load_pieces32(const uint8_t* p) {
    const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + kGemmPiece32Step);
    return make_uint4(lo.x, lo.y, hi.x, hi.y);
}

// Four int8 codes (one dword) -> four bf16 values (two dwords).  q + 128 is an unsigned byte; the byte -> float
// conversions and the subtraction of 128 are exact, and the float of an integer below 256 has a zero low half.
__device__ __forceinline__ void widen4(unsigned w, unsigned& lo, unsigned& hi) {
    const unsigned u = w ^ 0x80808080u;
    const float f0 = (float)(u & 0xffu) - 128.0f, f1 = (float)((u >> 8) & 0xffu) - 128.0f;
    const float f2 = (float)((u >> 16) & 0xffu) - 128.0f, f3 = (float)(u >> 24) - 128.0f;
    lo = perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
    hi = perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
}

// Level bytes of the four codes selected by idx (3 low bits per byte) and, for 16-entry tables, pick (which half).
template <int BITS>
__device__ __forceinline__ unsigned lookup4(const unsigned T[4], unsigned idx, unsigned pick) {
    if constexpr (BITS == 4) return perm(perm(T[3], T[2], idx), perm(T[1], T[0], idx), pick);
    else return perm(T[1], T[0], idx);
}

// One raw dword (8 codes: byte j = code[j] | code[4 + j] << 4) -> eight bf16 levels, k ascending.
template <int BITS>
__device__ __forceinline__ v8s decode8(unsigned w, const unsigned H[4], const unsigned L[4], unsigned C) {
    const unsigned i0 = w & 0x07070707u, i1 = (w >> 4) & 0x07070707u;
    unsigned p0 = 0, p1 = 0;
    if constexpr (BITS == 4) {
        p0 = ((w >> 1) & 0x04040404u) | C;
        p1 = ((w >> 5) & 0x04040404u) | C;
    }
    const unsigned h0 = lookup4<BITS>(H, i0, p0), l0 = lookup4<BITS>(L, i0, p0);
    const unsigned h1 = lookup4<BITS>(H, i1, p1), l1 = lookup4<BITS>(L, i1, p1);
    v4i d;
    d[0] = (int)perm(h0, l0, 0x05010400u);
    d[1] = (int)perm(h0, l0, 0x07030602u);
    d[2] = (int)perm(h1, l1, 0x05010400u);
    d[3] = (int)perm(h1, l1, 0x07030602u);
    return __builtin_bit_cast(v8s, d);
}

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ unsigned f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

template <int BITS, int NTW>
__global__ __launch_bounds__(256, NTW == 1 ? 3 : 2) void qgemm_levels_kernel(const int8_t* __restrict__ q, const float* __restrict__ scale,
                                                              int M, int K, int N, const uint8_t* __restrict__ gcodes,
                                                              const uint16_t* __restrict__ levels,
                                                              const float* __restrict__ bias, int out_fp32,
                                                              void* __restrict__ Y, int tiles_m, int tiles_n) {
    constexpr int WN = 32 * NTW, BN = 4 * WN;
    constexpr int LDS_BYTES = 2 * ABUF > 4 * EPI_WAVE ? 2 * ABUF : 4 * EPI_WAVE;
    __shared__ __attribute__((aligned(16))) unsigned char smem[LDS_BYTES];
    __shared__ float sc[BM];

    // consecutive workgroup ids go round-robin over the 8 XCDs: give each XCD a contiguous range of a tile order
    // that walks 8 row tiles per column tile, so that the tiles resident on one L2 share their panels
    const int ntiles = tiles_m * tiles_n;
    int tile;
    {
        const int x = blockIdx.x % 8, i = blockIdx.x / 8;
        const int base = ntiles / 8, rem = ntiles % 8;
        tile = x * base + (x < rem ? x : rem) + i;
    }
    int tm, tn;
    {
        constexpr int GM = 8;
        const int per_group = GM * tiles_n;
        const int group = tile / per_group, first_m = group * GM;
        const int gsize = tiles_m - first_m < GM ? tiles_m - first_m : GM;
        const int r = tile % per_group;
        tm = first_m + r % gsize;
        tn = r / gsize;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int t = threadIdx.x, lane = t % 64, wv = t / 64;
    const int KB = K / BK;
    const int ntile32 = (N + 31) / 32;

    // per-lane level tables of the lane's column in each of the wave's column tiles: high and low bytes of 16 bf16
    unsigned H[NTW][4], L[NTW][4];
    const uint8_t* bptr[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int tl = (n0 + wv * WN) / 32 + j;
        if (tl >= ntile32) tl = ntile32 - 1;
        int n = tl * 32 + lane % 32;
        if (n >= N) n = N - 1;
        const uint4 a = *reinterpret_cast<const uint4*>(levels + (size_t)n * 16);
        const uint4 b = *reinterpret_cast<const uint4*>(levels + (size_t)n * 16 + 8);
        const unsigned e[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};   // e[i] = level 2i | level 2i+1 << 16
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            L[j][i] = perm(e[2 * i + 1], e[2 * i], 0x06040200u);
            H[j][i] = perm(e[2 * i + 1], e[2 * i], 0x07050301u);
        }
        bptr[j] = gcodes + (size_t)tl * KB * UNIT + gemm_piece32_offset(lane);
    }
    unsigned C = 0x03020100u;
    asm volatile("" : "+v"(C));

    // A loader: 128 rows x 64 bytes per K block = 512 chunks of 16 codes, two per thread
    const int8_t* aptr[2];
    int aoff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int cid = t + 256 * i, row = cid / 4, c = cid % 4;
        int gr = m0 + row;
        if (gr >= M) gr = M - 1;
        aptr[i] = q + (size_t)gr * K + c * 16;
        aoff[i] = ((row / 32) * 8 + 2 * c) * PLANE + (row % 32) * 16;     // codes 16c .. 16c+15 = value chunks 2c, 2c+1
    }
    if (t < BM) sc[t] = m0 + t < M ? scale[m0 + t] : 0.0f;

    v16f acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    auto stage = [&](int buf, const v4i (&a)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            unsigned d[8];
#pragma unroll
            for (int x = 0; x < 4; ++x) widen4((unsigned)a[i][x], d[2 * x], d[2 * x + 1]);
            unsigned char* p = smem + buf * ABUF + aoff[i];
            *reinterpret_cast<uint4*>(p) = make_uint4(d[0], d[1], d[2], d[3]);
            *reinterpret_cast<uint4*>(p + PLANE) = make_uint4(d[4], d[5], d[6], d[7]);
        }
    };

    v4i aN[2];
    uint4 bC[NTW], bN[NTW];
#pragma unroll
    for (int i = 0; i < 2; ++i) aN[i] = *reinterpret_cast<const v4i*>(aptr[i]);
#pragma unroll
    for (int j = 0; j < NTW; ++j) bC[j] = load_pieces32(bptr[j]);
    stage(0, aN);
    __syncthreads();

    const int hh = lane / 32;
    const int rd_off = (lane % 32) * 16;
    for (int kb = 0; kb < KB; ++kb) {
        const int cur = kb & 1;
        const int kn = kb + 1 < KB ? kb + 1 : kb;     // the last block re-reads itself: branch-free, never used
#pragma unroll
        for (int i = 0; i < 2; ++i) aN[i] = *reinterpret_cast<const v4i*>(aptr[i] + (size_t)kn * BK);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bN[j] = load_pieces32(bptr[j] + (size_t)kn * UNIT);
        const unsigned char* A = smem + cur * ABUF;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = u / 2, p = u % 2;
            v8s b[NTW];
#pragma unroll
            for (int j = 0; j < NTW; ++j) {
                const unsigned raw[4] = {bC[j].x, bC[j].y, bC[j].z, bC[j].w};
                b[j] = decode8<BITS>(raw[u], H[j], L[j], C);
            }
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const v8s a = *reinterpret_cast<const v8s*>(&A[(i * 8 + 4 * s + 2 * hh + p) * PLANE + rd_off]);
#pragma unroll
                for (int j = 0; j < NTW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[j], acc[i][j], 0, 0, 0);
            }
        }
        // the other buffer's readers finished before the barrier that closed the previous block
        stage(cur ^ 1, aN);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bC[j] = bN[j];
        __syncthreads();
    }

    // ---- epilogue: y = acc * scale_t (+ bias), staged per wave through LDS so that a lane stores 16 bytes.
    // Lane holds column (lane % 32) and rows 8 (r / 4) + 4 (lane / 32) + r % 4 of every 32 x 32 accumulator tile.
    float bs[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int n = n0 + wv * WN + j * 32 + lane % 32;
        if (n >= N) n = N - 1;
        bs[j] = bias ? bias[n] : 0.0f;
    }
    unsigned char* slab = smem + wv * EPI_WAVE;
    const int ncol0 = n0 + wv * WN;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                const float y = acc[i][j][r] * sc[i * 32 + lr] + bs[j];
                *reinterpret_cast<float*>(&slab[lr * EPI_ROW + (lane % 32) * 4]) = y;
            }
            wave_sync();
            if (out_fp32) {
                float* Yf = reinterpret_cast<float*>(Y);
                const bool vec = N % 4 == 0;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int lr = p * 8 + lane / 8, cb = (lane % 8) * 4;
                    const uint4 v = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 4]);
                    const int row = m0 + i * 32 + lr, col = ncol0 + j * 32 + cb;
                    if (row < M) {
                        if (vec && col + 4 <= N) {
                            *reinterpret_cast<uint4*>(&Yf[(size_t)row * N + col]) = v;
                        } else {
                            const unsigned e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                            for (int x = 0; x < 4; ++x)
                                if (col + x < N) Yf[(size_t)row * N + col + x] = __uint_as_float(e[x]);
                        }
                    }
                }
            } else {
                uint16_t* Yh = reinterpret_cast<uint16_t*>(Y);
                const bool vec = N % 8 == 0;
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const int lr = p * 16 + lane / 4, cb = (lane % 4) * 8;    // 8 values per lane
                    const uint4 v0 = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 4]);
                    const uint4 v1 = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 4 + 16]);
                    const unsigned f[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                    unsigned h[8];
#pragma unroll
                    for (int x = 0; x < 8; ++x) h[x] = f32_to_bf16_rne(__uint_as_float(f[x]));
                    const int row = m0 + i * 32 + lr, col = ncol0 + j * 32 + cb;
                    if (row < M) {
                        if (vec && col + 8 <= N) {
                            *reinterpret_cast<uint4*>(&Yh[(size_t)row * N + col]) =
                                make_uint4(h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16);
                        } else {
#pragma unroll
                            for (int x = 0; x < 8; ++x)
                                if (col + x < N) Yh[(size_t)row * N + col + x] = (uint16_t)h[x];
                        }
                    }
                }
            }
            wave_sync();
        }
}

}  // namespace

hipError_t launch_qgemm_levels(hipStream_t st, const int8_t* q, const float* scale, int M, int K, const lrq_tlq_weight& w,
                               const float* bias, int out_dtype, void* Y) {
    const int fp32 = out_dtype == LRQ_OUT_FP32;
    // 128 x 256 tiles (two workgroups per CU) for long K loops; 128 x 128 (three per CU) for short ones and for N that
    // wastes much of a 256-wide tile - the same rule as the int8 GEMM's
    const bool narrow = K <= 2048 || (w.N % 256 != 0 && w.N <= 2048);
    const int bn = narrow ? 128 : 256;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (w.N + bn - 1) / bn;
    const dim3 grid(tiles_m * tiles_n), block(256);
#define LRQ_GO(B, T)                                                                                                       \
    hipLaunchKernelGGL((qgemm_levels_kernel<B, T>), grid, block, 0, st, q, scale, M, K, w.N, w.gemm_codes, w.levels, bias, \
                       fp32, Y, tiles_m, tiles_n)
    if (w.bits == 4) { if (narrow) LRQ_GO(4, 1); else LRQ_GO(4, 2); }
    else { if (narrow) LRQ_GO(3, 1); else LRQ_GO(3, 2); }
#undef LRQ_GO
    return hipGetLastError();
}

}  // namespace lrq
