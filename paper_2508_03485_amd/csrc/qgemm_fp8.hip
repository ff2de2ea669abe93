// Decode + FP8 MFMA GEMM (gfx950): the alternative value map of "Hardware Implementation" with I = 3 mantissa bits,
//   Y[t,n] = scale_t * wscale_fp8_n * sum_k q[t,k] * value(lut_fp8_n[code[n,k]])  (+ bias_n)
// Both operands of v_mfma_f32_32x32x64_f8f6f4 are FP8 E4M3: the 4-bit activation codes (integers in [-7, 7], written
// as E4M3 bytes by the rotate kernels) and the levels +-round(2^r 2^3) 2^(f-3) scaled by a per-channel power of two.
// Every product is exact in fp32; the instruction's fp32 accumulation rounds.
//
// Workgroup = 4 waves, tile 128 rows x 256 (or 128) columns; a wave owns NTW 32-column tiles of all 128 rows.  The
// activation bytes go global -> registers -> LDS (two buffers, the plane layout of the int8 GEMM); the packed weight
// codes go from global memory into registers (the int8 GEMM's tiling) and are decoded there through the lane's own
// 16-entry byte table.  One matrix instruction contracts a whole 64-wide K block: the code tiling gives lane half hh
// the k offsets 16 hh + [0, 16) and 32 + 16 hh + [0, 16), and the lane reads the activation bytes of the same k as two
// 16-byte chunks - an MFMA only needs both operands to agree on which k a lane's byte positions hold.
#include "lrq_internal.h"

namespace lrq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 128, MT = BM / 32;
constexpr int BK = kGemmBlockK;                 // 64
constexpr int PLANE = 32 * 16 + 32;             // one (row tile, 16-byte k chunk) plane in LDS, padded
constexpr int ABUF = MT * 4 * PLANE;
constexpr int UNIT = 64 * 16;                   // bytes of one (32-column tile, K block) unit of the code tiling

__device__ __forceinline__ unsigned perm(unsigned hi, unsigned lo, unsigned sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// the lane's codes of one K block: its channel's two 8-byte pieces of the unit (k = 16 (l / 32) + [0, 16) and 32 more)
__device__ __forceinline__ uint4 load_pieces32(const uint8_t* p) {
    const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + kGemmPiece32Step);
    return make_uint4(lo.x, lo.y, hi.x, hi.y);
}

// Raw dword (8 codes: byte j = code[j] | code[4 + j] << 4) -> the table bytes of codes 0..3 (lo) and 4..7 (hi).
template <int BITS>
__device__ __forceinline__ void decode8(unsigned w, const unsigned T[4], unsigned C, unsigned& lo, unsigned& hi) {
    const unsigned i0 = w & 0x07070707u, i1 = (w >> 4) & 0x07070707u;
    if constexpr (BITS == 4) {
        const unsigned p0 = ((w >> 1) & 0x04040404u) | C, p1 = ((w >> 5) & 0x04040404u) | C;
        lo = perm(perm(T[3], T[2], i0), perm(T[1], T[0], i0), p0);
        hi = perm(perm(T[3], T[2], i1), perm(T[1], T[0], i1), p1);
    } else {
        lo = perm(T[1], T[0], i0);
        hi = perm(T[1], T[0], i1);
    }
}

__device__ __forceinline__ unsigned f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

template <int BITS, int NTW>
__global__ __launch_bounds__(256, 2) void qgemm_fp8_kernel(const uint8_t* __restrict__ q, const float* __restrict__ scale, int M, int K,
                                                           int N, const uint8_t* __restrict__ gcodes,
                                                           const uint8_t* __restrict__ lut, const float* __restrict__ wscale,
                                                           const float* __restrict__ bias, int out_fp32, void* __restrict__ Y,
                                                           int tiles_m, int tiles_n) {
    constexpr int WN = 32 * NTW, BN = 4 * WN;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * ABUF];
    __shared__ float sc[BM];
    // consecutive workgroup ids go round-robin over the 8 XCDs: each XCD gets a contiguous range of a tile order that
    // walks 8 row tiles per column tile, so that the tiles resident on one L2 share their panels
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

    unsigned T[NTW][4];
    const uint8_t* bptr[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int tl = (n0 + wv * WN) / 32 + j;
        if (tl >= ntile32) tl = ntile32 - 1;
        int n = tl * 32 + lane % 32;
        if (n >= N) n = N - 1;
        const uint4 lv = *reinterpret_cast<const uint4*>(lut + (size_t)n * 16);
        T[j][0] = lv.x; T[j][1] = lv.y; T[j][2] = lv.z; T[j][3] = lv.w;
        bptr[j] = gcodes + (size_t)tl * KB * UNIT + gemm_piece32_offset(lane);
    }
    unsigned C = 0x03020100u;
    asm volatile("" : "+v"(C));

    // A loader: 128 rows x 64 bytes per K block = 512 chunks of 16 bytes, two per thread
    const uint8_t* aptr[2];
    int aoff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int cid = t + 256 * i, row = cid / 4, c = cid % 4;
        int gr = m0 + row;
        if (gr >= M) gr = M - 1;
        aptr[i] = q + (size_t)gr * K + c * 16;
        aoff[i] = ((row / 32) * 4 + c) * PLANE + (row % 32) * 16;
    }
    if (t < BM) sc[t] = m0 + t < M ? scale[m0 + t] : 0.0f;

    v16f acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    v4i aN[2];
    uint4 bC[NTW], bN[NTW];
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<v4i*>(&smem[aoff[i]]) = *reinterpret_cast<const v4i*>(aptr[i]);
#pragma unroll
    for (int j = 0; j < NTW; ++j) bC[j] = load_pieces32(bptr[j]);
    __syncthreads();

    const int rd_off = (lane / 32) * PLANE + (lane % 32) * 16;
    for (int kb = 0; kb < KB; ++kb) {
        const int cur = kb & 1;
        const int kn = kb + 1 < KB ? kb + 1 : kb;     // the last block re-reads itself: branch-free, never used
#pragma unroll
        for (int i = 0; i < 2; ++i) aN[i] = *reinterpret_cast<const v4i*>(aptr[i] + (size_t)kn * BK);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bN[j] = load_pieces32(bptr[j] + (size_t)kn * UNIT);
        v8i b[NTW];
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            const unsigned raw[4] = {bC[j].x, bC[j].y, bC[j].z, bC[j].w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {           // raw dword d: k offsets 32 (d / 2) + 16 hh + 8 (d % 2) + [0, 8)
                unsigned lo, hi;
                decode8<BITS>(raw[d], T[j], C, lo, hi);
                b[j][2 * d] = (int)lo;
                b[j][2 * d + 1] = (int)hi;
            }
        }
        const unsigned char* A = smem + cur * ABUF + rd_off;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const v4i a0 = *reinterpret_cast<const v4i*>(A + (i * 4 + 0) * PLANE);      // k = 16 hh + [0, 16)
            const v4i a1 = *reinterpret_cast<const v4i*>(A + (i * 4 + 2) * PLANE);      // k = 32 + 16 hh + [0, 16)
            const v8i a = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
#pragma unroll
            for (int j = 0; j < NTW; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b[j], acc[i][j], 0, 0, 0, 0, 0, 0);
        }
        // the other buffer's readers finished before the barrier that closed the previous block
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<v4i*>(&smem[(cur ^ 1) * ABUF + aoff[i]]) = aN[i];
#pragma unroll
        for (int j = 0; j < NTW; ++j) bC[j] = bN[j];
        __syncthreads();
    }

    // epilogue: lane holds column (lane % 32) and rows 8 (r / 4) + 4 (lane / 32) + r % 4 of every 32 x 32 accumulator tile
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int n = n0 + wv * WN + j * 32 + lane % 32;
        if (n >= N) continue;
        const float ws = wscale[n], bs = bias ? bias[n] : 0.0f;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = i * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4), row = m0 + lr;
                if (row < M) {
                    const float y = (acc[i][j][r] * sc[lr]) * ws + bs;
                    if (out_fp32) reinterpret_cast<float*>(Y)[(size_t)row * N + n] = y;
                    else reinterpret_cast<uint16_t*>(Y)[(size_t)row * N + n] = (uint16_t)f32_to_bf16_rne(y);
                }
            }
    }
}

}  // namespace

hipError_t launch_qgemm_fp8(hipStream_t st, const uint8_t* q8, const float* scale, int M, int K, const lrq_tlq_weight& w,
                            const float* bias, int out_dtype, void* Y) {
    const int fp32 = out_dtype == LRQ_OUT_FP32;
    const bool narrow = K <= 2048 || (w.N % 256 != 0 && w.N <= 2048);
    const int tiles_m = (M + BM - 1) / BM;
#define LRQ_GO(B, T)                                                                                                     \
    hipLaunchKernelGGL((qgemm_fp8_kernel<B, T>), dim3(tiles_m * ((w.N + 128 * T - 1) / (128 * T))), dim3(256), 0, st, q8, scale, M, K, \
                       w.N, w.gemm_codes, w.lut_fp8, w.wscale_fp8, bias, fp32, Y, tiles_m, (w.N + 128 * T - 1) / (128 * T))
    if (w.bits == 4) { if (narrow) LRQ_GO(4, 1); else LRQ_GO(4, 2); }
    else { if (narrow) LRQ_GO(3, 1); else LRQ_GO(3, 2); }
#undef LRQ_GO
    return hipGetLastError();
}

}  // namespace lrq
