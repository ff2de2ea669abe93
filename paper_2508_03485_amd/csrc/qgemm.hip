// Decode + int8 MFMA GEMM + rescale (gfx950):
//   Y[t,n] = scale_t * wscale_n * sum_k q[t,k] * lut_n[code[n,k]]  (+ bias_n)
// Activation codes q (int8, [M,K]) are staged through LDS and shared by the four waves of a
// workgroup; every wave owns its own slice of output channels, streams the packed 3/4-bit TLQ codes of
// those channels straight from global memory into registers and decodes them there with a per-lane
// level table (byte permutes), so decoded weights never touch LDS.  v_mfma_i32_32x32x32_i8 does the
// contraction with int32 accumulation ("SpeedUp and Latency": INT8 x INT8, higher-precision accumulate).
#include "lrq_internal.h"

namespace lrq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256;             // rows of Y per workgroup
constexpr int WAVES = 4;
constexpr int WN = 64;              // columns of Y per wave (two 32-wide MFMA tiles)
constexpr int BN = WAVES * WN;      // 256
constexpr int BK = kGemmBlockK;     // 64
constexpr int MT = BM / 32;         // 8 MFMA row tiles per wave
constexpr int NTW = WN / 32;        // 2 MFMA column tiles per wave
constexpr int PLANE = 32 * 16 + 64; // bytes of one (row tile, 16-byte k chunk) plane in LDS, padded
constexpr int ABUF = MT * 4 * PLANE;

__device__ __forceinline__ unsigned perm(unsigned hi, unsigned lo, unsigned sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// 4 codes (one per byte of sel, values 0..15) -> 4 int8 levels from a 16-entry table held in L[0..3].
__device__ __forceinline__ unsigned lut16(const unsigned L[4], unsigned sel) {
    const unsigned idx = sel & 0x07070707u;
    const unsigned a = perm(L[1], L[0], idx);
    const unsigned b = perm(L[3], L[2], idx);
    const unsigned pick = ((sel >> 1) & 0x04040404u) | 0x03020100u;   // byte j: j (from a) or 4 + j (from b)
    return perm(b, a, pick);
}

template <int BITS>
struct BRaw {
    unsigned d[BITS == 4 ? 4 : 3];
};

template <int BITS>
__device__ __forceinline__ BRaw<BITS> load_braw(const uint8_t* __restrict__ p) {
    BRaw<BITS> r;
    if constexpr (BITS == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        r.d[0] = v.x; r.d[1] = v.y; r.d[2] = v.z; r.d[3] = v.w;
    } else {
        const unsigned* q = reinterpret_cast<const unsigned*>(p);
        r.d[0] = q[0]; r.d[1] = q[1]; r.d[2] = q[2];
    }
    return r;
}

// Decode the 16 codes a lane feeds to MFMA step s (0 | 1) of the current K block.
template <int BITS>
__device__ __forceinline__ v4i decode_step(const BRaw<BITS>& raw, const unsigned L[4], int s) {
    v4i out;
    if constexpr (BITS == 4) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const unsigned w = raw.d[2 * s + d];
            out[2 * d] = (int)lut16(L, w & 0x0F0F0F0Fu);
            out[2 * d + 1] = (int)lut16(L, (w >> 4) & 0x0F0F0F0Fu);
        }
    } else {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const unsigned lo2 = (raw.d[s] >> (2 * g)) & 0x03030303u;
            const unsigned b2 = (raw.d[2] >> (4 * s + g)) & 0x01010101u;
            out[g] = (int)perm(L[1], L[0], (b2 << 2) | lo2);
        }
    }
    return out;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int BITS>
__global__ __launch_bounds__(256, 1) void qgemm_kernel(const int8_t* __restrict__ q, const float* __restrict__ scale,
                                                       int M, int K, int N, const uint8_t* __restrict__ gcodes,
                                                       const int8_t* __restrict__ lut, const float* __restrict__ wscale,
                                                       const float* __restrict__ bias, int out_fp32,
                                                       void* __restrict__ Y, int tiles_m, int tiles_n) {
    __shared__ __attribute__((aligned(16))) unsigned char As[2][ABUF];
    __shared__ float sc[BM];

    // XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so give each
    // XCD a contiguous range of tiles (they share rows of q / channels of W in that XCD's L2).
    const int ntiles = tiles_m * tiles_n;
    int tile = blockIdx.x;
    {
        const int per = (ntiles + 7) / 8;
        const int x = blockIdx.x % 8, i = blockIdx.x / 8;
        const int cand = x * per + i;
        // the remap is a bijection only when ntiles is a multiple of 8; otherwise keep the identity
        if (ntiles % 8 == 0) tile = cand;
    }
    const int tm = tile / tiles_n, tn = tile % tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;

    const int t = threadIdx.x, lane = t % 64, wv = t / 64;
    const int KB = K / BK;
    const int ntile32 = (N + 31) / 32;
    constexpr int UNIT = 64 * (BITS == 4 ? 16 : 12);

    // per-wave channel tiles and per-lane level tables / scales
    int wtile[NTW];
    bool wvalid[NTW];
    unsigned L[NTW][4];
    float wsc[NTW], bs[NTW];
    const uint8_t* bptr[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int tl = (n0 + wv * WN) / 32 + j;
        wvalid[j] = tl < ntile32;
        if (!wvalid[j]) tl = ntile32 - 1;
        wtile[j] = tl;
        int n = tl * 32 + lane % 32;
        if (n >= N) n = N - 1;
        const uint4 lv = *reinterpret_cast<const uint4*>(lut + (size_t)n * 16);
        L[j][0] = lv.x; L[j][1] = lv.y; L[j][2] = lv.z; L[j][3] = lv.w;
        wsc[j] = wscale[n];
        bs[j] = bias ? bias[n] : 0.0f;
        bptr[j] = gcodes + (size_t)tl * KB * UNIT + (size_t)lane * (UNIT / 64);
    }

    // A tile loader: 1024 chunks of 16 bytes, 4 per thread; chunk id -> (row, 16-byte column)
    const int8_t* aptr[4];
    int aoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int cid = t + 256 * i, row = cid / 4, c = cid % 4;
        int gr = m0 + row;
        if (gr >= M) gr = M - 1;
        aptr[i] = q + (size_t)gr * K + c * 16;
        aoff[i] = ((row / 32) * 4 + c) * PLANE + (row % 32) * 16;
    }
    {
        int r = m0 + t;
        sc[t] = r < M ? scale[r] : 0.0f;
    }

    v16i acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    uint4 areg[4];
    BRaw<BITS> braw[NTW];
#pragma unroll
    for (int i = 0; i < 4; ++i) areg[i] = *reinterpret_cast<const uint4*>(aptr[i]);
#pragma unroll
    for (int j = 0; j < NTW; ++j) braw[j] = load_braw<BITS>(bptr[j]);
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(&As[0][aoff[i]]) = areg[i];
    __syncthreads();

    const int rd_off = (lane / 32) * PLANE + (lane % 32) * 16;
    for (int kb = 0; kb < KB; ++kb) {
        const int cur = kb & 1;
        BRaw<BITS> bnext[NTW];
        const bool more = kb + 1 < KB;
        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i) areg[i] = *reinterpret_cast<const uint4*>(aptr[i] + (size_t)(kb + 1) * BK);
#pragma unroll
            for (int j = 0; j < NTW; ++j) bnext[j] = load_braw<BITS>(bptr[j] + (size_t)(kb + 1) * UNIT);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v4i b[NTW];
#pragma unroll
            for (int j = 0; j < NTW; ++j) b[j] = decode_step<BITS>(braw[j], L[j], s);
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const v4i a = *reinterpret_cast<const v4i*>(&As[cur][(i * 4 + s * 2) * PLANE + rd_off]);
#pragma unroll
                for (int j = 0; j < NTW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[j], acc[i][j], 0, 0, 0);
            }
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(&As[cur ^ 1][aoff[i]]) = areg[i];
#pragma unroll
            for (int j = 0; j < NTW; ++j) braw[j] = bnext[j];
        }
        __syncthreads();
    }

    // epilogue: lane holds column (lane % 32) and rows 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 tile
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int col = wtile[j] * 32 + lane % 32;
        if (!wvalid[j] || col >= N) continue;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = i * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                const int row = m0 + lr;
                if (row < M) {
                    const float y = ((float)acc[i][j][r] * sc[lr]) * wsc[j] + bs[j];
                    if (out_fp32) reinterpret_cast<float*>(Y)[(size_t)row * N + col] = y;
                    else reinterpret_cast<uint16_t*>(Y)[(size_t)row * N + col] = f32_to_bf16_rne(y);
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_qgemm(hipStream_t st, const int8_t* q, const float* scale, int M, int K,
                        const lrq_tlq_weight& w, const float* bias, int out_dtype, void* Y) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (w.N + BN - 1) / BN;
    const dim3 grid(tiles_m * tiles_n), block(256);
    const int fp32 = out_dtype == LRQ_OUT_FP32;
    if (w.bits == 4)
        hipLaunchKernelGGL(qgemm_kernel<4>, grid, block, 0, st, q, scale, M, K, w.N, w.gemm_codes, w.lut, w.wscale,
                           bias, fp32, Y, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL(qgemm_kernel<3>, grid, block, 0, st, q, scale, M, K, w.N, w.gemm_codes, w.lut, w.wscale,
                           bias, fp32, Y, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace lrq
