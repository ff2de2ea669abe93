// Decode + int8 MFMA GEMM + rescale (gfx950):
//   Y[t,n] = scale_t * wscale_n * sum_k q[t,k] * lut_n[code[n,k]]  (+ bias_n)
// Activation codes q (int8, [M,K]) are staged through LDS and shared by the four waves of a
// workgroup; every wave owns its own 64 output channels, streams the packed 3/4-bit TLQ codes of
// those channels straight from global memory into registers and decodes them there with a per-lane
// level table (byte permutes), so decoded weights never touch LDS.  v_mfma_i32_32x32x32_i8 does the
// contraction with int32 accumulation ("SpeedUp and Latency": INT8 x INT8, higher-precision accumulate).
// The epilogue rescales in fp32 and goes through LDS so that every lane stores 16 contiguous bytes.
#include "lrq_internal.h"

#include <cstdlib>

namespace lrq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WAVES = 4;
constexpr int WN = 64;              // columns of Y per wave (two 32-wide MFMA tiles)
constexpr int BN = WAVES * WN;      // 256
constexpr int BK = kGemmBlockK;     // 64
constexpr int NTW = WN / 32;        // 2 MFMA column tiles per wave
constexpr int PLANE = 32 * 16 + 64; // bytes of one (row tile, 16-byte k chunk) plane in LDS, padded
constexpr int EPI_ROW = 64 * 2 + 16;   // bytes of one staged output row of a wave (64 bf16 / 32 fp32) + pad
constexpr int EPI_WAVE = 32 * EPI_ROW; // one 32-row slab per wave

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

__device__ __forceinline__ unsigned f32_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// BM rows x 256 columns per workgroup of 4 waves; MT = BM / 32 MFMA row tiles per wave.
template <int BITS, int BM>
__global__ __launch_bounds__(256, BM == 128 ? 2 : 1) void qgemm_kernel(
    const int8_t* __restrict__ q, const float* __restrict__ scale, int M, int K, int N,
    const uint8_t* __restrict__ gcodes, const int8_t* __restrict__ lut, const float* __restrict__ wscale,
    const float* __restrict__ bias, int out_fp32, void* __restrict__ Y, int tiles_m, int tiles_n) {
    constexpr int MT = BM / 32;
    constexpr int ABUF = MT * 4 * PLANE;
    constexpr int ALOADS = BM * 4 / 256;        // 16-byte chunks of the A tile per thread
    constexpr int LDS_BYTES = (2 * ABUF > WAVES * EPI_WAVE) ? 2 * ABUF : WAVES * EPI_WAVE;
    __shared__ __attribute__((aligned(16))) unsigned char smem[LDS_BYTES];
    __shared__ float sc[BM];

    // XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so hand each XCD a
    // contiguous range of tiles (neighbouring tiles share rows of q / channels of W in that XCD's L2).
    const int ntiles = tiles_m * tiles_n;
    int tile;
    {
        const int x = blockIdx.x % 8, i = blockIdx.x / 8;
        const int base = ntiles / 8, rem = ntiles % 8;           // XCD x owns base + (x < rem) tiles
        tile = x * base + (x < rem ? x : rem) + i;
    }
    // column-major over tiles: consecutive tiles of an XCD walk down M and share the same weight columns
    const int tn = tile / tiles_m, tm = tile % tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;

    const int t = threadIdx.x, lane = t % 64, wv = t / 64;
    const int KB = K / BK;
    const int ntile32 = (N + 31) / 32;
    constexpr int UNIT = 64 * (BITS == 4 ? 16 : 12);

    unsigned L[NTW][4];
    const uint8_t* bptr[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int tl = (n0 + wv * WN) / 32 + j;
        if (tl >= ntile32) tl = ntile32 - 1;
        int n = tl * 32 + lane % 32;
        if (n >= N) n = N - 1;
        const uint4 lv = *reinterpret_cast<const uint4*>(lut + (size_t)n * 16);
        L[j][0] = lv.x; L[j][1] = lv.y; L[j][2] = lv.z; L[j][3] = lv.w;
        bptr[j] = gcodes + (size_t)tl * KB * UNIT + (size_t)lane * (UNIT / 64);
    }

    // A tile loader: BM*4 chunks of 16 bytes; chunk id -> (row, 16-byte column)
    const int8_t* aptr[ALOADS];
    int aoff[ALOADS];
#pragma unroll
    for (int i = 0; i < ALOADS; ++i) {
        const int cid = t + 256 * i, row = cid / 4, c = cid % 4;
        int gr = m0 + row;
        if (gr >= M) gr = M - 1;
        aptr[i] = q + (size_t)gr * K + c * 16;
        aoff[i] = ((row / 32) * 4 + c) * PLANE + (row % 32) * 16;
    }
    if (t < BM) {
        const int r = m0 + t;
        sc[t] = r < M ? scale[r] : 0.0f;
    }

    v16i acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // ---- prologue: A tile 0 -> LDS buffer 0; A tiles 1, 2 and B blocks 0, 1, 2 in flight in registers
    uint4 a1[ALOADS], a2[ALOADS];
    BRaw<BITS> b0[NTW], b1[NTW], b2[NTW];
    {
        uint4 a0[ALOADS];
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) a0[i] = *reinterpret_cast<const uint4*>(aptr[i]);
        const int k1 = KB > 1 ? 1 : 0, k2 = KB > 2 ? 2 : KB - 1;
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            b0[j] = load_braw<BITS>(bptr[j]);
            b1[j] = load_braw<BITS>(bptr[j] + (size_t)k1 * UNIT);
            b2[j] = load_braw<BITS>(bptr[j] + (size_t)k2 * UNIT);
        }
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) {
            a1[i] = *reinterpret_cast<const uint4*>(aptr[i] + (size_t)k1 * BK);
            a2[i] = *reinterpret_cast<const uint4*>(aptr[i] + (size_t)k2 * BK);
        }
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) *reinterpret_cast<uint4*>(&smem[aoff[i]]) = a0[i];
    }
    __syncthreads();

    const int rd_off = (lane / 32) * PLANE + (lane % 32) * 16;
    for (int kb = 0; kb < KB; ++kb) {
        const unsigned char* Acur = smem + (kb & 1) * ABUF;
        unsigned char* Anxt = smem + ((kb & 1) ^ 1) * ABUF;
        // stage A tile kb+1 (loaded two iterations ago) and start the loads of tile kb+3 / block kb+3
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) *reinterpret_cast<uint4*>(&Anxt[aoff[i]]) = a1[i];
        const int k3 = kb + 3 < KB ? kb + 3 : KB - 1;
        BRaw<BITS> b3[NTW];
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) {
            a1[i] = a2[i];
            a2[i] = *reinterpret_cast<const uint4*>(aptr[i] + (size_t)k3 * BK);
        }
#pragma unroll
        for (int j = 0; j < NTW; ++j) b3[j] = load_braw<BITS>(bptr[j] + (size_t)k3 * UNIT);

        v4i af0[MT], af1[MT], bd[NTW];
#pragma unroll
        for (int i = 0; i < MT; ++i) af0[i] = *reinterpret_cast<const v4i*>(&Acur[(i * 4 + 0) * PLANE + rd_off]);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bd[j] = decode_step<BITS>(b0[j], L[j], 0);
#pragma unroll
        for (int i = 0; i < MT; ++i) af1[i] = *reinterpret_cast<const v4i*>(&Acur[(i * 4 + 2) * PLANE + rd_off]);
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTW; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af0[i], bd[j], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bd[j] = decode_step<BITS>(b0[j], L[j], 1);
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTW; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af1[i], bd[j], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            b0[j] = b1[j];
            b1[j] = b2[j];
            b2[j] = b3[j];
        }
        __syncthreads();
    }

    // ---- epilogue: rescale in fp32, stage one 32-row slab per wave in LDS, store 16 bytes per lane.
    // Lane holds column (lane % 32) and rows 8*(r/4) + 4*(lane/32) + r%4 of every 32x32 accumulator tile.
    float wsc[NTW], bs[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int n = n0 + wv * WN + j * 32 + lane % 32;
        if (n >= N) n = N - 1;
        wsc[j] = wscale[n];
        bs[j] = bias ? bias[n] : 0.0f;
    }
    unsigned char* slab = smem + wv * EPI_WAVE;
    const int ncol0 = n0 + wv * WN;                 // first column of this wave
    const bool vec = (N % (out_fp32 ? 4 : 8)) == 0; // rows of Y are 16-byte aligned
    if (!out_fp32) {
        uint16_t* Yh = reinterpret_cast<uint16_t*>(Y);
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int j = 0; j < NTW; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lr = 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                    const float y = ((float)acc[i][j][r] * sc[i * 32 + lr]) * wsc[j] + bs[j];
                    *reinterpret_cast<uint16_t*>(&slab[lr * EPI_ROW + (j * 32 + lane % 32) * 2]) = (uint16_t)f32_to_bf16_rne(y);
                }
            __syncthreads();
            // 32 rows x 128 bytes: 8 lanes per row, 8 rows per pass
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int lr = p * 8 + lane / 8, cb = (lane % 8) * 8;        // 8 bf16 per lane
                const uint4 v = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 2]);
                const int row = m0 + i * 32 + lr, col = ncol0 + cb;
                if (row < M) {
                    if (vec && col + 8 <= N) {
                        *reinterpret_cast<uint4*>(&Yh[(size_t)row * N + col]) = v;
                    } else {
                        const uint16_t* e = reinterpret_cast<const uint16_t*>(&v);
                        for (int x = 0; x < 8; ++x)
                            if (col + x < N) Yh[(size_t)row * N + col + x] = e[x];
                    }
                }
            }
            __syncthreads();
        }
    } else {
        float* Yf = reinterpret_cast<float*>(Y);
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTW; ++j) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lr = 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
                    const float y = ((float)acc[i][j][r] * sc[i * 32 + lr]) * wsc[j] + bs[j];
                    *reinterpret_cast<float*>(&slab[lr * EPI_ROW + (lane % 32) * 4]) = y;
                }
                __syncthreads();
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int lr = p * 8 + lane / 8, cb = (lane % 8) * 4;    // 4 floats per lane
                    const uint4 v = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 4]);
                    const int row = m0 + i * 32 + lr, col = ncol0 + j * 32 + cb;
                    if (row < M) {
                        if (vec && col + 4 <= N) {
                            *reinterpret_cast<uint4*>(&Yf[(size_t)row * N + col]) = v;
                        } else {
                            const float* e = reinterpret_cast<const float*>(&v);
                            for (int x = 0; x < 4; ++x)
                                if (col + x < N) Yf[(size_t)row * N + col + x] = e[x];
                        }
                    }
                }
                __syncthreads();
            }
    }
}

template <int BITS, int BM>
hipError_t launch(hipStream_t st, const int8_t* q, const float* scale, int M, int K, const lrq_tlq_weight& w,
                  const float* bias, int fp32, void* Y) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (w.N + BN - 1) / BN;
    hipLaunchKernelGGL((qgemm_kernel<BITS, BM>), dim3(tiles_m * tiles_n), dim3(256), 0, st, q, scale, M, K, w.N,
                       w.gemm_codes, w.lut, w.wscale, bias, fp32, Y, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_qgemm(hipStream_t st, const int8_t* q, const float* scale, int M, int K,
                        const lrq_tlq_weight& w, const float* bias, int out_dtype, void* Y) {
    const int fp32 = out_dtype == LRQ_OUT_FP32;
    static const int bm = [] { const char* e = getenv("LRQ_GEMM_BM"); return e ? atoi(e) : 128; }();
    if (bm == 256) {
        if (w.bits == 4) return launch<4, 256>(st, q, scale, M, K, w, bias, fp32, Y);
        return launch<3, 256>(st, q, scale, M, K, w, bias, fp32, Y);
    }
    if (w.bits == 4) return launch<4, 128>(st, q, scale, M, K, w, bias, fp32, Y);
    return launch<3, 128>(st, q, scale, M, K, w, bias, fp32, Y);
}

}  // namespace lrq
