// Decode + int8 MFMA GEMM + rescale (gfx950):
//   Y[t,n] = scale_t * wscale_n * sum_k q[t,k] * lut_n[code[n,k]]  (+ bias_n)
// Activation codes q (int8, [M,K]) are staged through LDS (three rotating buffers) and shared by the four
// waves of a workgroup; every wave owns its own 64 output channels, streams the packed 3/4-bit TLQ codes of
// those channels straight from global memory into registers and decodes them there with per-lane
// level tables (byte permutes), so decoded weights never touch LDS.  v_mfma_i32_16x16x64_i8 does the
// contraction with int32 accumulation ("SpeedUp and Latency": INT8 x INT8, higher-precision accumulate): one
// instruction per 16 x 16 output tile and K block of 64.  (On pseudo-random operands the chip sustains 3.9 POP/s with
// this instruction and 3.3 POP/s with v_mfma_i32_32x32x32_i8: the matrix pipe is power-limited and this shape draws
// less per operation.)
// The epilogue rescales in fp32 and goes through LDS so that every lane stores 16 contiguous bytes.
#include "lrq_internal.h"

namespace lrq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int WAVES = 4;
constexpr int BK = kGemmBlockK;     // 64
constexpr int PLANE_PAD = 32;          // padding of a plane (swept 0 / 16 / 32 / 48: 32 leaves the fewest bank conflicts)
constexpr int AF_DIST = 2;             // A fragments are read this many row tiles (four MFMAs each) ahead of their use (swept 2 - 4: no difference)
constexpr int PLANE = 32 * 16 + PLANE_PAD;     // bytes of one (row tile, 16-byte k chunk) plane in LDS, padded
constexpr int EPI_ROW = 64 * 2 + 16;   // bytes of one staged output row of a wave (up to 64 bf16 / 32 fp32) + pad
constexpr int EPI_WAVE = 32 * EPI_ROW; // one 32-row slab per wave

__device__ __forceinline__ unsigned perm(unsigned hi, unsigned lo, unsigned sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// Raw operand codes of one lane for one K block and one 32-channel tile: its 16-byte slot of the code tiling, i.e. the
// 16 codes (k = 16 (lane / 16) + [0, 16) of the block) of channel lane % 16 of the tile in dwords 0, 1 and those of channel
// 16 + lane % 16 in dwords 2, 3; one nibble each, either bit-width.
template <int BITS>
struct BRaw {
    unsigned d[4];
};

template <int BITS>
__device__ __forceinline__ BRaw<BITS> load_braw(const uint8_t* __restrict__ p) {
    BRaw<BITS> r;
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    r.d[0] = v.x; r.d[1] = v.y; r.d[2] = v.z; r.d[3] = v.w;
    return r;
}

// Decode the 4 codes of operand dword g (0..3) of the slot's channel s (0 | 1).  Raw dword 2s + g/2 holds 8
// codes, byte j = code[j] | code[4+j] << 4.
// 4-bit: the level table has 16 entries (L[0..1] codes 0..7, L[2..3] codes 8..15 = negative twin): two 8-entry byte
// permutes and a third that picks per byte by the code's sign bit.  C = 0x03020100 must live in a VGPR so that the
// pick selector is a single v_and_or_b32.
// 3-bit: 8-entry table, the masked nibbles are the selectors of one byte permute.
template <int BITS>
__device__ __forceinline__ unsigned decode_dword(const BRaw<BITS>& raw, const unsigned L[4], int s, int g, unsigned C) {
    const unsigned w = raw.d[2 * s + g / 2];
    if constexpr (BITS == 4) {
        unsigned idx, pick;
        if (g % 2 == 0) {
            idx = w & 0x07070707u;
            pick = ((w >> 1) & 0x04040404u) | C;
        } else {
            idx = (w >> 4) & 0x07070707u;
            pick = ((w >> 5) & 0x04040404u) | C;
        }
        const unsigned a = perm(L[1], L[0], idx);
        const unsigned b = perm(L[3], L[2], idx);
        return perm(b, a, pick);
    } else {
        const unsigned idx = (g % 2 == 0 ? w : (w >> 4)) & 0x07070707u;
        return perm(L[1], L[0], idx);
    }
}

// Orders a wave's own LDS writes before its own later LDS reads (the LDS pipe serves one wave's requests in
// order; this only stops the compiler from moving accesses across it).  Enough for wave-private LDS regions.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// two floats -> two bf16 (round-to-nearest-even, v_cvt_pk_bf16_f32), a in the low half
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
    const f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// One K block of the main loop.  The A tiles rotate through three LDS buffers: block kb multiplies from `cur`
// (tile kb), stages tile kb+2 (held in aS, which is then reloaded with tile kb+4) into `st`, and - because tile kb+1
// in `nx` has been complete since the previous barrier - reads the first A fragments of block kb+1 before its own
// closing barrier, so that the next block starts on the matrix cores without waiting for LDS.
// bdCur holds the decoded B operands of block kb (one per 16-column tile); bRaw holds the raw codes of block kb+1, which
// are decoded into bdNxt between the matrix instructions of this block (so that the decode issues in their shadow) and
// then reloaded with block kb+3 (the other raw set, block kb+2, is in flight meanwhile).
// Packed 4-bit activation codes (A4P): a 16-byte chunk holds 32 codes, eight per dword, byte j of a dword = code[j] + 8 in
// the low nibble and code[4 + j] + 8 in the high nibble.  It is widened on its way into LDS to two 16-byte chunks of
// bytes in [1, 15]; the constant offset 8 leaves through the epilogue as a zero-point of -8 (times the channel's level sum).
template <bool A4P>
__device__ __forceinline__ void stage_a(unsigned char* dst, v4i a) {
    if constexpr (!A4P) {
        *reinterpret_cast<v4i*>(dst) = a;
    } else {
        v4i lo, hi;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const unsigned w = (unsigned)a[d];
            const unsigned l = w & 0x0f0f0f0fu, h = (w >> 4) & 0x0f0f0f0fu;
            if (d < 2) { lo[2 * d] = (int)l; lo[2 * d + 1] = (int)h; }
            else { hi[2 * (d - 2)] = (int)l; hi[2 * (d - 2) + 1] = (int)h; }
        }
        *reinterpret_cast<v4i*>(dst) = lo;
        *reinterpret_cast<v4i*>(dst + PLANE) = hi;
    }
}

template <int BITS, int RT, int NTW, int ALOADS, bool A4P>
__device__ __forceinline__ void kblock(unsigned char* smem, int cur, int st, int nx, v4i (&aS)[ALOADS],
                                       BRaw<BITS> (&bRaw)[NTW], int kb, int KB,
                                       const int8_t* const (&aptr)[ALOADS], const int (&aoff)[ALOADS],
                                       const uint8_t* const (&bptr)[NTW], const unsigned (&L)[2 * NTW][4], unsigned C,
                                       const v4i (&bdCur)[2 * NTW], v4i (&bdNxt)[2 * NTW], v4i (&acc)[RT][2 * NTW], int rd_off,
                                       v4i (&afp)[AF_DIST]) {
    constexpr int UNIT = 64 * 16;
    constexpr int CT = 2 * NTW;                     // 16-column tiles of a wave
    constexpr int ABK = A4P ? BK / 2 : BK;          // bytes of a token row per K block
    const unsigned char* Acur = smem + cur;
#pragma unroll
    for (int i = 0; i < ALOADS; ++i) stage_a<A4P>(&smem[st + aoff[i]], aS[i]);
    const int ka = kb + 4 < KB ? kb + 4 : KB - 1;
    const int kbn = kb + 3 < KB ? kb + 3 : KB - 1;
#pragma unroll
    for (int i = 0; i < ALOADS; ++i) aS[i] = *reinterpret_cast<const v4i*>(aptr[i] + (size_t)ka * ABK);
    v4i af[RT];
    constexpr int DPB = (CT * 4 + RT - 1) / RT;     // operand dwords decoded per row tile
    constexpr int DIST = AF_DIST;                   // A fragments are read this many row tiles ahead
#pragma unroll
    for (int p = 0; p < DIST; ++p) af[p] = afp[p];
#pragma unroll
    for (int p = 0; p < RT; ++p) {
        if (p == RT - 2) {          // next block's first fragments, early enough to land before the closing barrier
#pragma unroll
            for (int pp = 0; pp < DIST; ++pp)
                afp[pp] = *reinterpret_cast<const v4i*>(&smem[nx + (pp / 2) * 4 * PLANE + (pp % 2) * 256 + rd_off]);
        }
        if (p + DIST < RT)
            af[p + DIST] = *reinterpret_cast<const v4i*>(&Acur[((p + DIST) / 2) * 4 * PLANE + ((p + DIST) % 2) * 256 + rd_off]);
#pragma unroll
        for (int d = 0; d < DPB; ++d) {
            const int dd = p * DPB + d, ct = dd / 4;
            if (dd < CT * 4) bdNxt[ct][dd % 4] = (int)decode_dword<BITS>(bRaw[ct / 2], L[ct], ct % 2, dd % 4, C);
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
            acc[p][ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[p], bdCur[ct], acc[p][ct], 0, 0, 0);
        if (p == RT - 1) {
#pragma unroll
            for (int j = 0; j < NTW; ++j) bRaw[j] = load_braw<BITS>(bptr[j] + (size_t)kbn * UNIT);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
}

// BM rows x (4 waves x NTW x 32) columns per workgroup; RT = BM / 16 row tiles and 2 NTW column tiles of 16 per wave.  Shapes in use
// (launch_qgemm picks): 128 x 256 (NTW = 2, 128 accumulator registers per lane, two workgroups per CU), 128 x 128
// (NTW = 1, 64 accumulator registers, three per CU) and 64 x 128 for a few tokens (256-row shapes - half the decode
// work per MFMA - measured no faster, or slower, on every workload).  ZP: zero-point form (epilogue term).
template <int BITS, int BM, int NTW, bool ZP, bool A4P = false>
__global__ __launch_bounds__(256, BM * NTW <= 128 ? 3 : (BM * NTW <= 256 ? 2 : 1)) void qgemm_kernel(
    const int8_t* __restrict__ q, const float* __restrict__ scale, int M, int K, int N,
    const uint8_t* __restrict__ gcodes, const int8_t* __restrict__ lut, const float* __restrict__ wscale,
    const float* __restrict__ bias, int out_fp32, void* __restrict__ Y, int tiles_m, int tiles_n,
    const int32_t* __restrict__ zero, const int32_t* __restrict__ colsum, int const_zero) {
    static_assert(!A4P || ZP, "the packed form needs the zero-point term of the epilogue");
    constexpr int RT = BM / 16, CT = 2 * NTW;
    constexpr int WN = 32 * NTW, BN = WAVES * WN;
    constexpr int ABUF = (BM / 32) * 4 * PLANE;
    constexpr int ACHUNKS = A4P ? BM * 2 : BM * 4;                 // 16-byte chunks of the A tile in global memory
    constexpr int ALOADS = ACHUNKS >= 256 ? ACHUNKS / 256 : 1;      // per thread (fewer chunks than threads: some are fetched twice)
    constexpr int ABK = A4P ? BK / 2 : BK;
    constexpr int LDS_BYTES = (3 * ABUF > WAVES * EPI_WAVE) ? 3 * ABUF : WAVES * EPI_WAVE;
    __shared__ __attribute__((aligned(16))) unsigned char smem[LDS_BYTES];
    __shared__ __attribute__((aligned(16))) float sc[BM];
    __shared__ __attribute__((aligned(16))) int zr[BM];          // per-token zero-points (zero-point form only)

    // XCD-aware tile order.  Consecutive workgroup ids go round-robin over the 8 XCDs (each with its own L2), so
    // XCD x is handed a contiguous range of a linear tile order; that order walks 8-row-tile groups n-fastest
    // within 8 consecutive m (grouped ordering), so the ~64 tiles resident on an XCD at any time form an
    // 8 x 8 patch that shares each row panel of q and each channel panel of W eight ways through that L2.
    const int ntiles = tiles_m * tiles_n;
    int tile;
    {
        const int x = blockIdx.x % 8, i = blockIdx.x / 8;
        const int base = ntiles / 8, rem = ntiles % 8;           // XCD x owns base + (x < rem) tiles
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
    constexpr int UNIT = 64 * 16;

    // level tables of the lane's channel (lane % 16) in each of the wave's 16-column tiles, and the lane's slot of every
    // 32-channel tile
    unsigned L[CT][4];
    const uint8_t* bptr[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int tl = (n0 + wv * WN) / 32 + j;
        if (tl >= ntile32) tl = ntile32 - 1;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int n = tl * 32 + h * 16 + lane % 16;
            if (n >= N) n = N - 1;
            const uint4 lv = *reinterpret_cast<const uint4*>(lut + (size_t)n * 16);
            L[2 * j + h][0] = lv.x; L[2 * j + h][1] = lv.y; L[2 * j + h][2] = lv.z; L[2 * j + h][3] = lv.w;
        }
        bptr[j] = gcodes + (size_t)tl * KB * UNIT + (size_t)lane * (UNIT / 64);
    }

    // A tile loader: BM*4 chunks of 16 bytes; chunk id -> (row, 16-byte column)
    const int8_t* aptr[ALOADS];
    int aoff[ALOADS];
#pragma unroll
    for (int i = 0; i < ALOADS; ++i) {
        const int cid = (t + 256 * i) % ACHUNKS;
        const int row = A4P ? cid / 2 : cid / 4, c = A4P ? 2 * (cid % 2) : cid % 4;      // c: first 16-byte chunk in LDS
        int gr = m0 + row;
        if (gr >= M) gr = M - 1;
        aptr[i] = A4P ? q + (size_t)gr * (K / 2) + (c / 2) * 16 : q + (size_t)gr * K + c * 16;
        aoff[i] = ((row / 32) * 4 + c) * PLANE + (row % 32) * 16;
    }
    if (t < BM) {
        const int r = m0 + t;
        sc[t] = r < M ? scale[r] : 0.0f;
        zr[t] = (ZP && r < M) ? (zero ? zero[r] : const_zero) : 0;
    }

    v4i acc[RT][CT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0;

    // ---- prologue: A tiles 0, 1 -> LDS buffers 0, 1; A tiles 2 (aO), 3 (aE) in registers; B block 0 decoded (bdA), raw
    // codes of blocks 1 (bO) and 2 (bE) in registers
    unsigned C = 0x03020100u;
    asm volatile("" : "+v"(C));
    v4i aO[ALOADS], aE[ALOADS];
    BRaw<BITS> bE[NTW], bO[NTW];
    v4i bdA[CT], bdB[CT];
    {
        v4i a0[ALOADS], a1[ALOADS];
        BRaw<BITS> b0[NTW];
        const int k1 = KB > 1 ? 1 : 0, k2 = KB > 2 ? 2 : KB - 1, k3 = KB > 3 ? 3 : KB - 1;
#pragma unroll
        for (int j = 0; j < NTW; ++j) b0[j] = load_braw<BITS>(bptr[j]);
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) {
            a0[i] = *reinterpret_cast<const v4i*>(aptr[i]);
            a1[i] = *reinterpret_cast<const v4i*>(aptr[i] + (size_t)k1 * ABK);
        }
        // same issue order as the steady state of the K loop (A set, B block, A set, B block), so that the wait
        // counters the compiler derives at the loop head are the loop's own and not a conservative merge
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) aO[i] = *reinterpret_cast<const v4i*>(aptr[i] + (size_t)k2 * ABK);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bO[j] = load_braw<BITS>(bptr[j] + (size_t)k1 * UNIT);
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) aE[i] = *reinterpret_cast<const v4i*>(aptr[i] + (size_t)k3 * ABK);
#pragma unroll
        for (int j = 0; j < NTW; ++j) bE[j] = load_braw<BITS>(bptr[j] + (size_t)k2 * UNIT);
#pragma unroll
        for (int i = 0; i < ALOADS; ++i) {
            stage_a<A4P>(&smem[aoff[i]], a0[i]);
            stage_a<A4P>(&smem[ABUF + aoff[i]], a1[i]);
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int g = 0; g < 4; ++g) bdA[ct][g] = (int)decode_dword<BITS>(b0[ct / 2], L[ct], ct % 2, g, C);
    }
    __syncthreads();

    // fragment of row tile i (16 rows) of a buffer: + (i / 2) * 4 * PLANE + (i % 2) * 256; the lane's row lane % 16 and
    // its 16-byte k chunk lane / 16
    const int rd_off = (lane / 16) * PLANE + (lane % 16) * 16;
    v4i afp[AF_DIST];
#pragma unroll
    for (int p = 0; p < AF_DIST; ++p)
        afp[p] = *reinterpret_cast<const v4i*>(&smem[(p / 2) * 4 * PLANE + (p % 2) * 256 + rd_off]);

    int o0 = 0, o1 = ABUF, o2 = 2 * ABUF;       // LDS buffers of tiles kb, kb+1, kb+2
    int kb = 0;
    // two K blocks per trip with no branch in between: with a conditional second block the compiler has to assume the
    // shorter path at the loop head and drains the whole load queue there (s_waitcnt vmcnt(0)) on every trip
    for (; kb + 1 < KB; kb += 2) {
        kblock<BITS, RT, NTW, ALOADS, A4P>(smem, o0, o2, o1, aO, bO, kb, KB, aptr, aoff, bptr, L, C, bdA, bdB, acc, rd_off, afp);
        kblock<BITS, RT, NTW, ALOADS, A4P>(smem, o1, o0, o2, aE, bE, kb + 1, KB, aptr, aoff, bptr, L, C, bdB, bdA, acc, rd_off, afp);
        const int t0 = o0;      // two blocks done: tiles kb+2, kb+3, kb+4 live in o2, o0, o1
        o0 = o2;
        o2 = o1;
        o1 = t0;
    }
    if (kb < KB)                // odd number of K blocks
        kblock<BITS, RT, NTW, ALOADS, A4P>(smem, o0, o2, o1, aO, bO, kb, KB, aptr, aoff, bptr, L, C, bdA, bdB, acc, rd_off, afp);

    // ---- epilogue: rescale in fp32.  Lane holds column (lane % 16) and rows 4 (lane / 16) + (0..3) of every 16 x 16
    // accumulator tile.
    float wsc[CT], bs[CT];
    int csum[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        int n = n0 + wv * WN + ct * 16 + lane % 16;
        if (n >= N) n = N - 1;
        wsc[ct] = wscale[n];
        bs[ct] = bias ? bias[n] : 0.0f;
        csum[ct] = ZP ? colsum[n] : 0;
    }
    // y of accumulator register x of tile (i, ct); the zero-point form adds zero_t * colsum_n to the integer sum
    // (64-bit: the product can exceed 32 bits)
    auto rescale4 = [&](int i, int ct, float (&y)[4]) {
        const int lr0 = i * 16 + 4 * (lane / 16);
        const float4 s4 = *reinterpret_cast<const float4*>(&sc[lr0]);
        const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
        int zv[4] = {0, 0, 0, 0};
        if constexpr (ZP) {
            const int4 z4 = *reinterpret_cast<const int4*>(&zr[lr0]);
            zv[0] = z4.x; zv[1] = z4.y; zv[2] = z4.z; zv[3] = z4.w;
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int a = acc[i][ct][x];
            const float tot = ZP ? (float)((long long)a + (long long)zv[x] * (long long)csum[ct]) : (float)a;
            y[x] = (tot * sv[x]) * wsc[ct] + bs[ct];
        }
    };
    const int ncol0 = n0 + wv * WN;                 // first column of this wave
    unsigned char* slab = smem + wv * EPI_WAVE;
    if (!out_fp32) {
        // bf16: one 32-row slab (two row tiles) per wave staged in LDS (wave-private, so only wave-level ordering is needed
        // after the K loop's final barrier); every lane then stores 16 contiguous bytes, a row segment of the wave is
        // WN * 2 bytes
        uint16_t* Yh = reinterpret_cast<uint16_t*>(Y);
        const bool vec = N % 8 == 0;                // rows of Y are 16-byte aligned
#pragma unroll
        for (int i2 = 0; i2 < RT / 2; ++i2) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    float y[4];
                    rescale4(2 * i2 + h, ct, y);
                    const unsigned d[2] = {pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        *reinterpret_cast<uint16_t*>(&slab[(16 * h + 4 * (lane / 16) + x) * EPI_ROW + (ct * 16 + lane % 16) * 2]) =
                            (uint16_t)(d[x / 2] >> (16 * (x % 2)));
                }
            wave_sync();
            // 32 rows x (WN * 2) bytes: WN / 8 lanes per row, 16 bytes per lane
            constexpr int LPR = WN / 8, RPP = 64 / LPR;
#pragma unroll
            for (int p = 0; p < 32 / RPP; ++p) {
                const int lr = p * RPP + lane / LPR, cb = (lane % LPR) * 8;   // 8 bf16 per lane
                const uint4 v = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 2]);
                const int row = m0 + i2 * 32 + lr, col = ncol0 + cb;
                if (row < M) {
                    if (vec && col + 8 <= N) {
                        *reinterpret_cast<uint4*>(&Yh[(size_t)row * N + col]) = v;
                    } else {
                        const unsigned e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int x = 0; x < 8; ++x)
                            if (col + x < N) Yh[(size_t)row * N + col + x] = (uint16_t)(e[x / 2] >> (16 * (x % 2)));
                    }
                }
            }
            wave_sync();
        }
    } else {
        // fp32: the same staging, 32 rows x 32 columns at a time
        float* Yf = reinterpret_cast<float*>(Y);
        const bool vec = N % 4 == 0;
#pragma unroll
        for (int i2 = 0; i2 < RT / 2; ++i2)
#pragma unroll
            for (int j = 0; j < NTW; ++j) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        float y[4];
                        rescale4(2 * i2 + h, 2 * j + c, y);
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            *reinterpret_cast<float*>(&slab[(16 * h + 4 * (lane / 16) + x) * EPI_ROW + (c * 16 + lane % 16) * 4]) = y[x];
                    }
                wave_sync();
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int lr = p * 8 + lane / 8, cb = (lane % 8) * 4;    // 4 floats per lane
                    const uint4 v = *reinterpret_cast<const uint4*>(&slab[lr * EPI_ROW + cb * 4]);
                    const int row = m0 + i2 * 32 + lr, col = ncol0 + j * 32 + cb;
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
                wave_sync();
            }
    }
}

template <int BITS, int BM, int NTW>
hipError_t launch(hipStream_t st, const int8_t* q, const float* scale, const int32_t* zero, int M, int K,
                  const lrq_tlq_weight& w, const float* bias, int fp32, void* Y, bool packed4) {
    constexpr int BN = WAVES * 32 * NTW;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (w.N + BN - 1) / BN;
    if (packed4)
        hipLaunchKernelGGL((qgemm_kernel<BITS, BM, NTW, true, true>), dim3(tiles_m * tiles_n), dim3(256), 0, st, q, scale, M, K, w.N,
                           w.gemm_codes, w.lut, w.wscale, bias, fp32, Y, tiles_m, tiles_n, static_cast<const int32_t*>(nullptr),
                           w.colsum, -8);
    else if (zero)
        hipLaunchKernelGGL((qgemm_kernel<BITS, BM, NTW, true>), dim3(tiles_m * tiles_n), dim3(256), 0, st, q, scale, M, K, w.N,
                           w.gemm_codes, w.lut, w.wscale, bias, fp32, Y, tiles_m, tiles_n, zero, w.colsum, 0);
    else
        hipLaunchKernelGGL((qgemm_kernel<BITS, BM, NTW, false>), dim3(tiles_m * tiles_n), dim3(256), 0, st, q, scale, M, K, w.N,
                           w.gemm_codes, w.lut, w.wscale, bias, fp32, Y, tiles_m, tiles_n, zero, w.colsum, 0);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_qgemm(hipStream_t st, const int8_t* q, const float* scale, const int32_t* zero, int M, int K,
                        const lrq_tlq_weight& w, const float* bias, int out_dtype, void* Y, bool packed4) {
    if (packed4 && zero) return hipErrorInvalidValue;
    const int fp32 = out_dtype == LRQ_OUT_FP32;
    // Tile shape.  128 x 256 (two workgroups per CU) is the fastest on long K loops; 128 x 128 (three per CU)
    // hides the prologue / epilogue of short K loops better and wastes less on N that is not a multiple of 256;
    // 64 x 128 serves inputs of a few tokens (conditioning vectors), where taller tiles multiply padding.
    const bool narrow = K <= 2048 || (w.N % 256 != 0 && w.N <= 2048);
    if (M <= 64) {
        if (w.bits == 4) return launch<4, 64, 1>(st, q, scale, zero, M, K, w, bias, fp32, Y, packed4);
        return launch<3, 64, 1>(st, q, scale, zero, M, K, w, bias, fp32, Y, packed4);
    }
    if (narrow) {
        if (w.bits == 4) return launch<4, 128, 1>(st, q, scale, zero, M, K, w, bias, fp32, Y, packed4);
        return launch<3, 128, 1>(st, q, scale, zero, M, K, w, bias, fp32, Y, packed4);
    }
    if (w.bits == 4) return launch<4, 128, 2>(st, q, scale, zero, M, K, w, bias, fp32, Y, packed4);
    return launch<3, 128, 2>(st, q, scale, zero, M, K, w, bias, fp32, Y, packed4);
}

}  // namespace lrq
