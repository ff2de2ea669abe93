// Dense outlier-aware rotation u = x . R (Method, ARS case equation, second branch with R materialised) followed by the
// per-token quantizer, with the bulk of the product on the bf16 matrix cores.
//
// The codes are defined in fp64: u[t, j] = sum over ascending k of x[t, k] R[k, j] (every product of two bf16 values is
// exact, every addition rounds once), amax_t = max_j |u|, code = rint(u * (qmax / amax_t)).  A bf16 MFMA with fp32
// accumulation cannot give u to that accuracy, but it gives an approximation u~ with a bound eps_t on |u~ - u| that holds
// for every element of the row, and almost every rounding decision is already settled by u~:
//   * the row maximum is attained among the elements with |u~| >= max |u~| - 2 eps_t (normally one or two); those are
//     recomputed exactly (the definition's own chain of fused multiply-adds) and give amax_t bit for bit;
//   * an element whose u~ * inv lies farther than eps_t * inv (plus fp64 round-off) from the nearest half-integer rounds to
//     the same code as the exact value; the others (a few per thousand) are recomputed exactly.
// Rows where this does not pay (more uncertain elements than the lists hold: tiny |u| against large |x|) are recomputed
// as a whole.  Nothing depends on how the error is distributed - only on the bound, which is derived below from a
// stated model of the matrix instruction's rounding and checked by a GPU test against the exact values.
//
// Error bound.  A run of m = CHUNK / 16 chained v_mfma_f32_32x32x16_bf16 starts from a zero accumulator.  Model of one
// instruction, D = C + sum_{i<16} a_i b_i: every addend is aligned to the largest one and truncated below 2^-26 of it, the
// sum is rounded or truncated to 24 bits: |D - exact| <= (17 * 2^-26 + 2^-23) * (|C| + sum |a_i b_i|) < ETA * (|C| + sum |a_i b_i|),
// ETA = 2^-21 (measured on this chip: at most 5.8 * 2^-24 over adversarial exponent mixes).  Over a run, |C| is at most
// the sum of |a b| of the run's earlier steps, so the run's error is at most ETA * m * S_run.  GROUP runs are then summed
// in fp32 by ordinary vector additions (round to nearest: each errs by at most 2^-24 of its result, which is at most the
// group's sum of |a b|): (GROUP - 1) * 2^-24 * S_group.  Groups are added to an fp64 accumulator (exact to 2^-53).  In all
//   |u~ - u| <= (ETA * m + (GROUP - 1) * 2^-24) * S,   S = sum_k |x_k| |R_kj|
// (second-order terms are far below the slack with which S itself is evaluated), and S is bounded per row without touching
// R's columns one by one:
//   S <= rho * sqrt(sum_{|x_k| < theta} x_k^2)  +  sum_{|x_k| >= theta} |x_k| * max_j |R_kj|
// (Cauchy-Schwarz on the many small entries, rho = max_j ||R[:, j]||_2; the few large ones - salient channels - term by
// term), theta = 4 * mean |x|.  u~ is stored as fp32: one more rounding, 2^-24 |u~| <= 2^-24 S.
#include "lrq_internal.h"

namespace lrq {
namespace {

constexpr int kWave = 64;
constexpr double kMagic = 6755399441055744.0;   // 1.5 * 2^52: adding it rounds to an integer, ties to even
constexpr int CAPC = 4;                          // amax candidates kept per row
constexpr float kBoundSlack = 1.004f;            // covers the fp32 arithmetic in which the bound itself is evaluated

// Monotone map double -> uint64 (unsigned order = numeric order), so that an unsigned atomic maximum is a maximum of doubles.
// The zero-point form keeps, per row, the key of max u and the key of max (-u); the symmetric form the bits of max |u|.
__device__ __forceinline__ unsigned long long okey(double v) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    return (b >> 63) ? ~b : b | 0x8000000000000000ull;
}
__device__ __forceinline__ double okey_value(unsigned long long k) {
    return __longlong_as_double((long long)((k >> 63) ? k & 0x7fffffffffffffffull : ~k));
}

// The per-token quantizer of a row (Preliminaries, Eq. 1).  Symmetric form: inv = qmax / amax, code = rint(u inv).  Zero-point
// form: range = max - min, L = 2^b - 1, inv = L / range, z = rint(min inv), x_q = clamp(rint(u inv) - z, 0, L), s = range / L,
// stored as q = x_q - 2^(b-1) and zero = z + 2^(b-1); a constant row takes x_q = 0 and (s, z) = (|c|, sign c), (1, 0) for c = 0.
struct RowQuant {
    double inv, zsub;       // code = clamp(rint(u inv) - zsub, -half, half - 1) in the zero-point form
    float scale;
    int izero;
};
template <bool ASYM>
__device__ __forceinline__ RowQuant row_quant(unsigned long long kmax, unsigned long long kmin, double qmax) {
    RowQuant r;
    if constexpr (!ASYM) {
        const double amax = __longlong_as_double((long long)kmax);
        r.inv = amax > 0.0 ? qmax / amax : 0.0;
        r.zsub = 0.0;
        r.scale = (float)(amax / qmax);
        r.izero = 0;
    } else {
        const double L = 2.0 * qmax + 1.0, half = qmax + 1.0;       // qmax = 2^(b-1) - 1
        const double vmax = okey_value(kmax), vmin = -okey_value(kmin), rng = vmax - vmin;
        double sc, z;
        if (rng > 0.0) {
            r.inv = L / rng;
            sc = rng / L;
            z = rint(vmin * r.inv);
            r.zsub = z + half;
        } else {
            r.inv = 0.0;
            sc = vmin != 0.0 ? fabs(vmin) : 1.0;
            z = vmin > 0.0 ? 1.0 : (vmin < 0.0 ? -1.0 : 0.0);
            r.zsub = half;                      // every code is x_q = 0, i.e. q = -2^(b-1)
        }
        r.scale = (float)sc;
        r.izero = (int)(z + half);
    }
    return r;
}
// the code of one exact value (low byte of the result); product, rounding and clamp round separately
template <bool ASYM>
__device__ __forceinline__ int exact_code(double u, const RowQuant& p, double qmax) {
    if constexpr (!ASYM) {
        return __double2loint(u * p.inv + kMagic);
    } else {
        const double r = (u * p.inv + kMagic) - kMagic;
        const double t = fmin(fmax(r - p.zsub, -(qmax + 1.0)), qmax);
        return __double2loint(t + kMagic);
    }
}

typedef short v8s __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ float wave_sumf(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_maxf(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// ---- statistics of a K x K bf16 matrix A, one workgroup per row: maxabs[row] = max_j |A[row, j]| (if maxabs) and
// *sumsq_max = max over rows of sum_j A[row, j]^2 (if sumsq_max; float bits, atomic max - zero it first).  Run on R it
// gives max_j |R_kj| per k; run on R transposed it gives rho^2.  zero_words: the launch on R also clears the scalars.
__global__ __launch_bounds__(256) void matrix_row_stats_kernel(const uint16_t* __restrict__ A, int K, float* __restrict__ maxabs,
                                                               unsigned* __restrict__ sumsq_max, unsigned* __restrict__ zero_words,
                                                               int n_zero) {
    __shared__ float red[8];
    const int t = threadIdx.x, row = blockIdx.x;
    if (zero_words && row == 0 && t < n_zero) zero_words[t] = 0u;
    const uint4* src = reinterpret_cast<const uint4*>(A + (size_t)row * K);
    float mx = 0.0f, ss = 0.0f;
    for (int c = t; c < K / 8; c += 256) {
        const uint4 v = src[c];
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = bf16_lo(w[i]), b = bf16_hi(w[i]);
            mx = fmaxf(mx, fmaxf(fabsf(a), fabsf(b)));
            ss += a * a + b * b;
        }
    }
    mx = wave_maxf(mx);
    ss = wave_sumf(ss);
    if (t % kWave == 0) { red[t / kWave] = mx; red[4 + t / kWave] = ss; }
    __syncthreads();
    if (t == 0) {
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        ss = (red[4] + red[5]) + (red[6] + red[7]);
        if (maxabs) maxabs[row] = mx;
        if (sumsq_max) atomicMax(sumsq_max, __float_as_uint(ss));      // non-negative floats order like their bit patterns
    }
}

// Rt[j, k] = R[k, j], 64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ R, int K, uint16_t* __restrict__ Rt) {
    __shared__ uint16_t tile[64][66];
    const int t = threadIdx.x, k0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    {
        const int r = t / 4, c = (t % 4) * 16;
        const uint4 a = *reinterpret_cast<const uint4*>(R + (size_t)(k0 + r) * K + j0 + c);
        const uint4 b = *reinterpret_cast<const uint4*>(R + (size_t)(k0 + r) * K + j0 + c + 8);
        const unsigned w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            tile[r][c + 2 * i] = (uint16_t)(w[i] & 0xffffu);
            tile[r][c + 2 * i + 1] = (uint16_t)(w[i] >> 16);
        }
    }
    __syncthreads();
    {
        const int r = t / 4, c = (t % 4) * 16;      // output row j0 + r, columns k0 + c ...
        unsigned w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = (unsigned)tile[c + 2 * i][r] | ((unsigned)tile[c + 2 * i + 1][r] << 16);
        uint4* dst = reinterpret_cast<uint4*>(Rt + (size_t)(j0 + r) * K + k0 + c);
        dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
        dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
    }
}

// ---- u~ = x . R on the bf16 matrix cores.  Workgroup = 8 waves (4 x 2), tile 128 tokens x 128 columns, wave tile
// 32 x 64 (two 32 x 32 accumulator tiles).  Both operand tiles (x rows and R columns, i.e. rows of Rt) go global ->
// registers -> LDS: stage s is loaded two iterations before it is stored to one of three LDS buffers and three before
// it is multiplied.  LDS rows are padded to 144 bytes so that the 16-byte fragment reads of 16 consecutive rows fall
// on distinct banks.
// Accumulation has three levels.  A run of CHUNK = 32 k (half a stage) is two chained matrix instructions that start on
// a zero accumulator (the instruction's constant-zero addend, no clearing).  The fp32 tiles of a finished run are
// added - one vector fp32 addition per value, rounded to nearest, eight times more accurate than the addition inside
// the matrix instruction - to fp32 group tiles, GROUP = 8 runs (256 k) to a group, and a finished group is added to the
// fp64 tiles.  These additions are spread between the matrix instructions of the following steps, so they issue while
// the matrix cores work; the conversion to fp64 (the expensive part: twelve issue cycles per value against eight
// cycles of matrix work per value and 64 k) happens once per group only.
// Besides u~ the kernel writes, per row and 64-column segment (a wave's width), the maximum of |u~| (segmax): the
// search for the row maximum then reads one value per segment instead of the whole row.
// (X, Rt and Ut are deliberately not declared __restrict__: with that promise the compiler moves the prefetch loads past
// the compiler barrier that keeps them ahead of the arithmetic, down to their LDS stores.)
constexpr int DT_M = 128, DT_N = 128, DT_K = 64, DT_ROW = 144, DT_BUF = DT_M * DT_ROW;
constexpr int DT_SEG = 64;          // columns per segment maximum
constexpr int kChunk = 32;          // run length of the fp32 accumulation inside the matrix instruction
constexpr int kGroup = 8;           // runs per fp32 group sum

// fragments of one 16-k step of a wave: its 32 rows of the x tile, columns 0..31 and 32..63 of its R tile
__device__ __forceinline__ void read_fragments(const unsigned char* A, const unsigned char* B, int s, v8s (&f)[3]) {
    f[0] = *reinterpret_cast<const v8s*>(A + s * 32);
    f[1] = *reinterpret_cast<const v8s*>(B + s * 32);
    f[2] = *reinterpret_cast<const v8s*>(B + 32 * DT_ROW + s * 32);
}
// One stage = two runs of CHUNK = 32 k: steps 0, 1 accumulate into fresh fp32 tiles A, steps 2, 3 into fresh tiles B.
// The bookkeeping of finished runs is spread between the matrix instructions, eight values after each: during steps 0, 1
// the B tiles of the previous stage (`prev`) are added to the group tiles and, if they close a group (FLUSH), the group
// tiles join the fp64 tiles; during steps 2, 3 this stage's A tiles are added to the group tiles or, if they open a
// group (FIRST), replace them.
// The fragments of step s + 1 are read from LDS before the matrix instructions of step s are issued (LDS latency is
// longer than a matrix instruction); fr holds those of step 0 on entry and those of the next stage's step 0 (buffer
// An / Bn, complete since the previous barrier) on return.
// The staged registers st (this thread's four 16-byte pieces of the stage that is two ahead) go to LDS one per step, at
// dst[i], and are reloaded from byte offset src[i] + goff_x of x (i < 2) or src[i] + goff_r of Rt (the stage that is four
// ahead; 32-bit offsets, taken modulo 2^32: both arrays are smaller than 4 GiB) right away: spread like this the LDS writes of
// the eight waves overlap the matrix work instead of preceding it.
template <bool FIRST, bool FLUSH>
__device__ __forceinline__ void multiply_stage(const unsigned char* A, const unsigned char* B, const unsigned char* An,
                                               const unsigned char* Bn, v8s (&fr)[3], v4u (&st)[4], unsigned char* const (&dst)[4],
                                               const unsigned char* xb, const unsigned char* rb, const unsigned (&src)[4],
                                               unsigned goff_x, unsigned goff_r, double (&wide)[2][16], v16f (&group)[2],
                                               v16f (&prev)[2]) {
    static_assert(DT_K == 2 * kChunk && kChunk == 32, "two runs of two matrix instructions per stage");
    const v16f zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    v16f ta[2], tb[2];
    v8s fo[3];                       // fragments of the odd steps
#pragma unroll
    for (int s = 0; s < DT_K / 16; ++s) {
        if (s % 2 == 0) read_fragments(A, B, s + 1, fo);
        else if (s + 1 < DT_K / 16) read_fragments(A, B, s + 1, fr);
        else read_fragments(An, Bn, 0, fr);
        *reinterpret_cast<v4u*>(dst[s]) = st[s];
        st[s] = *reinterpret_cast<const v4u*>((s < 2 ? xb : rb) + (size_t)(src[s] + (s < 2 ? goff_x : goff_r)));
        asm volatile("" ::: "memory");                   // keeps the load here, ahead of the arithmetic that follows
        __builtin_amdgcn_sched_barrier(0);
        const v8s a = s % 2 == 0 ? fr[0] : fo[0];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const v8s b = s % 2 == 0 ? fr[1 + j] : fo[1 + j];
            if (s == 0) ta[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, zero, 0, 0, 0);
            if (s == 1) ta[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, ta[j], 0, 0, 0);
            if (s == 2) tb[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, zero, 0, 0, 0);
            if (s == 3) tb[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, tb[j], 0, 0, 0);
            // slot 0..3 of this half of the stage: tile slot / 2, values 8 (slot % 2) ... + 7 (tile 0 first: its last
            // matrix instruction was issued before tile 1's)
            const int slot = 2 * (s % 2) + j, tile = slot / 2;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int r = 8 * (slot % 2) + i;
                if (s < 2) {
                    const float g = group[tile][r] + prev[tile][r];
                    group[tile][r] = g;
                    if (FLUSH) wide[tile][r] += (double)g;
                } else {
                    group[tile][r] = FIRST ? ta[tile][r] : group[tile][r] + ta[tile][r];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    prev[0] = tb[0];
    prev[1] = tb[1];
}

// Maximum over the 32 lanes of a half-wave of 16 values per lane: one full exchange, then exchanges that halve the number
// of values a lane carries (the lane with bit W set keeps the upper W values, its partner the lower ones); lane l ends
// with value number l % 16 (the return value).  (The halving width is a template parameter: with a loop variable the
// register array would be indexed dynamically, i.e. through chains of compares and selects.)
template <int W>
__device__ __forceinline__ void halve_exchange(float (&vals)[16], int lane) {
    const bool up = (lane & W) != 0;
#pragma unroll
    for (int h = 0; h < W; ++h) {
        const float keep = up ? vals[h + W] : vals[h];
        const float send = up ? vals[h] : vals[h + W];
        vals[h] = fmaxf(keep, __shfl_xor(send, W, kWave));
    }
}
__device__ __forceinline__ float half_wave_max16(float (&vals)[16], int lane) {
#pragma unroll
    for (int r = 0; r < 16; ++r) vals[r] = fmaxf(vals[r], __shfl_xor(vals[r], 16, kWave));
    halve_exchange<8>(vals, lane);
    halve_exchange<4>(vals, lane);
    halve_exchange<2>(vals, lane);
    halve_exchange<1>(vals, lane);
    return vals[0];
}

// Tile order: ids go round-robin over the 8 XCDs; each XCD walks a contiguous range of an order that keeps 8 row tiles
// together and runs over the column tiles fastest, so that an XCD's L2 sees each x panel and each R panel several times
// in a row.  id -> first row and first column of the tile.
struct TileOrigin {
    int m0, n0;
};
__device__ __forceinline__ TileOrigin tile_origin(int id, int tiles_m, int tiles_n) {
    const int ntiles = tiles_m * tiles_n;
    const int x = id % 8, i = id / 8;
    const int base = ntiles / 8, rem = ntiles % 8;
    const int tile = x * base + (x < rem ? x : rem) + i;
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = tile / per_group, first_m = group * GM;
    const int gsize = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    const int r = tile % per_group;
    TileOrigin o;
    o.m0 = (first_m + r % gsize) * DT_M;
    o.n0 = (r / gsize) * DT_N;
    return o;
}
// this thread's four load streams of a tile (rows r0 and r0 + 64 of the x tile and of the R tile)
// as byte offsets into x (the first two) and Rt (M K < 2^31 and K <= 16384: they fit 32 bits)
__device__ __forceinline__ void tile_sources(int M, int K, TileOrigin o, int r0, int cc, unsigned (&src)[4]) {
    int g0 = o.m0 + r0, g1 = o.m0 + r0 + 64;
    if (g0 >= M) g0 = M - 1;
    if (g1 >= M) g1 = M - 1;
    src[0] = ((unsigned)g0 * (unsigned)K) * 2u + cc * 16;
    src[1] = ((unsigned)g1 * (unsigned)K) * 2u + cc * 16;
    src[2] = ((unsigned)(o.n0 + r0) * (unsigned)K) * 2u + cc * 16;
    src[3] = ((unsigned)(o.n0 + r0 + 64) * (unsigned)K) * 2u + cc * 16;
}

// The workgroups are persistent: workgroup b takes the tiles b, b + gridDim.x, ... (gridDim.x a multiple of 8 whenever a
// workgroup has more than one tile, so that it stays on its XCD's range).  The operand pipeline does not drain between
// tiles: the loads that would run past the end of a tile's K fetch the first four stages of the workgroup's next tile, so
// that tile starts with two stages in LDS and two in registers, as the prologue leaves the first one (K >= 256; a tile
// of two stages runs the prologue again).
// ASYM (zero-point form of the quantizer): the segment values are max u~ and, in the second half of segmax, max (-u~)
// instead of max |u~|.
template <bool ASYM>
__global__ __launch_bounds__(512, 2) void dense_rotate_bf16_kernel(const uint16_t* X, const uint16_t* Rt, int M, int K, float* Ut,
                                                                    float* segmax, int tiles_m, int tiles_n) {
    __shared__ __attribute__((aligned(16))) unsigned char As[3 * DT_BUF];
    __shared__ __attribute__((aligned(16))) unsigned char Bs[3 * DT_BUF];
    const int ntiles = tiles_m * tiles_n;
    const int t = threadIdx.x, lane = t % kWave, wv = t / kWave;
    const int wm = wv / 2, wn = wv % 2;
    // loader: 1024 16-byte pieces per operand tile and stage, two per thread and operand (rows r0 and r0 + 64)
    const int r0 = t / 8, cc = t % 8;
    const int d0 = r0 * DT_ROW + cc * 16, d1 = d0 + 64 * DT_ROW;
    const int nk = K / DT_K;
    const bool chained = nk >= 4;                        // the next tile's first stages ride in this tile's pipeline
    const int a_off = (wm * 32 + lane % 32) * DT_ROW + (lane / 32) * 16;
    const int b_off = (wn * 64 + lane % 32) * DT_ROW + (lane / 32) * 16;

    int id = blockIdx.x;
    TileOrigin cur = tile_origin(id, tiles_m, tiles_n);
    const unsigned char* xb = reinterpret_cast<const unsigned char*>(X);
    const unsigned char* rb = reinterpret_cast<const unsigned char*>(Rt);
    unsigned src[4];
    tile_sources(M, K, cur, r0, cc, src);
    v4u ev[4], od[4];
    v8s fr[3];
    int b0 = 0, b1 = 1, b2 = 2;                          // LDS buffers of stages kb, kb + 1, kb + 2
    bool primed = false;                                 // stages 0, 1 in LDS, 2, 3 in registers, fragments of stage 0 read
    for (;;) {
        const bool has_next = id + (int)gridDim.x < ntiles;
        const TileOrigin nto = tile_origin(has_next ? id + (int)gridDim.x : id, tiles_m, tiles_n);
        // the next tile's streams are this tile's shifted by a uniform amount (modulo 2^32) unless one of the two tiles is cut
        // by the end of the matrix (clamped rows): such a transition is not chained, the next tile runs the prologue
        const bool link = chained && has_next && cur.m0 + DT_M <= M && nto.m0 + DT_M <= M;
        const unsigned to_next_x = (unsigned)(nto.m0 - cur.m0) * (unsigned)K * 2u, to_next_r = (unsigned)(nto.n0 - cur.n0) * (unsigned)K * 2u;
        // offsets of the stages past this tile's end (selected by masks, not branches: the loop body stays one block);
        // a transition that is not chained re-reads this tile's last stage, which is harmless
        const unsigned next_x = link ? to_next_x : (unsigned)(nk - 1) * DT_K * 2, next_r = link ? to_next_r : (unsigned)(nk - 1) * DT_K * 2;
        const unsigned next_step = link ? DT_K * 2 : 0;
        if (!primed) {
            // prologue: stages 0, 1 in LDS buffers b0, b1; stages 2 (even) and 3 (odd) in registers (a tile of two stages
            // re-reads its last one: harmless, never multiplied)
            const unsigned o1 = (unsigned)(nk > 1 ? 1 : 0) * DT_K * 2, o2 = (unsigned)(nk > 2 ? 2 : nk - 1) * DT_K * 2,
                           o3 = (unsigned)(nk > 3 ? 3 : nk - 1) * DT_K * 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ev[i] = *reinterpret_cast<const v4u*>((i < 2 ? xb : rb) + (size_t)src[i]);
                od[i] = *reinterpret_cast<const v4u*>((i < 2 ? xb : rb) + (size_t)(src[i] + o1));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                unsigned char* base = i < 2 ? As : Bs;
                const int d = i % 2 == 0 ? d0 : d1;
                *reinterpret_cast<v4u*>(&base[b0 * DT_BUF + d]) = ev[i];
                *reinterpret_cast<v4u*>(&base[b1 * DT_BUF + d]) = od[i];
                ev[i] = *reinterpret_cast<const v4u*>((i < 2 ? xb : rb) + (size_t)(src[i] + o2));
                od[i] = *reinterpret_cast<const v4u*>((i < 2 ? xb : rb) + (size_t)(src[i] + o3));
            }
            __syncthreads();
            read_fragments(&As[b0 * DT_BUF + a_off], &Bs[b0 * DT_BUF + b_off], 0, fr);
        }

        double wide[2][16];
        v16f group[2], prev[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                wide[j][r] = 0.0;
                group[j][r] = 0.0f;
                prev[j][r] = 0.0f;
            }
        // A group is the eight runs of four stages: stage 4 i opens group i with its first run (FIRST) and, before that,
        // adds the last run of stage 4 i - 1 to group i - 1 and flushes it (FLUSH).  Stage 0 has nothing to flush: it
        // "flushes" the zero-initialised tiles, which changes nothing.
        static_assert(kGroup == 8 && 2 * kChunk == DT_K, "the loop body below is written out for groups of four stages");
        // Two stages: the first multiplies from b0 and refills b2 from the even registers (stage KB + 2, loaded two
        // iterations ago; they then take stage KB + 4), the second multiplies from b1 and refills b0, the buffer that stage
        // KB just left, from the odd ones.  Stage s >= nk is stage s - nk of the next tile (a transition that is not chained:
        // a harmless re-read of this tile's last stage).  (A macro, not a lambda: captured register arrays would be spilled to
        // scratch memory.)
#define LRQ_DENSE_LOAD_FROM(S, OX, OR)                                                                                    \
        const unsigned past_##OX = 0u - (unsigned)((S) >= nk);             /* all ones: the stage belongs to the next tile */ \
        const unsigned in_##OX = (unsigned)(S) * DT_K * 2, step_##OX = (unsigned)((S) - nk) * next_step;                   \
        const unsigned OX = (in_##OX & ~past_##OX) | ((next_x + step_##OX) & past_##OX);                                   \
        const unsigned OR = (in_##OX & ~past_##OX) | ((next_r + step_##OX) & past_##OX);
#define LRQ_DENSE_STAGE_PAIR(FIRST_A, FLUSH_A, FIRST_B, FLUSH_B, KB)                                                     \
        {                                                                                                                 \
            unsigned char* const dst_a[4] = {&As[b2 * DT_BUF + d0], &As[b2 * DT_BUF + d1], &Bs[b2 * DT_BUF + d0],         \
                                             &Bs[b2 * DT_BUF + d1]};                                                      \
            LRQ_DENSE_LOAD_FROM((KB) + 4, oax, oar)                                                                       \
            multiply_stage<FIRST_A, FLUSH_A>(&As[b0 * DT_BUF + a_off], &Bs[b0 * DT_BUF + b_off], &As[b1 * DT_BUF + a_off], \
                                             &Bs[b1 * DT_BUF + b_off], fr, ev, dst_a, xb, rb, src, oax, oar, wide, group, prev); \
            __builtin_amdgcn_sched_barrier(0);                                                                            \
            __syncthreads();                                                                                              \
            unsigned char* const dst_b[4] = {&As[b0 * DT_BUF + d0], &As[b0 * DT_BUF + d1], &Bs[b0 * DT_BUF + d0],         \
                                             &Bs[b0 * DT_BUF + d1]};                                                      \
            LRQ_DENSE_LOAD_FROM((KB) + 5, obx, obr)                                                                       \
            multiply_stage<FIRST_B, FLUSH_B>(&As[b1 * DT_BUF + a_off], &Bs[b1 * DT_BUF + b_off], &As[b2 * DT_BUF + a_off], \
                                             &Bs[b2 * DT_BUF + b_off], fr, od, dst_b, xb, rb, src, obx, obr, wide, group, prev); \
            __builtin_amdgcn_sched_barrier(0);                                                                            \
            __syncthreads();                                                                                              \
            const int f = b0;                            /* stages KB + 2, KB + 3, KB + 4 live in b2, b0, b1 */           \
            b0 = b2;                                                                                                      \
            b2 = b1;                                                                                                      \
            b1 = f;                                                                                                       \
        }
        int kb = 0;
        for (; kb + 3 < nk; kb += 4) {
            LRQ_DENSE_STAGE_PAIR(true, true, false, false, kb)
            LRQ_DENSE_STAGE_PAIR(false, false, false, false, kb + 2)
        }
        if (kb < nk) LRQ_DENSE_STAGE_PAIR(true, true, false, false, kb)      // K % 256 == 128: two more stages
#undef LRQ_DENSE_STAGE_PAIR
#undef LRQ_DENSE_LOAD_FROM
        // the last run, and what its group holds
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) wide[j][r] += (double)(group[j][r] + prev[j][r]);

        // lane holds column (lane % 32) and rows 8 (r / 4) + 4 (lane / 32) + r % 4 of each 32 x 32 accumulator tile
        const int m0 = cur.m0, n0 = cur.n0;
        float vals[16], neg[16];                         // per row that this lane touches: max over its two columns
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
            const float u0 = (float)wide[0][r], u1 = (float)wide[1][r];
            if (row < M) {
                float* dst = Ut + (size_t)row * K + n0 + wn * 64 + lane % 32;
                dst[0] = u0;
                dst[32] = u1;
            }
            vals[r] = ASYM ? fmaxf(u0, u1) : fmaxf(fabsf(u0), fabsf(u1));
            neg[r] = ASYM ? fmaxf(-u0, -u1) : 0.0f;
        }
        const float hi = half_wave_max16(vals, lane);
        const float lo = ASYM ? half_wave_max16(neg, lane) : 0.0f;
        if ((lane & 16) == 0) {
            const int r = lane % 16;
            const int row = m0 + wm * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
            if (row < M) {
                const size_t at = (size_t)row * (K / DT_SEG) + (n0 + wn * 64) / DT_SEG;
                segmax[at] = hi;
                if (ASYM) segmax[(size_t)M * (K / DT_SEG) + at] = lo;
            }
        }
        if (!has_next) break;
        id += (int)gridDim.x;
        cur = nto;
        tile_sources(M, K, cur, r0, cc, src);
        primed = link;           // chained: the pipeline already holds the next tile's first four stages
    }
}

// ---- per row (one wave each): the bound eps_t, then the candidates for the row maximum, found from the segment maxima
// (only the segments that reach the limit are read from u~).
// mode[row] = 1 marks a row that is recomputed as a whole (more candidates than the list holds).
// RES: K <= 4096, the row of x stays in registers between the passes (it is read once).
// ASYM (zero-point form): two searches, for the row's maximum (side 0) and for its minimum (side 1, on the maxima of -u~
// in the second half of segmax); ccount [M, 2] and cidx [M, 2, CAPC] hold both, amax_bits [M, 2] is cleared for both.
// The symmetric form uses side 0 only (same strides).
template <bool RES, bool ASYM>
__global__ __launch_bounds__(256) void dense_row_candidates_kernel(const uint16_t* __restrict__ X, const float* __restrict__ Ut,
                                                                   const float* __restrict__ segmax, int M, int K,
                                                                   const float* __restrict__ rowmaxR,
                                                                   const unsigned* __restrict__ rho2_bits, float err_factor,
                                                                   double* __restrict__ eps, unsigned long long* __restrict__ amax_bits,
                                                                   int* __restrict__ ccount, uint16_t* __restrict__ cidx,
                                                                   int* __restrict__ mode) {
    constexpr int NX = RES ? 8 : 1;
    const int lane = threadIdx.x % kWave, row = blockIdx.x * 4 + threadIdx.x / kWave;
    if (row >= M) return;
    const uint4* xs = reinterpret_cast<const uint4*>(X + (size_t)row * K);
    const int nxc = K / 8, nseg = K / DT_SEG;
    uint4 xr[NX];
    if constexpr (RES) {
#pragma unroll
        for (int i = 0; i < NX; ++i) xr[i] = lane + kWave * i < nxc ? xs[lane + kWave * i] : make_uint4(0u, 0u, 0u, 0u);
    }
    auto xchunk = [&](int i, int c) { return RES ? xr[i] : xs[c]; };
    const int xiters = RES ? NX : (nxc + kWave - 1) / kWave;

    float s1 = 0.0f;
#pragma unroll
    for (int i = 0; i < xiters; ++i) {
        const int c = lane + kWave * i;
        if (c < nxc) {
            const uint4 v = xchunk(RES ? i : 0, c);
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) s1 += fabsf(bf16_lo(w[d])) + fabsf(bf16_hi(w[d]));
        }
    }
    s1 = wave_sumf(s1);
    const float theta = 4.0f * s1 / (float)K;
    float small2 = 0.0f, big = 0.0f;
#pragma unroll
    for (int i = 0; i < xiters; ++i) {
        const int c = lane + kWave * i;
        if (c < nxc) {
            const uint4 v = xchunk(RES ? i : 0, c);
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
            const float4 r0 = reinterpret_cast<const float4*>(rowmaxR)[2 * c], r1 = reinterpret_cast<const float4*>(rowmaxR)[2 * c + 1];
            const float rm[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float a = fabsf(bf16_lo(w[d])), b = fabsf(bf16_hi(w[d]));
                if (a >= theta) big += a * rm[2 * d]; else small2 += a * a;
                if (b >= theta) big += b * rm[2 * d + 1]; else small2 += b * b;
            }
        }
    }
    small2 = wave_sumf(small2);
    big = wave_sumf(big);
    const float rho = sqrtf(__uint_as_float(*rho2_bits)) * kBoundSlack;
    const float S = (rho * sqrtf(small2) * kBoundSlack + big) * kBoundSlack;       // >= sum_k |x_k| |R_kj| for every j
    const double e = (double)S * (double)err_factor;
    // row maximum of |u~| (zero-point form: maximum and minimum of u~) and the elements within 2 eps of it
    int whole = 0, cnt[2] = {0, 0};
    const float* ur = Ut + (size_t)row * K;
#pragma unroll
    for (int side = 0; side < (ASYM ? 2 : 1); ++side) {
        const float* sm = segmax + (size_t)side * M * nseg + (size_t)row * nseg;
        float mx = -INFINITY;
        for (int c = lane; c < nseg; c += kWave) mx = fmaxf(mx, sm[c]);
        mx = wave_maxf(mx);
        int n = 0;
        if (S > 0.0f && !whole) {                // otherwise x is all zero (or not finite) and there is nothing to decide
            const float lf = (float)((double)mx - 2.0 * e);
            const float lim = lf - fabsf(lf) * 1e-6f;                                  // rounded down: never misses a candidate
            for (int base = 0; base < nseg && !whole; base += kWave) {
                const int c = base + lane;
                unsigned long long segs = __ballot(c < nseg && sm[c] >= lim);        // segments that hold a candidate
                while (segs && !whole) {
                    const int seg = base + __ffsll((long long)segs) - 1;
                    segs &= segs - 1;
                    const float v = ur[seg * DT_SEG + lane];
                    const bool hit = (ASYM ? (side == 0 ? v : -v) : fabsf(v)) >= lim;
                    const unsigned long long hits = __ballot(hit);
                    const int k = __popcll(hits);
                    if (n + k > CAPC) {
                        whole = 1;
                    } else {
                        if (hit) cidx[((size_t)row * 2 + side) * CAPC + n + __popcll(hits & ((1ull << lane) - 1ull))] = (uint16_t)(seg * DT_SEG + lane);
                        n += k;
                    }
                }
            }
        }
        cnt[side] = n;
    }
    if (whole) cnt[0] = cnt[1] = 0;
    if (lane == 0) {
        eps[row] = e;
        // no search (all-zero row): u is 0 everywhere
        const bool zero_row = !(S > 0.0f);
        amax_bits[2 * (size_t)row] = ASYM && zero_row ? okey(0.0) : 0ull;
        amax_bits[2 * (size_t)row + 1] = ASYM && zero_row ? okey(0.0) : 0ull;
        ccount[2 * (size_t)row] = cnt[0];
        ccount[2 * (size_t)row + 1] = cnt[1];
        mode[row] = whole;
    }
}

// ---- the definition's chain for single elements: u = sum over ascending k of x[row, k] * R[k, col], one fused
// multiply-add per term (the products are exact).  Every lane of a wave owns one element, but the wave fetches the
// operands together: in one load instruction eight neighbouring lanes read the eight 16-byte pieces of one element's
// next 128 bytes (64 k) of its x row / R column (Rt holds R's columns contiguously), so every cache line is requested
// once and used in full - a lane reading its own stream 16 bytes at a time asks for each line eight times over and the
// chain then runs at a tenth of its arithmetic rate.  The pieces go through a wave-private LDS buffer (element rows
// padded to 144 bytes: conflict-free 16-byte reads) to the lane that owns the element; the loads of the next 64 k are
// in flight while the current ones are summed.
constexpr int XE_ROW = 144, XE_BUF = 64 * XE_ROW;        // one operand's staging buffer of a wave (9216 bytes)

__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

struct Pieces {
    v4u x[8], r[8];
};
// (xp / rp are not __restrict__: see dense_rotate_bf16_kernel)
__device__ __forceinline__ Pieces load_pieces(const unsigned char* const (&xp)[8], const unsigned char* const (&rp)[8], size_t off) {
    Pieces p;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        p.x[q] = *reinterpret_cast<const v4u*>(xp[q] + off);
        p.r[q] = *reinterpret_cast<const v4u*>(rp[q] + off);
    }
    return p;
}

// All 64 lanes must call this together (lanes without an element pass any valid row / col and ignore the result).
// K % 64 == 0.  lds: this wave's 2 * XE_BUF bytes.
// XDIRECT: every lane reads its own x row itself, 16 bytes at a time, and only the R columns go through LDS - for waves whose
// neighbouring lanes share rows (the list of undecided elements keeps a row's entries together, about nine to a row at
// config 4): lanes with the same address are served by one request, so the cooperative fetch buys nothing for x there
// and its trip through LDS is half of the kernel's LDS traffic.
template <bool XDIRECT>
__device__ __forceinline__ double exact_element_wave(const uint16_t* X, const uint16_t* Rt, int K, int row, int col,
                                                     unsigned char* lds) {
    const int lane = threadIdx.x % kWave;
    const unsigned char* xp[8];
    const unsigned char* rp[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int e = 8 * q + lane / 8;                 // the element whose piece (lane % 8) this lane fetches in load q
        const int er = __shfl(row, e, kWave), ec = __shfl(col, e, kWave);
        xp[q] = XDIRECT ? reinterpret_cast<const unsigned char*>(X + (size_t)row * K) + q * 16
                        : reinterpret_cast<const unsigned char*>(X + (size_t)er * K) + (lane % 8) * 16;
        rp[q] = reinterpret_cast<const unsigned char*>(Rt + (size_t)ec * K) + (lane % 8) * 16;
    }
    unsigned char* xs = lds;
    unsigned char* rs = lds + XE_BUF;
    const int wr = (lane / 8) * XE_ROW + (lane % 8) * 16;        // + 8 q rows for load q
    const int rd = lane * XE_ROW;
    const int nb = K / 64;
    double u = 0.0;
    Pieces nxt = load_pieces(xp, rp, 0);
    for (int b = 0; b < nb; ++b) {
        // stage batch b (the previous batch was read into registers before this point)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (!XDIRECT) *reinterpret_cast<v4u*>(xs + wr + 8 * q * XE_ROW) = nxt.x[q];
            *reinterpret_cast<v4u*>(rs + wr + 8 * q * XE_ROW) = nxt.r[q];
        }
        v4u xv[8], rv[8];
        if (XDIRECT) {
#pragma unroll
            for (int i = 0; i < 8; ++i) xv[i] = nxt.x[i];
        }
        wave_lds_sync();
        nxt = load_pieces(xp, rp, (size_t)(b + 1 < nb ? b + 1 : b) * 128);     // past the end: a harmless re-read
        asm volatile("" ::: "memory");                   // keeps these loads ahead of the arithmetic below
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (!XDIRECT) xv[i] = *reinterpret_cast<const v4u*>(xs + rd + i * 16);
            rv[i] = *reinterpret_cast<const v4u*>(rs + rd + i * 16);
        }
        wave_lds_sync();                                 // the reads are issued before the next batch is staged
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                u = fma((double)bf16_lo(xv[i][d]), (double)bf16_lo(rv[i][d]), u);
                u = fma((double)bf16_hi(xv[i][d]), (double)bf16_hi(rv[i][d]), u);
            }
        __builtin_amdgcn_sched_barrier(0);
    }
    return u;
}

// amax candidates: thread i -> slot i / M of row i % M (slot 0 of every row first, so that the waves are full); the
// zero-point form runs the slots of side 0 (maximum), then those of side 1 (minimum, kept as the maximum of -u).
template <bool ASYM>
__global__ __launch_bounds__(256) void dense_exact_amax_kernel(const uint16_t* X, const uint16_t* Rt, int M, int K,
                                                               const int* __restrict__ ccount, const uint16_t* __restrict__ cidx,
                                                               unsigned long long* __restrict__ amax_bits) {
    __shared__ __attribute__((aligned(16))) unsigned char stage[4 * 2 * XE_BUF];
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    int row = 0, col = 0, side = 0;
    bool have = false;
    if (i < (long)M * CAPC * (ASYM ? 2 : 1)) {
        side = (int)(i / ((long)M * CAPC));
        const long j = i - (long)side * M * CAPC;
        const int slot = (int)(j / M);
        row = (int)(j % M);
        have = slot < ccount[2 * (size_t)row + side];
        col = have ? (int)cidx[((size_t)row * 2 + side) * CAPC + slot] : 0;
    }
    if (__ballot(have) == 0ull) return;                  // nothing in this wave
    const double u = exact_element_wave<false>(X, Rt, K, row, col, stage + (threadIdx.x / kWave) * 2 * XE_BUF);
    if (have) {
        if constexpr (ASYM) atomicMax(&amax_bits[2 * (size_t)row + side], okey(side == 0 ? u : -u));
        else atomicMax(&amax_bits[2 * (size_t)row], (unsigned long long)__double_as_longlong(fabs(u)));
    }
}

// ---- codes from u~ with the exact amax (zero-point form: the exact maximum and minimum); the elements the bound leaves
// undecided go to the row's list (one wave per row)
template <bool ASYM>
__global__ __launch_bounds__(256) void dense_quant_flag_kernel(const float* __restrict__ Ut, int M, int K, double qmax,
                                                               const double* __restrict__ eps,
                                                               const unsigned long long* __restrict__ amax_bits,
                                                               int8_t* __restrict__ q, float* __restrict__ scale,
                                                               int32_t* __restrict__ zero, int* __restrict__ fcount,
                                                               uint16_t* __restrict__ fidx, int capf, int* __restrict__ mode) {
    extern __shared__ int lds_cnt[];            // one counter per wave
    const int wv = threadIdx.x / kWave, lane = threadIdx.x % kWave, row = blockIdx.x * 4 + wv;
    if (lane == 0) lds_cnt[wv] = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (row >= M) return;
    if (mode[row]) {                            // recomputed as a whole later
        if (lane == 0) fcount[row] = 0;
        return;
    }
    const RowQuant rq = row_quant<ASYM>(amax_bits[2 * (size_t)row], amax_bits[2 * (size_t)row + 1], qmax);
    const double inv = rq.inv;
    const double delta = eps[row] * inv * (1.0 + 1e-6) + 1e-12;
    const double keep = 0.5 - delta;            // |p - rint(p)| below this: the code is settled
    const float4* us = reinterpret_cast<const float4*>(Ut + (size_t)row * K);
    uint16_t* myidx = fidx + (size_t)row * capf;
    for (int c = lane; c < K / 8; c += kWave) {
        const float4 v0 = us[2 * c], v1 = us[2 * c + 1];
        const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        unsigned b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double p = (double)v[i] * inv;
            double r = (p + kMagic) - kMagic;
            if (!(fabs(p - r) < keep)) {
                const int slot = atomicAdd(&lds_cnt[wv], 1);
                if (slot < capf) myidx[slot] = (uint16_t)(c * 8 + i);
            }
            r = ASYM ? fmin(fmax(r - rq.zsub, -(qmax + 1.0)), qmax) : fmin(fmax(r, -qmax), qmax);
            b[i] = (unsigned)__double2loint(r + kMagic) & 0xffu;
        }
        *reinterpret_cast<uint2*>(q + (size_t)row * K + (size_t)c * 8) =
            make_uint2(b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24), b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) {
        const int n = lds_cnt[wv];
        scale[row] = rq.scale;
        if (ASYM) zero[row] = rq.izero;
        if (n > capf) {
            mode[row] = 1;
            fcount[row] = 0;
        } else {
            fcount[row] = n;
        }
    }
}

// ---- exclusive prefix sum of the per-row counts, offs[0 .. M] (one workgroup of 1024 threads; 16384 counts per pass
// through LDS so that global reads and writes are coalesced; a thread sums its 16 counts, the sums are scanned inside
// each wave with lane shifts and the 16 wave totals by every thread itself: three barriers per pass)
__global__ __launch_bounds__(1024) void dense_scan_counts_kernel(const int* __restrict__ cnt, int M, int* __restrict__ offs) {
    __shared__ int buf[16384];
    __shared__ int wave_total[16];
    const int t = threadIdx.x, lane = t % kWave, wv = t / kWave;
    int carry = 0;
    for (int base = 0; base < M; base += 16384) {
        for (int i = t; i < 16384; i += 1024) buf[i] = base + i < M ? cnt[base + i] : 0;
        __syncthreads();
        int s = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += buf[t * 16 + i];
        int incl = s;                                   // inclusive scan of s over the wave
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int v = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += v;
        }
        if (lane == kWave - 1) wave_total[wv] = incl;
        __syncthreads();
        int before = 0, all = 0;                        // totals of the waves before this one, and of all 16
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int v = wave_total[w];
            if (w < wv) before += v;
            all += v;
        }
        int run = carry + before + incl - s;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int c = buf[t * 16 + i];
            buf[t * 16 + i] = run;
            run += c;
        }
        carry += all;
        __syncthreads();
        for (int i = t; i < 16384; i += 1024)
            if (base + i < M) offs[base + i] = buf[i];
    }
    if (t == 0) offs[M] = carry;
}

// ---- undecided elements: exact value, exact code.  Thread i takes list entry i (row found by bisection of offs).
template <bool ASYM>
__global__ __launch_bounds__(256) void dense_exact_codes_kernel(const uint16_t* X, const uint16_t* Rt, int M, int K, double qmax,
                                                                const int* __restrict__ offs, const uint16_t* __restrict__ fidx,
                                                                int capf, const unsigned long long* __restrict__ amax_bits,
                                                                int8_t* __restrict__ q) {
    __shared__ __attribute__((aligned(16))) unsigned char stage[4 * 2 * XE_BUF];
    const int total = offs[M];
    const int lane = threadIdx.x % kWave;
    for (int base = blockIdx.x * 256 + (threadIdx.x - lane); base < total; base += gridDim.x * 256) {     // wave-uniform
        const int i = base + lane;
        const bool have = i < total;
        int row = 0, col = 0;
        if (have) {
            int lo = 0, hi = M;                         // largest row with offs[row] <= i
            while (hi - lo > 1) {
                const int mid = (lo + hi) / 2;
                if (offs[mid] <= i) lo = mid; else hi = mid;
            }
            row = lo;
            col = (int)fidx[(size_t)row * capf + (i - offs[row])];
        }
        const double u = exact_element_wave<true>(X, Rt, K, row, col, stage + (threadIdx.x / kWave) * 2 * XE_BUF);
        if (have) {
            const RowQuant rq = row_quant<ASYM>(amax_bits[2 * (size_t)row], amax_bits[2 * (size_t)row + 1], qmax);
            q[(size_t)row * K + col] = (int8_t)exact_code<ASYM>(u, rq, qmax);
        }
    }
}

// ---- rows recomputed as a whole (one workgroup per row, rows with mode == 0 leave at once): every column's chain,
// twice - once for the maximum (zero-point form: maximum and minimum), once for the codes - with the row of x in LDS; R
// is read row by row, coalesced.
template <bool ASYM>
__global__ __launch_bounds__(256) void dense_exact_rows_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ R,
                                                               int K, double qmax, const int* __restrict__ mode,
                                                               int8_t* __restrict__ q, float* __restrict__ scale,
                                                               int32_t* __restrict__ zero) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int row = blockIdx.x, t = threadIdx.x;
    if (!mode[row]) return;
    uint16_t* xr = reinterpret_cast<uint16_t*>(lds_raw);
    double* red = reinterpret_cast<double*>(lds_raw + (((size_t)K * 2 + 15) & ~(size_t)15));
    for (int k = t; k < K; k += 256) xr[k] = X[(size_t)row * K + k];
    __syncthreads();
    RowQuant rq = {};
    for (int pass = 0; pass < 2; ++pass) {
        double mx = ASYM ? -INFINITY : 0.0, mn = -INFINITY;      // mn: maximum of -u
        for (int col = t; col < K; col += 256) {
            const uint16_t* r = R + col;
            double u = 0.0;
            for (int k = 0; k < K; ++k)
                u = fma((double)__uint_as_float((unsigned)xr[k] << 16), (double)__uint_as_float((unsigned)r[(size_t)k * K] << 16), u);
            if (pass == 0) {
                mx = fmax(mx, ASYM ? u : fabs(u));
                if (ASYM) mn = fmax(mn, -u);
            } else {
                q[(size_t)row * K + col] = (int8_t)exact_code<ASYM>(u, rq, qmax);
            }
        }
        if (pass == 0) {
#pragma unroll
            for (int o = kWave / 2; o > 0; o >>= 1) {
                mx = fmax(mx, __shfl_xor(mx, o, kWave));
                if (ASYM) mn = fmax(mn, __shfl_xor(mn, o, kWave));
            }
            if (t % kWave == 0) { red[t / kWave] = mx; red[4 + t / kWave] = mn; }
            __syncthreads();
            const double vmax = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
            const double nmin = fmax(fmax(red[4], red[5]), fmax(red[6], red[7]));
            rq = ASYM ? row_quant<true>(okey(vmax), okey(nmin), qmax)
                      : row_quant<false>((unsigned long long)__double_as_longlong(vmax), 0ull, qmax);
            if (t == 0) {
                scale[row] = rq.scale;
                if (ASYM) zero[row] = rq.izero;
            }
        }
    }
}

}  // namespace

DenseFastWs dense_fast_layout(int M, int K) {
    DenseFastWs w;
    size_t o = 0;
    auto take = [&](size_t bytes) { const size_t at = o; o += round256(bytes); return at; };
    w.capf = ((32 + K / 64) + 7) & ~7;
    w.ut = take((size_t)M * K * sizeof(float));
    w.rt = take((size_t)K * K * sizeof(uint16_t));          // rt | rowmax | scalars: the layout of dense_prepared_layout
    w.rowmax = take((size_t)K * sizeof(float));
    w.scalars = take(256);
    w.segmax = take((size_t)2 * M * (K / DT_SEG) * sizeof(float));       // max |u~|, or max u~ and max (-u~)
    w.eps = take((size_t)M * sizeof(double));
    w.amax = take((size_t)2 * M * sizeof(unsigned long long));     // [M, 2]: maximum and (zero-point form) minimum side
    w.ccount = take((size_t)2 * M * sizeof(int));
    w.cidx = take((size_t)2 * M * CAPC * sizeof(uint16_t));
    w.fcount = take((size_t)M * sizeof(int));
    w.fidx = take((size_t)M * w.capf * sizeof(uint16_t));
    w.foffs = take(((size_t)M + 1) * sizeof(int));
    w.mode = take((size_t)M * sizeof(int));
    w.total = o;
    return w;
}

bool dense_fast_applies(int M, int K, bool zero_point, bool prescale) {
    (void)zero_point;      // both forms of the quantizer are served
    return !prescale && M > 64 && K % 128 == 0 && K <= 16384 && (size_t)M * K < ((size_t)1 << 31);
}

// What the fast evaluation derives from R alone: Rt bf16 [K, K] | max_j |R_kj| float [K] | scalars (256 bytes: rho^2).
struct DensePrepared {
    size_t rt, rowmax, scalars, total;
};
static DensePrepared dense_prepared_layout(int K) {
    DensePrepared p;
    p.rt = 0;
    p.rowmax = round256((size_t)K * K * sizeof(uint16_t));
    p.scalars = p.rowmax + round256((size_t)K * sizeof(float));
    p.total = p.scalars + 256;
    return p;
}
size_t dense_prepared_bytes(int K) { return dense_prepared_layout(K).total; }

hipError_t launch_dense_prepare(hipStream_t st, const uint16_t* R, int K, void* prepared) {
    const DensePrepared P = dense_prepared_layout(K);
    unsigned char* base = static_cast<unsigned char*>(prepared);
    uint16_t* Rt = reinterpret_cast<uint16_t*>(base + P.rt);
    float* rowmax = reinterpret_cast<float*>(base + P.rowmax);
    unsigned* scalars = reinterpret_cast<unsigned*>(base + P.scalars);       // [0]: rho^2 as float bits
    hipLaunchKernelGGL(matrix_row_stats_kernel, dim3(K), dim3(256), 0, st, R, K, rowmax, static_cast<unsigned*>(nullptr), scalars, 64);
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3(K / 64, K / 64), dim3(256), 0, st, R, K, Rt);
    hipLaunchKernelGGL(matrix_row_stats_kernel, dim3(K), dim3(256), 0, st, Rt, K, static_cast<float*>(nullptr), scalars,
                       static_cast<unsigned*>(nullptr), 0);
    return hipGetLastError();
}

namespace {
template <bool ASYM>
hipError_t launch_dense_fast(hipStream_t st, const uint16_t* X, const uint16_t* R, const void* prepared, int M, int K, int act_bits,
                             void* ws, int8_t* q, float* scale, int32_t* zero) {
    const DenseFastWs L = dense_fast_layout(M, K);
    unsigned char* base = static_cast<unsigned char*>(ws);
    float* Ut = reinterpret_cast<float*>(base + L.ut);
    // R's transpose and statistics: the caller's prepared copy, or the workspace's own (same layout at L.rt)
    const DensePrepared P = dense_prepared_layout(K);
    const unsigned char* pbase = prepared ? static_cast<const unsigned char*>(prepared) : base + L.rt;
    const uint16_t* Rt = reinterpret_cast<const uint16_t*>(pbase + P.rt);
    const float* rowmax = reinterpret_cast<const float*>(pbase + P.rowmax);
    const unsigned* scalars = reinterpret_cast<const unsigned*>(pbase + P.scalars);       // [0]: rho^2 as float bits
    float* segmax = reinterpret_cast<float*>(base + L.segmax);
    double* eps = reinterpret_cast<double*>(base + L.eps);
    unsigned long long* amax = reinterpret_cast<unsigned long long*>(base + L.amax);
    int* ccount = reinterpret_cast<int*>(base + L.ccount);
    uint16_t* cidx = reinterpret_cast<uint16_t*>(base + L.cidx);
    int* fcount = reinterpret_cast<int*>(base + L.fcount);
    uint16_t* fidx = reinterpret_cast<uint16_t*>(base + L.fidx);
    int* foffs = reinterpret_cast<int*>(base + L.foffs);
    int* mode = reinterpret_cast<int*>(base + L.mode);
    const double qmax = (double)((1 << (act_bits - 1)) - 1);
    // ETA * m for the runs of the matrix instruction, 2^-24 for each of the GROUP - 1 fp32 additions of a group and for the
    // fp32 store of u~
    const float err_factor = (float)(ldexp(1.0, -21) * (kChunk / 16) + ldexp(1.0, -24) * kGroup);

    if (!prepared) {       // R's transpose and statistics: computed here, into the same layout inside the workspace
        const hipError_t e = launch_dense_prepare(st, R, K, base + L.rt);
        if (e != hipSuccess) return e;
    }
    const int tiles_m = (M + DT_M - 1) / DT_M, tiles_n = K / DT_N;
    // one workgroup fits a CU (LDS): 256 persistent workgroups when there are more tiles than that
    const int ntiles = tiles_m * tiles_n;
    hipLaunchKernelGGL(dense_rotate_bf16_kernel<ASYM>, dim3(ntiles > 256 ? 256 : ntiles), dim3(512), 0, st, X, Rt, M, K, Ut, segmax,
                       tiles_m, tiles_n);
    if (K <= 4096)
        hipLaunchKernelGGL((dense_row_candidates_kernel<true, ASYM>), dim3((M + 3) / 4), dim3(256), 0, st, X, Ut, segmax, M, K, rowmax,
                           scalars, err_factor, eps, amax, ccount, cidx, mode);
    else
        hipLaunchKernelGGL((dense_row_candidates_kernel<false, ASYM>), dim3((M + 3) / 4), dim3(256), 0, st, X, Ut, segmax, M, K, rowmax,
                           scalars, err_factor, eps, amax, ccount, cidx, mode);
    hipLaunchKernelGGL(dense_exact_amax_kernel<ASYM>, dim3((unsigned)(((long)M * CAPC * (ASYM ? 2 : 1) + 255) / 256)), dim3(256), 0, st,
                       X, Rt, M, K, ccount, cidx, amax);
    hipLaunchKernelGGL(dense_quant_flag_kernel<ASYM>, dim3((M + 3) / 4), dim3(256), 4 * sizeof(int), st, Ut, M, K, qmax, eps, amax, q,
                       scale, zero, fcount, fidx, L.capf, mode);
    hipLaunchKernelGGL(dense_scan_counts_kernel, dim3(1), dim3(1024), 0, st, fcount, M, foffs);
    hipLaunchKernelGGL(dense_exact_codes_kernel<ASYM>, dim3(2048), dim3(256), 0, st, X, Rt, M, K, qmax, foffs, fidx, L.capf, amax, q);
    const size_t rows_lds = (((size_t)K * 2 + 15) & ~(size_t)15) + 8 * sizeof(double);
    hipLaunchKernelGGL(dense_exact_rows_kernel<ASYM>, dim3(M), dim3(256), rows_lds, st, X, R, K, qmax, mode, q, scale, zero);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_dense_rotate_quant_fast(hipStream_t st, const uint16_t* X, const uint16_t* R, const void* prepared, int M, int K,
                                          int act_bits, void* ws, int8_t* q, float* scale, int32_t* zero) {
    return zero ? launch_dense_fast<true>(st, X, R, prepared, M, K, act_bits, ws, q, scale, zero)
                : launch_dense_fast<false>(st, X, R, prepared, M, K, act_bits, ws, q, scale, zero);
}

}  // namespace lrq
