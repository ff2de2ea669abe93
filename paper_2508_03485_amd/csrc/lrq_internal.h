// Internal declarations shared by the HIP translation units of liblrq (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lrq.h"

namespace lrq {

inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }


// ---- launchers implemented in the .hip files; each returns hipGetLastError() after the launch ----

// Per-token quantizer description handed to the kernels by value (host-filled).
struct QuantSpec {
    int asym;               // 0: symmetric absmax form, 1: zero-point form of Eq. 1
    double qmax, norm;      // symmetric: 2^(a-1) - 1 and qmax * sqrt(h)
    double L, half, sqrt_h; // zero-point form: 2^a - 1, 2^(a-1), sqrt(h)
    int32_t* zero;          // zero-point form: output [M]
    const float* prescale;  // per-channel factor applied to x before the rotation ([K], nullptr = none)
    int packed;             // 1: 4-bit codes are written two per byte (excess-8 nibbles, see lrq.h), row stride K / 2
    int fp8;                // 1: 4-bit codes are written as FP8 E4M3 bit patterns
};

// u = x.(I (x) H_h) in fp64, per-token statistics, round to codes.  K % 8 == 0, h | K, h power of two.
// zero == nullptr selects the symmetric quantizer, otherwise the zero-point form (zero receives z + 2^(a-1)).
// prescale (every launcher): nullptr, or fp32 [K] multiplied into x channel-wise before the rotation.
// packed (symmetric 4-bit codes only): q receives the packed nibbles ([M, K/2] bytes); only the shapes for which
// hadamard_packs_in_kernel is true may be launched that way.
hipError_t launch_hadamard_quant(hipStream_t st, const uint16_t* X, int M, int K, int h, int act_bits,
                                 int8_t* q, float* scale, int32_t* zero, const float* prescale, bool packed = false,
                                 bool fp8 = false);
// int8 codes in [-7, 7] -> FP8 E4M3 bit patterns, in place (n bytes, n % 16 == 0)
hipError_t launch_codes_to_fp8(hipStream_t st, int8_t* q, size_t n);
// Y = scale_t * wscale_fp8_n * sum_k q * lut_fp8 (+ bias) on the FP8 matrix cores; q8: E4M3 bit patterns [M, K]
hipError_t launch_qgemm_fp8(hipStream_t st, const uint8_t* q8, const float* scale, int M, int K, const lrq_tlq_weight& w,
                            const float* bias, int out_dtype, void* Y);
bool hadamard_packs_in_kernel(int K, int h);
// q int8 [M, K] (codes in [-7, 7]) -> packed nibbles [M, K/2]
hipError_t launch_pack_nibbles(hipStream_t st, const int8_t* q, int M, int K, uint8_t* q4);
// u = x (no rotation), same quantizer.
hipError_t launch_plain_quant(hipStream_t st, const uint16_t* X, int M, int K, int act_bits,
                              int8_t* q, float* scale, int32_t* zero, const float* prescale);
// u = x.R in fp64 (k ascending), written to U [M,K] doubles, then quantized from U.
hipError_t launch_dense_rotate_quant(hipStream_t st, const uint16_t* X, const uint16_t* R, int M, int K,
                                     int act_bits, double* U, int8_t* q, float* scale, int32_t* zero,
                                     const float* prescale);

// The same rotation + quantizer with the bulk product on the bf16 matrix cores, a certified error bound and exact
// recomputation of the undecided elements (either form of the quantizer, no pre-scale; dense_fast_applies says when).
// Bit-identical codes and scales.  ws: dense_fast_layout(M, K).total bytes.
struct DenseFastWs {
    size_t ut, rt, rowmax, scalars, segmax, eps, amax, ccount, cidx, fcount, fidx, foffs, mode, total;
    int capf;       // undecided elements a row's list holds
};
DenseFastWs dense_fast_layout(int M, int K);
bool dense_fast_applies(int M, int K, bool zero_point, bool prescale);
// prepared: NULL, or dense_prepared_bytes(K) bytes that launch_dense_prepare filled from this R (its transpose and the
// statistics the error bound needs): then the call skips that preprocessing.
// zero: NULL (symmetric quantizer) or the per-token zero-points of the zero-point form (then q holds x_q - 2^(b-1)).
hipError_t launch_dense_rotate_quant_fast(hipStream_t st, const uint16_t* X, const uint16_t* R, const void* prepared, int M, int K,
                                          int act_bits, void* ws, int8_t* q, float* scale, int32_t* zero);
size_t dense_prepared_bytes(int K);
hipError_t launch_dense_prepare(hipStream_t st, const uint16_t* R, int K, void* prepared);

// u = ((x.R1).P).R2 with block-diagonal R1, R2 (bf16 [K/B,B,B]), fp64 throughout, perm in gather form; U [M,K]
// and Zp [M,K] doubles are scratch.  B % 128 == 0, B | K.
hipError_t launch_blockperm_rotate_quant(hipStream_t st, const uint16_t* X, int M, int K, int B, const uint16_t* R1,
                                         const int32_t* perm, const uint16_t* R2, int act_bits, double* U, double* Zp,
                                         int8_t* q, float* scale, int32_t* zero, const float* prescale);

// Calibration: greedy block rotations R1, R2 and staggered permutation from calibration activations; metric J.
size_t ars_build_workspace_bytes(int T, int K, int B);
hipError_t launch_ars_build_rotation(hipStream_t st, const uint16_t* Xcal, int T, int K, int B, int n_steps,
                                     const double* Rtilde, const double* Q1, const double* Q2, uint16_t* R1,
                                     int32_t* perm, uint16_t* R2, void* ws);
size_t smooth_workspace_bytes(int K);
hipError_t launch_smooth_factor(hipStream_t st, const uint16_t* Xcal, int T, const float* W, int N, int K, double alpha,
                                float* s, float* inv_s, float* W_out, void* ws);
size_t fluctuation_workspace_bytes();
hipError_t launch_fluctuation_metric(hipStream_t st, const uint16_t* X, size_t n, double* J, void* ws);

hipError_t launch_tlq_quantize_pack(hipStream_t st, const float* W, int N, int K, int bits, int I,
                                    const float* alpha_grid, int n_alpha, const float* beta_grid, int n_beta,
                                    const lrq_tlq_weight& out, const float* gamma_grid, int n_gamma, float* gamma_pos,
                                    float* gamma_neg);

// zero == nullptr: symmetric codes; otherwise the epilogue adds zero_t * colsum_n to the integer sum.
// packed4: q holds packed 4-bit activation codes ([M, K/2] bytes, excess-8 nibbles); zero must then be nullptr.
hipError_t launch_qgemm(hipStream_t st, const int8_t* q, const float* scale, const int32_t* zero, int M, int K,
                        const lrq_tlq_weight& w, const float* bias, int out_dtype, void* Y, bool packed4 = false);

// Y = scale_t * sum_k q * levels (+ bias) on the bf16 matrix cores; w.levels must be set.
hipError_t launch_qgemm_levels(hipStream_t st, const int8_t* q, const float* scale, int M, int K, const lrq_tlq_weight& w,
                               const float* bias, int out_dtype, void* Y);

// Raises a kernel's dynamic-LDS limit (hipFuncAttributeMaxDynamicSharedMemorySize) the first time it is asked for on
// the current device; later calls for the same (kernel, device) return at once.  Safe from several host threads.
hipError_t allow_large_lds(const void* kernel, int bytes);

// ---- private GEMM weight layout ----
// Channels are grouped in tiles of 32, K in blocks of 64.  One (channel tile, K block) unit is 64 slots of 16 bytes:
// slot (c, kq), c = 0..15, kq = 0..3, at byte (16 kq + c) * 16 of the unit, holds the codes of k = 16 kq + [0, 16) of
// the block for channel c of the tile (first 8 bytes) and channel 16 + c (last 8 bytes); one nibble per code, byte j
// of a dword = code[k + j] | code[k + 4 + j] << 4 (k = 0 / 8 for the two dwords of a channel).  Lane 16 kq + c of a
// wave that loads slot (c, kq) thus holds the B operands of two v_mfma_i32_16x16x64_i8 (column c of two neighbouring
// 16-column tiles, the lane group's 16 k).  A 32-column matrix instruction (lane = channel l % 32, k half l / 32)
// reads its channel's 8-byte halves of the slots kq = l / 32 and kq = 2 + l / 32.
// Units are stored [channel tile][K block].
constexpr int kGemmTileN = 32;
constexpr int kGemmBlockK = 64;

// byte offset, inside a unit, of the first of the two 8-byte pieces that lane l of a 32-column matrix instruction
// reads (k = 16 (l / 32) + [0, 16)); the second (k = 32 + 16 (l / 32) + [0, 16)) lies kGemmPiece32Step bytes further
__host__ __device__ inline int gemm_piece32_offset(int l) { return ((l / 32) * 16 + l % 16) * 16 + ((l % 32) / 16) * 8; }
constexpr int kGemmPiece32Step = 2 * 16 * 16;

inline size_t gemm_codes_bytes(int N, int K, int bits) {
    size_t tiles = (size_t)(N + kGemmTileN - 1) / kGemmTileN;
    size_t kblocks = (size_t)K / kGemmBlockK;
    (void)bits;                       // one nibble per code for 3- and 4-bit codes alike
    return tiles * kblocks * 64 * 16;
}

}  // namespace lrq
