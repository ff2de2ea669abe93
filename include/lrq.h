/*
 * lrq.h - C ABI of the MI355X (gfx950) quantized-linear hot path of LRQ-DiT.
 *
 * The library implements one W-A-quantized linear layer of a Diffusion Transformer:
 *   activations  -> (optional smoothing pre-scale) -> Adaptive Rotation Scheme (Hadamard, or the
 *                   outlier-aware rotation in dense or structured R1.P.R2 form, chosen per layer)
 *                   -> per-token uniform quantization to 4/6/8-bit codes
 *   weights      -> packed 3/4-bit Twin-Log Quantization (TLQ) codes, decoded through a per-channel
 *                   level table into int8 MFMA operands inside the GEMM
 *   output       -> int32 accumulators rescaled per token x per channel.
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library neither frees nor keeps
 *     it after the call returns.  Structs (lrq_rotation, lrq_tlq_weight) live in HOST memory and are
 *     read during the call only; the pointers inside them are device pointers.
 *   - Work is enqueued on the caller's stream (a hipStream_t passed as void*, NULL = default stream)
 *     and is asynchronous: no entry point synchronises the device.
 *   - Arrays are dense and row-major.  X[M,K] activations (tokens x hidden), W[N,K] weights (output
 *     channel x hidden), Y[M,N].  bf16 buffers hold raw bfloat16 bit patterns (uint16).
 *   - Return value: LRQ_OK (0) or a negative lrq_status.  All argument validation happens on the host
 *     before anything is launched, so a failing call has enqueued nothing.
 *   - Pointers must be aligned to 16 bytes (what any device allocator returns).
 *   - No entry point allocates or frees device memory, so calls can be recorded into a HIP graph.  The first
 *     launch of a kernel that needs more than 64 KB of LDS raises that kernel's limit (hipFuncSetAttribute),
 *     once per kernel and device: run each call shape once outside stream capture before capturing it.
 *   - Calls may come from several host threads; calls that share a workspace or an output must be ordered
 *     by the caller (same stream, or events).
 */
#ifndef LRQ_H_
#define LRQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LRQ_OK = 0,
    LRQ_EINVAL = -1,       /* null pointer, non-positive size, misaligned pointer, inconsistent struct   */
    LRQ_EUNSUPPORTED = -2, /* bit-width, block size or shape outside what the kernels implement          */
    LRQ_EWORKSPACE = -3,   /* workspace pointer null or smaller than the *_workspace_bytes() answer      */
    LRQ_EHIP = -4,         /* the HIP runtime reported an error while launching                           */
    LRQ_ESCRATCH = -5      /* lrq_qlinear_static: the layer does not fit the library's built-in scratch buffer */
} lrq_status;

typedef enum {
    LRQ_ROT_NONE = 0, LRQ_ROT_HADAMARD = 1, LRQ_ROT_DENSE = 2, LRQ_ROT_BLOCKPERM = 3, LRQ_ROT_DENSE_F64 = 4
} lrq_rotation_kind;
typedef enum { LRQ_OUT_BF16 = 0, LRQ_OUT_FP32 = 1 } lrq_out_dtype;

/*
 * Per-layer rotation choice of the Adaptive Rotation Scheme (paper: Method, "Adaptive Rotation
 * Scheme", case equation X.R_H if J < threshold, X.R1.P.R2 otherwise).
 *   LRQ_ROT_HADAMARD  u = x . (I (x) H_h): block-diagonal Sylvester Hadamard of block size
 *                     had_block = h, a power of two dividing K (Preliminaries, Eq. hadamard).  The
 *                     transform is taken unnormalised (+-1 entries) and 1/sqrt(h) goes into the scale.
 *   LRQ_ROT_DENSE     u = x . R with R a K x K bf16 matrix (row-major, device): any orthogonal matrix,
 *                     e.g. the paper's greedy outlier-aware product R1.P.R2 materialised.  The codes are those of
 *                     the fp64 sum over ascending k; the bulk of the product runs on the bf16 matrix cores and
 *                     every rounding decision that their error bound does not settle is recomputed in fp64.
 *   LRQ_ROT_DENSE_F64 the same rotation evaluated entirely in fp64 (about ten times slower; same codes and scales,
 *                     and it leaves u as doubles [M, K] at the head of the rotation workspace): the reference the
 *                     fast evaluation is checked against.
 *   LRQ_ROT_BLOCKPERM u = ((x . R1) . P) . R2: the outlier-aware branch in the structured form the paper
 *                     prints.  R1, R2 are block-diagonal with blocks of `block` channels, stored as bf16
 *                     [K/block, block, block] (block g acts on channels g*block ...); P is the staggered
 *                     channel permutation in gather form, (z . P)[:, j] = z[:, perm[j]], perm int32 [K]
 *                     (a permutation of 0..K-1: the library does not verify that, it only clamps every
 *                     index into range).  Both products are plain fp64 sums in ascending k; nothing is rounded
 *                     between the stages.  block must be a multiple of 128 that divides K.  Costs
 *                     O(K * block) per token instead of O(K^2).
 *   LRQ_ROT_NONE      u = x.
 */
typedef struct {
    int kind;        /* lrq_rotation_kind                                   */
    int had_block;   /* h for LRQ_ROT_HADAMARD, ignored otherwise           */
    const void* R;   /* bf16 [K,K] device pointer for LRQ_ROT_DENSE or NULL */
    int block;             /* LRQ_ROT_BLOCKPERM: block size of R1, R2, else ignored     */
    const void* R1;        /* LRQ_ROT_BLOCKPERM: bf16 [K/block, block, block] (device)  */
    const int32_t* perm;   /* LRQ_ROT_BLOCKPERM: int32 [K] (device)                     */
    const void* R2;        /* LRQ_ROT_BLOCKPERM: bf16 [K/block, block, block] (device)  */
    const float* prescale; /* any kind: NULL, or fp32 [K] (device) multiplied into x channel by channel before the
                              rotation - the reciprocal smoothing factor of lrq_smooth_factor (Experiment,
                              "Implementation Details": difficulty migration from activations to weights)     */
    const void* R_prepared; /* LRQ_ROT_DENSE: NULL, or the device buffer lrq_ars_dense_prepare filled from this R (a rotation
                              is fixed at calibration time: its transpose and the statistics the error bound needs are then
                              computed once instead of in every call).  Must be NULL or refilled if R's contents change.  */
} lrq_rotation;

/*
 * A TLQ-quantized weight matrix (paper: Method, "Twin-Log Quantization for Weights").  The caller
 * allocates every array (device memory, sizes below) and fills N, K, bits, I before the call to
 * lrq_tlq_quantize_pack, which writes the arrays.
 *   codes      uint8 [N, K*bits/8]  canonical packing of the signed b-bit codes W_q = W_q+ - W_q-
 *              (Eq. log-based quantizer), each stored as its low b bits.
 *              bits = 4: byte j = code[2j] | code[2j+1] << 4.
 *              bits = 3: every 8 codes form a 24-bit little-endian group, code i at bits [3i, 3i+3).
 *   s_pos/s_neg double [N], z_pos/z_neg int32 [N]: scales and zero-points of the two log-domain twins
 *              (Eq. hyperparameters clip); alpha/beta float [N]: the clip factors the search picked.
 *   lut        int8 [N, 16] (16 entries per channel for either bit-width, the first 2^bits used):
 *              lut[n][c & (2^bits-1)] is the int8 MFMA operand of signed code c, i.e. the level
 *              +-round(2^r 2^I) 2^(f-I) of "Hardware Implementation" divided by wscale[n] and rounded.
 *   wscale     float [N]: max_c |level| / 127.
 *   gemm_codes uint8 [lrq_tlq_gemm_codes_bytes()]: the same codes re-tiled for the GEMM's operand
 *              loader (private layout, subject to change; only lrq_qlinear reads it).
 *   colsum     int32 [N]: the sum over k of the channel's decoded int8 levels; multiplied by a token's
 *              zero-point in the *_asym calls (Eq. 1 of the paper keeps a zero-point per quantizer).
 *   levels     bf16 [N, 16] or NULL (then not written, and the *_levels calls refuse the struct):
 *              levels[n][c & (2^bits-1)] is the level +-round(2^r 2^I) 2^(f-I) itself, rounded to nearest-even
 *              bf16 - exact for 0 <= I <= 7, where a level has at most 8 significant bits.
 *   lut_fp8    uint8 [N, 16] or NULL, wscale_fp8 float [N] or NULL (then not written, and the *_fp8 calls refuse the
 *              struct): the levels with I = 3 mantissa bits, +-round(2^r 2^3) 2^(f-3) - four significant bits, an FP8
 *              E4M3 number's worth ("Hardware Implementation": I is a free parameter of the integerisation) - divided
 *              by the power of two wscale_fp8[n] = 2^(floor(log2 max_c |level|) - 7) and rounded to E4M3 (nearest
 *              even; exact for levels within 2^13 of the largest, subnormal spacing 2^-9 below, zero below 2^-10).
 *              lut_fp8[n][c & (2^bits-1)] is the E4M3 bit pattern, operand of the FP8 matrix instruction.
 *   err_pos/err_neg double [N] or NULL (then not written): the value of the search objective sum (W_f - W)^2 of each
 *              twin at the chosen clip factors (+inf for a twin without a valid candidate).  The sum runs in a fixed
 *              order - 256 interleaved partial sums over ascending k, then the partial sums in ascending order.
 */
typedef struct {
    int N, K;
    int bits;            /* 3 | 4                                                              */
    int I;               /* integerisation bits of 2^r ~ round(2^r 2^I) 2^-I; < 0: exact 2^e   */
    uint8_t* codes;
    double* s_pos;
    double* s_neg;
    int32_t* z_pos;
    int32_t* z_neg;
    float* alpha;
    float* beta;
    int8_t* lut;
    float* wscale;
    uint8_t* gemm_codes;
    int32_t* colsum;     /* int32 [N]: sum_k lut[n][code[n,k]], the weight of an activation zero-point */
    uint16_t* levels;    /* bf16 [N,16] or NULL: the levels themselves, operands of the *_levels calls  */
    uint8_t* lut_fp8;    /* uint8 [N,16] or NULL: E4M3 bit patterns of the I = 3 levels / wscale_fp8            */
    float* wscale_fp8;   /* float [N] or NULL: the power-of-two scale of lut_fp8                                 */
    double* err_pos;     /* double [N] or NULL: search objective of the positive twin at its chosen factors */
    double* err_neg;     /* double [N] or NULL: the same for the negative twin                              */
} lrq_tlq_weight;

/* Human-readable text of a status code (static storage). */
const char* lrq_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int lrq_version(void);

/* Sizes in bytes of the caller-allocated arrays of lrq_tlq_weight; 0 on invalid arguments. */
size_t lrq_tlq_codes_bytes(int N, int K, int bits);
size_t lrq_tlq_gemm_codes_bytes(int N, int K, int bits);

/* Workspace of lrq_tlq_quantize_pack (bytes; 0 is a valid answer). */
size_t lrq_tlq_workspace_bytes(int N, int K, int bits);

/*
 * lrq_tlq_quantize_pack - calibrate and pack weight codes for a bit-width.
 * Paper: Method, "Twin-Log Quantization for Weights": Eq. log-based quantizer (codes), Eq.
 * hyperparameters clip (search-based clipping, s+-, z+-), Eq. dequant (levels used by the search
 * objective), "Hardware Implementation" (exponent split and integerisation -> lut, wscale).
 *   W           float [N,K], the weights already smoothed and rotated into the activation basis.
 *   bits        3 | 4.    I: see lrq_tlq_weight.
 *   alpha_grid  float [n_alpha] device, candidate clip factors of the positive twin, scanned in order;
 *   beta_grid   float [n_beta]  device, same for the negative twin.  1 <= n <= 64.
 *   out         host struct whose device arrays are written (out->N/K/bits/I must equal the arguments).
 *   ws          device workspace of at least lrq_tlq_workspace_bytes(N,K,bits) bytes (may be NULL if 0).
 * Per output channel and per sign the first grid value minimising sum (W_f - W)^2 wins; a candidate
 * whose clipped maximum does not exceed the minimum is skipped; exact zeros take code 0.
 * Requires K % 64 == 0 and K <= 16384.  Errors: LRQ_EINVAL, LRQ_EUNSUPPORTED, LRQ_EWORKSPACE, LRQ_EHIP.
 */
int lrq_tlq_quantize_pack(void* stream, const float* W, int N, int K, int bits, int I,
                          const float* alpha_grid, int n_alpha, const float* beta_grid, int n_beta,
                          lrq_tlq_weight* out, void* ws, size_t ws_bytes);

/*
 * lrq_tlq_quantize_pack with a lower clip (an extension, not in the paper: its Eq. hyperparameters clip only clips
 * the large-magnitude end, so W_min stays the log of the channel's tiniest weight and most levels are spent far below
 * the weights that matter).  A second factor gamma, searched jointly with alpha (beta), raises the lower end:
 *     s = (alpha W_max - gamma W_min) / intervals,   z = round(gamma W_min / s)
 * (log2 values are negative for |w| < 1, so gamma < 1 clips; smaller magnitudes clamp to the lowest level of their
 * twin).  gamma_grid float [n_gamma] device, 1 <= n_gamma <= 64, scanned inside the loop over alpha (beta); the grid
 * {1} reproduces lrq_tlq_quantize_pack bit for bit.  gamma_pos / gamma_neg: float [N] device or NULL, receive the
 * chosen factors.  Everything else as lrq_tlq_quantize_pack.
 */
int lrq_tlq_quantize_pack_clip(void* stream, const float* W, int N, int K, int bits, int I,
                               const float* alpha_grid, int n_alpha, const float* beta_grid, int n_beta,
                               const float* gamma_grid, int n_gamma, lrq_tlq_weight* out, float* gamma_pos,
                               float* gamma_neg, void* ws, size_t ws_bytes);

/* Workspace of lrq_ars_rotate_quant (bytes). */
size_t lrq_ars_workspace_bytes(int M, int K, const lrq_rotation* rot, int act_bits);

/*
 * lrq_ars_rotate_quant - rotate and quantize an activation tile for a given per-layer rotation choice.
 * Paper: Method, "Adaptive Rotation Scheme" (rotation choice), Preliminaries Eq. 1 in its symmetric
 * per-token form (Experiment, "Implementation Details": per-token dynamic activation quantization).
 *   X         bf16 [M,K].            rot: see lrq_rotation.       act_bits: 4 | 6 | 8 (the settings of the paper's tables).
 *   q         int8 [M,K] out: codes in [-qmax, qmax], qmax = 2^(act_bits-1) - 1 (4- and 6-bit codes are held
 *             in int8 containers), q = rint(u * (qmax / amax_t)), round-half-even, amax_t = max_k |u|.
 *   scale     float [M] out: amax_t / (qmax * sqrt(h)) for Hadamard, amax_t / qmax otherwise, so that
 *             q * scale approximates x . (normalised rotation).  An all-zero token gives q = 0, scale 0.
 * The rotation, the maximum and the rounding decision are taken in fp64 on the exact bf16 values.
 * Requires K % 8 == 0; Hadamard: had_block a power of two dividing K, K <= 16384.
 */
int lrq_ars_rotate_quant(void* stream, const void* X, int M, int K, const lrq_rotation* rot,
                         int act_bits, int8_t* q, float* scale, void* ws, size_t ws_bytes);

/*
 * Diagnostics of the LRQ_ROT_DENSE evaluation (host only, launches nothing): byte offsets, inside the workspace that
 * lrq_ars_rotate_quant was given, of what its matrix-core evaluation leaves behind -
 *   offsets[0]  float  [M, K]  the approximation u~ of u = x . R (bf16 matrix cores, fp64 accumulation of 64-k runs)
 *   offsets[1]  double [M]     the bound eps_t on |u~ - u| that holds for every element of token t
 *   offsets[2]  int32  [M]     how many elements of token t the bound left undecided and were recomputed in fp64
 *   offsets[3]  int32  [M]     1 for a token that was recomputed as a whole (0 otherwise)
 * Returns LRQ_OK, or LRQ_EUNSUPPORTED when that evaluation does not serve the shape (then the fp64 evaluation runs:
 * M <= 64, K % 128 != 0, K > 16384, M * K >= 2^31; also whenever a pre-scale or the zero-point form is used).
 */
int lrq_ars_dense_diagnostics(int M, int K, size_t offsets[4]);

/*
 * Preprocessing of a dense rotation matrix (Method, ARS case equation, outlier-aware branch: R is computed offline, so
 * what the run-time call derives from R alone can be computed offline too).  lrq_ars_dense_prepare writes R's transpose
 * and the per-row / per-column statistics of the error bound into `prepared` (device, at least
 * lrq_ars_dense_prepared_bytes(K) bytes, 256-byte aligned); a lrq_rotation of kind LRQ_ROT_DENSE whose R_prepared points
 * there skips that work in lrq_ars_rotate_quant / lrq_qlinear (three small launches per call) and gives the same codes.
 * lrq_ars_dense_prepared_bytes returns 0 for a K the matrix-core evaluation does not serve (K % 128 != 0 or K > 16384);
 * lrq_ars_dense_prepare then returns LRQ_EUNSUPPORTED.  R: bf16 [K, K] device.  Errors: LRQ_EINVAL (null pointer,
 * K <= 0, misaligned or short buffer), LRQ_EHIP.
 */
size_t lrq_ars_dense_prepared_bytes(int K);
int lrq_ars_dense_prepare(void* stream, const void* R, int K, void* prepared, size_t prepared_bytes);

/* Workspace of lrq_qlinear (bytes): activation codes, scales and rotation scratch. */
size_t lrq_workspace_bytes(int M, int N, int K, const lrq_rotation* rot, int act_bits);

/*
 * lrq_qlinear - fused rotate, quantize, decode, GEMM and rescale:
 *   Y[t,n] = scale_t * wscale_n * sum_k q[t,k] * lut_n[code[n,k]]  (+ bias_n)
 * Paper: last equation of "Hardware Implementation" (integer product times activation scale), with
 * the int8 level table in place of the shift datapath; "SpeedUp and Latency" (INT8 x INT8 GEMM with
 * higher-precision accumulation).
 *   X, M, K, rot, act_bits  as for lrq_ars_rotate_quant.
 *   w          host struct written by lrq_tlq_quantize_pack (w->K must equal K).
 *   bias       float [N] or NULL.
 *   out_dtype  LRQ_OUT_BF16 (round-to-nearest-even) | LRQ_OUT_FP32.       Y: [M, N] out.
 *   ws         device workspace of at least lrq_workspace_bytes(M, N, K, rot, act_bits) bytes.
 * Runs as the rotate+quantize kernel(s) followed by the decode+MFMA GEMM kernel on the same stream.
 * Requires K % 64 == 0.
 */
int lrq_qlinear(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y,
                void* ws, size_t ws_bytes);

/*
 * lrq_qlinear_static - lrq_qlinear for callers that cannot allocate device memory or carry a workspace around:
 * code running under HIP stream capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and bit-identical results as lrq_qlinear, minus the workspace: the activation codes, the token scales
 * and the rotation scratch live in a buffer of lrq_static_scratch_bytes() = 64 MiB that is part of the library's
 * code object (every device the library runs on holds one copy until the process ends).  The call allocates and
 * frees nothing.
 *   - A layer whose lrq_workspace_bytes(M, N, K, rot, act_bits) exceeds the buffer is refused with LRQ_ESCRATCH and
 *     nothing is launched (Hadamard layers fit up to M * K of about 6.7e7: all layers of the 8192- and 4608-token
 *     workloads; dense rotations up to M * K of about 7e6).
 *   - Every call on a device uses that device's one buffer: calls that may overlap on one device (different
 *     streams, or several host threads) race on it and must be ordered by the caller.  The buffer keeps the previous
 *     call's contents; the kernels overwrite what they read, nothing relies on its state.
 *   - lrq_init() resolves the buffer's device address for the current device (lrq_qlinear_static does the same on
 *     its first call on a device): call it once per device before a stream capture.  Returns LRQ_OK or LRQ_EHIP.
 */
int lrq_init(void);
size_t lrq_static_scratch_bytes(void);
int lrq_qlinear_static(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                       const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y);

/*
 * lrq_qgemm - the GEMM + rescale stage of lrq_qlinear alone, on activation codes already produced by
 * lrq_ars_rotate_quant (q int8 [M,K], scale float [M]).  Same formula, same constraints; no workspace.
 */
int lrq_qgemm(void* stream, const int8_t* q, const float* scale, int M, int K,
              const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y);

/*
 * The same layer on the levels themselves (paper: "Hardware Implementation", exponent split f / r and the
 * integerisation of 2^r with I bits), without the per-channel int8 renormalisation that lrq_qlinear applies to them:
 *   Y[t,n] = scale_t * sum_k q[t,k] * v_n(code[n,k])  (+ bias_n),   v_n(c) = +-round(2^r 2^I) 2^(f-I) = w->levels[n][c].
 * Levels (for 0 <= I <= 7) and activation codes are bf16 values, so the contraction runs on the bf16 matrix cores
 * with every product exact and fp32 accumulation: the fidelity reference of the int8 path at half its matrix rate.
 * Requires w->levels != NULL and 0 <= w->I <= 7 (LRQ_EUNSUPPORTED otherwise); everything else (arguments, workspace
 * = lrq_workspace_bytes, constraints, errors) as for lrq_qgemm / lrq_qlinear.
 */
int lrq_qgemm_levels(void* stream, const int8_t* q, const float* scale, int M, int K,
                     const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y);
int lrq_qlinear_levels(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                       const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y,
                       void* ws, size_t ws_bytes);

/*
 * Zero-point variants: the activation quantizer exactly as the paper's Eq. 1 (Preliminaries), per token:
 *   s = (x_max - x_min) / (2^b - 1), z = round(x_min / s), x_q = clamp(round(x / s) - z, 0, 2^b - 1), x_f = s (x_q + z).
 * The quotients x / s are taken as products with one reciprocal inv = (2^b - 1) / (x_max - x_min); rounding is
 * half-to-even; a constant token takes x_q = 0 and (s, z) = (|c|, sign c).  Outputs are in the form the integer GEMM
 * consumes: q = x_q - 2^(b-1) (int8 [M,K]), zero = z + 2^(b-1) (int32 [M]), scale = s (/ sqrt(h) for Hadamard)
 * (float [M]), so that x_f = scale * (q + zero).  The linear layer then is
 *   Y[t,n] = scale_t * wscale_n * (sum_k q[t,k] lut_n[code[n,k]] + zero_t * colsum_n)  (+ bias_n).
 * Everything else (arguments, constraints, workspace rules, errors) is as for the symmetric calls;
 * lrq_workspace_bytes_asym gives lrq_qlinear_asym's workspace.
 */
int lrq_ars_rotate_quant_asym(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                              int8_t* q, float* scale, int32_t* zero, void* ws, size_t ws_bytes);
int lrq_qgemm_asym(void* stream, const int8_t* q, const float* scale, const int32_t* zero, int M, int K,
                   const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y);
size_t lrq_workspace_bytes_asym(int M, int N, int K, const lrq_rotation* rot, int act_bits);
int lrq_qlinear_asym(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                     const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes);

/*
 * Packed 4-bit activation codes (the W4A4 / W3A4 settings of the paper's tables; the paper leaves the storage of the
 * codes open).  Same quantizer as lrq_ars_rotate_quant with act_bits = 4 - symmetric, codes in [-7, 7] - but two codes
 * per byte, half the bytes between the two stages of the layer:
 *   q4  uint8 [M, K/2]: every 8 consecutive codes of a token make 4 bytes; byte j of the group holds code[j] + 8 in its
 *       low nibble and code[4 + j] + 8 in its high nibble (nibbles in 1 .. 15, "excess-8").
 * lrq_qgemm_packed4 widens the nibbles to bytes on their way into LDS and removes the offset in the epilogue
 * (acc - 8 * colsum_n), so its outputs equal lrq_qgemm's on the unpacked codes bit for bit.  Hadamard rotations (and no
 * rotation) pack inside the rotate kernel; the other kinds quantize to int8 codes in the workspace and pack in a second
 * pass.  Requires K % 16 == 0 (K % 64 == 0 for the GEMM); everything else as for the unpacked calls.
 */
size_t lrq_ars_workspace_bytes_packed4(int M, int K, const lrq_rotation* rot);
int lrq_ars_rotate_quant_packed4(void* stream, const void* X, int M, int K, const lrq_rotation* rot, uint8_t* q4, float* scale,
                                 void* ws, size_t ws_bytes);
int lrq_qgemm_packed4(void* stream, const uint8_t* q4, const float* scale, int M, int K, const lrq_tlq_weight* w,
                      const float* bias, int out_dtype, void* Y);
size_t lrq_workspace_bytes_packed4(int M, int N, int K, const lrq_rotation* rot);
int lrq_qlinear_packed4(void* stream, const void* X, int M, int K, const lrq_rotation* rot, const lrq_tlq_weight* w,
                        const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes);

/*
 * The layer with FP8 E4M3 operands on both sides (v_mfma_f32_32x32x64_f8f6f4; the alternative value map of
 * "Hardware Implementation" with I = 3: no int8 table, the levels keep their own four bits).  Only for 4-bit activation
 * codes: an integer in [-7, 7] is an E4M3 value, a 6- or 8-bit code is not.
 *   lrq_ars_rotate_quant_fp8  as lrq_ars_rotate_quant with act_bits = 4, but q8 uint8 [M, K] receives the codes as E4M3
 *                             bit patterns (same scale).  Workspace: lrq_ars_workspace_bytes(M, K, rot, 4).
 *   lrq_qgemm_fp8             Y[t,n] = scale_t * wscale_fp8_n * sum_k q[t,k] * value(lut_fp8_n[code[n,k]])  (+ bias_n).
 *                             Every product is exact in fp32; the fp32 accumulation of the matrix instruction rounds
 *                             (order unspecified), so outputs carry a relative error of about sqrt(K) 2^-24.
 *   lrq_qlinear_fp8           both stages; workspace lrq_workspace_bytes(M, N, K, rot, 4).
 * Requires w->lut_fp8 and w->wscale_fp8 (LRQ_EINVAL otherwise), K % 64 == 0; errors as for the int8 calls.
 */
int lrq_ars_rotate_quant_fp8(void* stream, const void* X, int M, int K, const lrq_rotation* rot, uint8_t* q8, float* scale,
                             void* ws, size_t ws_bytes);
int lrq_qgemm_fp8(void* stream, const uint8_t* q8, const float* scale, int M, int K, const lrq_tlq_weight* w,
                  const float* bias, int out_dtype, void* Y);
int lrq_qlinear_fp8(void* stream, const void* X, int M, int K, const lrq_rotation* rot, const lrq_tlq_weight* w,
                    const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes);

/*
 * Calibration of the outlier-aware branch (paper: Method, "Adaptive Rotation Scheme": greedy rotations
 * R^i = E_c* R~ Q E_c*, R^ = prod_i R^i, built block-wise; staggered permutation P; second rotation).
 * Runs once per layer, off the inference path.
 *   Xcal     bf16 [T, K] device: calibration activations of the layer.
 *   block    block size B of both rotations (multiple of 128, at most 1024, dividing K).
 *   n_steps  greedy updates per block (>= 1).
 *   Rtilde   double [B, B] device: the initial orthogonal matrix R~ (its first row should be constant 1/sqrt(B),
 *            which spreads channel 0 evenly over the block).
 *   Q1, Q2   double [K/B, n_steps, B, B] device: the orthogonal matrix Q of every block and step, for the
 *            first and the second rotation (the paper draws them at random: the caller does, and passes them in).
 *   R1, R2   bf16 [K/B, B, B] device, written; perm int32 [K] device, written (gather form): exactly the
 *            arrays a LRQ_ROT_BLOCKPERM rotation takes.
 *   ws       device workspace of lrq_ars_build_workspace_bytes(T, K, block) bytes.
 * Step i of a block: c* = its channel with the largest |value| over the T tokens (first one on ties); E exchanges
 * channels 0 and c*; activations and running product are multiplied, left to right, by E, R~, Q[i], E.  P: channels
 * sorted by range max - min of Xcal.R1 (descending, ties by index) and dealt across the blocks left to right on
 * even rounds, right to left on odd rounds.  All sums run term by term in ascending index with separately rounded
 * fp64 multiply and add; the working state stays fp64 and only R1, R2 are rounded (once) to bf16.
 * Errors: LRQ_EINVAL, LRQ_EUNSUPPORTED, LRQ_EWORKSPACE, LRQ_EHIP.
 */
size_t lrq_ars_build_workspace_bytes(int T, int K, int block);
int lrq_ars_build_rotation(void* stream, const void* Xcal, int T, int K, int block, int n_steps,
                           const double* Rtilde, const double* Q1, const double* Q2, void* R1, int32_t* perm,
                           void* R2, void* ws, size_t ws_bytes);

/*
 * Smoothing factor with migration strength alpha (paper: Experiment, "Implementation Details", strength 0.5; the
 * factor is the cited SmoothQuant one): per input channel c
 *     s_c = max_t |Xcal[t,c]|^alpha / max_n |W[n,c]|^(1-alpha)          (s_c = 1 if either maximum is 0)
 * evaluated in fp64 (alpha == 0.5 as sqrt(a / w), otherwise with pow).  Runs once per layer, off the inference path.
 *   Xcal bf16 [T, K], W fp32 [N, K] device inputs.
 *   s     fp32 [K] device, written: fp32(s_c).
 *   inv_s fp32 [K] device, written: fp32(1 / s_c) - the `prescale` of lrq_rotation.
 *   W_out fp32 [N, K] device or NULL: if given, receives W[n,c] * s[c] (one fp32 multiplication; may alias W) -
 *         the smoothed weights that then go through the rotation and lrq_tlq_quantize_pack.
 *   ws    device workspace of lrq_smooth_workspace_bytes(K) bytes.
 * Requires K % 8 == 0.  Errors: LRQ_EINVAL, LRQ_EUNSUPPORTED, LRQ_EWORKSPACE, LRQ_EHIP.
 */
size_t lrq_smooth_workspace_bytes(int K);
int lrq_smooth_factor(void* stream, const void* Xcal, int T, const float* W, int N, int K, double alpha, float* s,
                      float* inv_s, float* W_out, void* ws, size_t ws_bytes);

/*
 * Fluctuation metric of a layer's activations (paper: Method, Eq. J): J = ||X||_F / sqrt(M K) for X bf16 [M, K]
 * (M = batch x tokens).  J_out: double[1] device, written.  ws: device workspace of
 * lrq_fluctuation_workspace_bytes() bytes.  Requires (M K) % 8 == 0.  The sum of squares is taken in fp64 in a
 * fixed order (the same input gives the same bits on every run).
 * lrq_ars_select (host only, launches nothing): the case equation that follows Eq. J - LRQ_ROT_HADAMARD when
 * J < threshold, LRQ_ROT_BLOCKPERM otherwise (the paper uses threshold 1); LRQ_EINVAL if either argument is NaN.
 */
size_t lrq_fluctuation_workspace_bytes(void);
int lrq_fluctuation_metric(void* stream, const void* X, int M, int K, double* J_out, void* ws, size_t ws_bytes);
int lrq_ars_select(double J, double threshold);

#ifdef __cplusplus
}
#endif
#endif /* LRQ_H_ */
