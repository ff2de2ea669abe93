// extern "C" entry points of liblrq: argument validation (host only, before any launch), workspace
// carving and dispatch to the kernels.
#include "lrq_internal.h"

#include <mutex>
#include <set>
#include <utility>

namespace lrq {

hipError_t allow_large_lds(const void* kernel, int bytes) {
    static std::mutex mu;
    static std::set<std::pair<const void*, int>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({kernel, dev})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.insert({kernel, dev});
    return e;
}

}  // namespace lrq

namespace {

inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
using lrq::round256;

constexpr int kMaxRowLds = 16384;   // a token row / weight row is staged in LDS as doubles

int check_rotation(const lrq_rotation* rot, int K) {
    if (!rot) return LRQ_EINVAL;
    if (rot->prescale && !aligned16(rot->prescale)) return LRQ_EINVAL;
    switch (rot->kind) {
        case LRQ_ROT_NONE:
            return K <= kMaxRowLds ? LRQ_OK : LRQ_EUNSUPPORTED;
        case LRQ_ROT_HADAMARD:
            if (rot->had_block <= 0) return LRQ_EINVAL;
            if (!is_pow2(rot->had_block) || K % rot->had_block != 0) return LRQ_EUNSUPPORTED;
            return K <= kMaxRowLds ? LRQ_OK : LRQ_EUNSUPPORTED;
        case LRQ_ROT_DENSE:
        case LRQ_ROT_DENSE_F64:
            if (!rot->R || !aligned16(rot->R)) return LRQ_EINVAL;
            if (rot->R_prepared && (reinterpret_cast<uintptr_t>(rot->R_prepared) & 255) != 0) return LRQ_EINVAL;
            return K % 64 == 0 ? LRQ_OK : LRQ_EUNSUPPORTED;
        case LRQ_ROT_BLOCKPERM:
            if (!rot->R1 || !rot->R2 || !rot->perm || rot->block <= 0) return LRQ_EINVAL;
            if (!aligned16(rot->R1) || !aligned16(rot->R2) || !aligned16(rot->perm)) return LRQ_EINVAL;
            if (rot->block % 128 != 0 || K % rot->block != 0) return LRQ_EUNSUPPORTED;
            return K <= kMaxRowLds ? LRQ_OK : LRQ_EUNSUPPORTED;
        default:
            return LRQ_EINVAL;
    }
}

int check_act(const void* X, int M, int K, const lrq_rotation* rot, int act_bits) {
    if (!X || M <= 0 || K <= 0 || !aligned16(X)) return LRQ_EINVAL;
    if (act_bits != 4 && act_bits != 6 && act_bits != 8) return LRQ_EUNSUPPORTED;
    if (K % 8 != 0) return LRQ_EUNSUPPORTED;
    return check_rotation(rot, K);
}

int check_weight(const lrq_tlq_weight* w) {
    if (!w || w->N <= 0 || w->K <= 0) return LRQ_EINVAL;
    if (w->bits != 3 && w->bits != 4) return LRQ_EUNSUPPORTED;
    if (!w->codes || !w->s_pos || !w->s_neg || !w->z_pos || !w->z_neg || !w->alpha || !w->beta || !w->lut ||
        !w->wscale || !w->gemm_codes || !w->colsum)
        return LRQ_EINVAL;
    if (!aligned16(w->codes) || !aligned16(w->lut) || !aligned16(w->gemm_codes)) return LRQ_EINVAL;
    if (w->levels && !aligned16(w->levels)) return LRQ_EINVAL;
    if (w->lut_fp8 && !aligned16(w->lut_fp8)) return LRQ_EINVAL;
    return LRQ_OK;
}

// ---- built-in scratch of lrq_qlinear_static -------------------------------------------------------------------
// One fixed array per device, part of the code object: callers that cannot allocate (stream capture, serving loops)
// get the activation codes / scales / rotation scratch of a layer from here instead of from a workspace argument.
// `scratch` is a host-side stand-in for the symbol; the device address is resolved once per device with
// hipGetSymbolAddress and only that address is ever handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the current device's copy of `scratch` (resolved on first use).
int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LRQ_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LRQ_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LRQ_OK;
}

struct ArsWs {
    size_t u_off, zp_off, total;
};
ArsWs ars_layout(int M, int K, const lrq_rotation* rot) {
    ArsWs l{0, 0, 0};
    if (rot && (rot->kind == LRQ_ROT_DENSE || rot->kind == LRQ_ROT_DENSE_F64)) {
        // U doubles for the evaluation in fp64; the matrix-core evaluation lays its own buffers over the same bytes
        l.total = round256((size_t)M * K * sizeof(double));
        if (rot->kind == LRQ_ROT_DENSE && lrq::dense_fast_applies(M, K, false, rot->prescale != nullptr)) {
            const size_t fast = lrq::dense_fast_layout(M, K).total;
            if (fast > l.total) l.total = fast;
        }
    }
    if (rot && rot->kind == LRQ_ROT_BLOCKPERM) {       // U doubles (first Z = x.R1, finally u), then Zp doubles
        l.zp_off = round256((size_t)M * K * sizeof(double));
        l.total = l.zp_off + round256((size_t)M * K * sizeof(double));
    }
    return l;
}

int run_rotate_quant(hipStream_t st, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                     int8_t* q, float* scale, int32_t* zero, void* ws) {
    hipError_t e = hipSuccess;
    const uint16_t* x = static_cast<const uint16_t*>(X);
    switch (rot->kind) {
        case LRQ_ROT_NONE:
            e = lrq::launch_plain_quant(st, x, M, K, act_bits, q, scale, zero, rot->prescale);
            break;
        case LRQ_ROT_HADAMARD:
            e = lrq::launch_hadamard_quant(st, x, M, K, rot->had_block, act_bits, q, scale, zero, rot->prescale);
            break;
        case LRQ_ROT_BLOCKPERM:
            e = lrq::launch_blockperm_rotate_quant(
                st, x, M, K, rot->block, static_cast<const uint16_t*>(rot->R1), rot->perm,
                static_cast<const uint16_t*>(rot->R2), act_bits, static_cast<double*>(ws),
                reinterpret_cast<double*>(static_cast<char*>(ws) + ars_layout(M, K, rot).zp_off), q, scale, zero,
                rot->prescale);
            break;
        default:
            if (rot->kind == LRQ_ROT_DENSE && lrq::dense_fast_applies(M, K, zero != nullptr, rot->prescale != nullptr))
                e = lrq::launch_dense_rotate_quant_fast(st, x, static_cast<const uint16_t*>(rot->R), rot->R_prepared, M, K, act_bits,
                                                        ws, q, scale, zero);
            else
                e = lrq::launch_dense_rotate_quant(st, x, static_cast<const uint16_t*>(rot->R), M, K, act_bits,
                                                   static_cast<double*>(ws), q, scale, zero, rot->prescale);
            break;
    }
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char* lrq_status_string(int status) {
    switch (status) {
        case LRQ_OK: return "ok";
        case LRQ_EINVAL: return "invalid argument (null pointer, non-positive size, misaligned pointer or inconsistent struct)";
        case LRQ_EUNSUPPORTED: return "unsupported bit-width, block size or shape";
        case LRQ_EWORKSPACE: return "workspace missing or too small";
        case LRQ_EHIP: return "HIP runtime error at launch";
        case LRQ_ESCRATCH: return "the layer needs more scratch memory than the library's built-in buffer holds (use the call that takes a workspace)";
        default: return "unknown status";
    }
}

int lrq_version(void) { return 400; }   // 0.4.0: lrq_tlq_weight grew err_pos / err_neg; lrq_qlinear_static; the probes left the library

size_t lrq_tlq_codes_bytes(int N, int K, int bits) {
    if (N <= 0 || K <= 0 || (bits != 3 && bits != 4) || K % 8 != 0) return 0;
    return (size_t)N * K / 8 * bits;
}

size_t lrq_tlq_gemm_codes_bytes(int N, int K, int bits) {
    if (N <= 0 || K <= 0 || (bits != 3 && bits != 4) || K % 8 != 0) return 0;
    // K that is not a multiple of the GEMM's K block cannot be fed to lrq_qlinear; keep the buffer non-empty
    const int Kp = (K + lrq::kGemmBlockK - 1) / lrq::kGemmBlockK * lrq::kGemmBlockK;
    return lrq::gemm_codes_bytes(N, Kp, bits);
}

size_t lrq_tlq_workspace_bytes(int N, int K, int bits) {
    (void)N; (void)K; (void)bits;
    return 0;
}

static int tlq_impl(void* stream, const float* W, int N, int K, int bits, int I, const float* alpha_grid, int n_alpha,
                    const float* beta_grid, int n_beta, const float* gamma_grid, int n_gamma, lrq_tlq_weight* out,
                    float* gamma_pos, float* gamma_neg) {
    if (!W || !alpha_grid || !beta_grid || !out || N <= 0 || K <= 0 || !aligned16(W)) return LRQ_EINVAL;
    if (n_alpha < 1 || n_alpha > 64 || n_beta < 1 || n_beta > 64) return LRQ_EINVAL;
    if (bits != 3 && bits != 4) return LRQ_EUNSUPPORTED;
    if (out->N != N || out->K != K || out->bits != bits || out->I != I) return LRQ_EINVAL;
    int st = check_weight(out);
    if (st != LRQ_OK) return st;
    if (K % 64 != 0 || K > kMaxRowLds || I > 20) return LRQ_EUNSUPPORTED;
    hipError_t e = lrq::launch_tlq_quantize_pack(static_cast<hipStream_t>(stream), W, N, K, bits, I, alpha_grid,
                                                 n_alpha, beta_grid, n_beta, *out, gamma_grid, n_gamma, gamma_pos,
                                                 gamma_neg);
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_tlq_quantize_pack(void* stream, const float* W, int N, int K, int bits, int I, const float* alpha_grid,
                          int n_alpha, const float* beta_grid, int n_beta, lrq_tlq_weight* out, void* ws,
                          size_t ws_bytes) {
    (void)ws; (void)ws_bytes;
    return tlq_impl(stream, W, N, K, bits, I, alpha_grid, n_alpha, beta_grid, n_beta, nullptr, 0, out, nullptr, nullptr);
}

int lrq_tlq_quantize_pack_clip(void* stream, const float* W, int N, int K, int bits, int I, const float* alpha_grid,
                               int n_alpha, const float* beta_grid, int n_beta, const float* gamma_grid, int n_gamma,
                               lrq_tlq_weight* out, float* gamma_pos, float* gamma_neg, void* ws, size_t ws_bytes) {
    (void)ws; (void)ws_bytes;
    if (!gamma_grid || n_gamma < 1 || n_gamma > 64) return LRQ_EINVAL;
    return tlq_impl(stream, W, N, K, bits, I, alpha_grid, n_alpha, beta_grid, n_beta, gamma_grid, n_gamma, out, gamma_pos,
                    gamma_neg);
}

size_t lrq_ars_workspace_bytes(int M, int K, const lrq_rotation* rot, int act_bits) {
    (void)act_bits;
    if (M <= 0 || K <= 0) return 0;
    return ars_layout(M, K, rot).total;
}

size_t lrq_ars_dense_prepared_bytes(int K) {
    if (K <= 0 || K % 128 != 0 || K > 16384) return 0;
    return lrq::dense_prepared_bytes(K);
}

int lrq_ars_dense_prepare(void* stream, const void* R, int K, void* prepared, size_t prepared_bytes) {
    if (!R || !prepared || K <= 0) return LRQ_EINVAL;
    const size_t need = lrq_ars_dense_prepared_bytes(K);
    if (need == 0) return LRQ_EUNSUPPORTED;
    if (prepared_bytes < need || (reinterpret_cast<uintptr_t>(prepared) & 255) != 0 || (reinterpret_cast<uintptr_t>(R) & 15) != 0)
        return LRQ_EINVAL;
    const hipError_t e = lrq::launch_dense_prepare(static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(R), K, prepared);
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_ars_dense_diagnostics(int M, int K, size_t offsets[4]) {
    if (M <= 0 || K <= 0 || !offsets) return LRQ_EINVAL;
    if (!lrq::dense_fast_applies(M, K, false, false)) return LRQ_EUNSUPPORTED;
    const lrq::DenseFastWs l = lrq::dense_fast_layout(M, K);
    offsets[0] = l.ut;
    offsets[1] = l.eps;
    offsets[2] = l.fcount;
    offsets[3] = l.mode;
    return LRQ_OK;
}

static int ars_impl(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits, int8_t* q,
                    float* scale, int32_t* zero, bool asym, void* ws, size_t ws_bytes) {
    int st = check_act(X, M, K, rot, act_bits);
    if (st != LRQ_OK) return st;
    if (!q || !scale || !aligned16(q) || (asym && !zero)) return LRQ_EINVAL;
    const size_t need = ars_layout(M, K, rot).total;
    if (need > 0 && (!ws || ws_bytes < need || !aligned16(ws))) return LRQ_EWORKSPACE;
    return run_rotate_quant(static_cast<hipStream_t>(stream), X, M, K, rot, act_bits, q, scale, asym ? zero : nullptr, ws);
}

int lrq_ars_rotate_quant(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                         int8_t* q, float* scale, void* ws, size_t ws_bytes) {
    return ars_impl(stream, X, M, K, rot, act_bits, q, scale, nullptr, false, ws, ws_bytes);
}

int lrq_ars_rotate_quant_asym(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                              int8_t* q, float* scale, int32_t* zero, void* ws, size_t ws_bytes) {
    return ars_impl(stream, X, M, K, rot, act_bits, q, scale, zero, true, ws, ws_bytes);
}

size_t lrq_workspace_bytes(int M, int N, int K, const lrq_rotation* rot, int act_bits) {
    (void)N; (void)act_bits;
    if (M <= 0 || K <= 0) return 0;
    return round256((size_t)M * K) + round256((size_t)M * sizeof(float)) + ars_layout(M, K, rot).total;
}

size_t lrq_workspace_bytes_asym(int M, int N, int K, const lrq_rotation* rot, int act_bits) {
    if (M <= 0 || K <= 0) return 0;
    return lrq_workspace_bytes(M, N, K, rot, act_bits) + round256((size_t)M * sizeof(int32_t));
}

enum class Gemm { kInt8, kInt8Zero, kLevels };

// the *_levels calls need the bf16 level table, and levels that are bf16 values
static int check_levels(const lrq_tlq_weight* w) {
    if (!w->levels) return LRQ_EINVAL;
    return (w->I < 0 || w->I > 7) ? LRQ_EUNSUPPORTED : LRQ_OK;
}

static int qgemm_impl(void* stream, const int8_t* q, const float* scale, const int32_t* zero, Gemm kind, int M, int K,
                      const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y) {
    const bool asym = kind == Gemm::kInt8Zero;
    if (!q || !scale || !Y || M <= 0 || K <= 0 || !aligned16(q) || !aligned16(Y) || (asym && !zero)) return LRQ_EINVAL;
    int st = check_weight(w);
    if (st != LRQ_OK) return st;
    if (w->K != K) return LRQ_EINVAL;
    if (out_dtype != LRQ_OUT_BF16 && out_dtype != LRQ_OUT_FP32) return LRQ_EUNSUPPORTED;
    if (K % lrq::kGemmBlockK != 0) return LRQ_EUNSUPPORTED;
    hipError_t e;
    if (kind == Gemm::kLevels) {
        st = check_levels(w);
        if (st != LRQ_OK) return st;
        e = lrq::launch_qgemm_levels(static_cast<hipStream_t>(stream), q, scale, M, K, *w, bias, out_dtype, Y);
    } else {
        e = lrq::launch_qgemm(static_cast<hipStream_t>(stream), q, scale, asym ? zero : nullptr, M, K, *w, bias, out_dtype, Y);
    }
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_qgemm_levels(void* stream, const int8_t* q, const float* scale, int M, int K, const lrq_tlq_weight* w,
                     const float* bias, int out_dtype, void* Y) {
    return qgemm_impl(stream, q, scale, nullptr, Gemm::kLevels, M, K, w, bias, out_dtype, Y);
}

int lrq_qgemm(void* stream, const int8_t* q, const float* scale, int M, int K, const lrq_tlq_weight* w,
              const float* bias, int out_dtype, void* Y) {
    return qgemm_impl(stream, q, scale, nullptr, Gemm::kInt8, M, K, w, bias, out_dtype, Y);
}

int lrq_qgemm_asym(void* stream, const int8_t* q, const float* scale, const int32_t* zero, int M, int K,
                   const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y) {
    return qgemm_impl(stream, q, scale, zero, Gemm::kInt8Zero, M, K, w, bias, out_dtype, Y);
}

static int qlinear_impl(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                        const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes,
                        Gemm kind) {
    const bool asym = kind == Gemm::kInt8Zero;
    int st = check_act(X, M, K, rot, act_bits);
    if (st != LRQ_OK) return st;
    st = check_weight(w);
    if (st != LRQ_OK) return st;
    if (kind == Gemm::kLevels) {
        st = check_levels(w);
        if (st != LRQ_OK) return st;
    }
    if (!Y || !aligned16(Y) || w->K != K) return LRQ_EINVAL;
    if (out_dtype != LRQ_OUT_BF16 && out_dtype != LRQ_OUT_FP32) return LRQ_EUNSUPPORTED;
    if (K % lrq::kGemmBlockK != 0) return LRQ_EUNSUPPORTED;
    const size_t need = asym ? lrq_workspace_bytes_asym(M, w->N, K, rot, act_bits) : lrq_workspace_bytes(M, w->N, K, rot, act_bits);
    if (!ws || ws_bytes < need || !aligned16(ws)) return LRQ_EWORKSPACE;
    // workspace: q | scale | rotation scratch | zero (zero-point form only)
    char* base = static_cast<char*>(ws);
    int8_t* q = reinterpret_cast<int8_t*>(base);
    float* scale = reinterpret_cast<float*>(base + round256((size_t)M * K));
    void* rot_ws = base + round256((size_t)M * K) + round256((size_t)M * sizeof(float));
    int32_t* zero = asym ? reinterpret_cast<int32_t*>(static_cast<char*>(rot_ws) + ars_layout(M, K, rot).total) : nullptr;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = run_rotate_quant(s, X, M, K, rot, act_bits, q, scale, zero, rot_ws);
    if (st != LRQ_OK) return st;
    hipError_t e = kind == Gemm::kLevels ? lrq::launch_qgemm_levels(s, q, scale, M, K, *w, bias, out_dtype, Y)
                                         : lrq::launch_qgemm(s, q, scale, zero, M, K, *w, bias, out_dtype, Y);
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_qlinear_levels(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                       const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes) {
    return qlinear_impl(stream, X, M, K, rot, act_bits, w, bias, out_dtype, Y, ws, ws_bytes, Gemm::kLevels);
}

int lrq_qlinear(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes) {
    return qlinear_impl(stream, X, M, K, rot, act_bits, w, bias, out_dtype, Y, ws, ws_bytes, Gemm::kInt8);
}

// ---- packed 4-bit activation codes -------------------------------------------------------------------------------
static bool packs_in_kernel(const lrq_rotation* rot, int K) {
    return !rot->prescale && ((rot->kind == LRQ_ROT_HADAMARD && lrq::hadamard_packs_in_kernel(K, rot->had_block)) ||
                              (rot->kind == LRQ_ROT_NONE && lrq::hadamard_packs_in_kernel(K, 1)));
}

size_t lrq_ars_workspace_bytes_packed4(int M, int K, const lrq_rotation* rot) {
    if (M <= 0 || K <= 0 || !rot) return 0;
    // rotations whose kernels do not pack themselves quantize to int8 codes in the workspace first
    return (packs_in_kernel(rot, K) ? 0 : round256((size_t)M * K)) + ars_layout(M, K, rot).total;
}

static int rotate_quant_packed4(hipStream_t st, const void* X, int M, int K, const lrq_rotation* rot, uint8_t* q4, float* scale,
                                void* ws) {
    if (packs_in_kernel(rot, K)) {
        const int h = rot->kind == LRQ_ROT_HADAMARD ? rot->had_block : 1;
        return lrq::launch_hadamard_quant(st, static_cast<const uint16_t*>(X), M, K, h, 4, reinterpret_cast<int8_t*>(q4), scale,
                                          nullptr, nullptr, true) == hipSuccess ? LRQ_OK : LRQ_EHIP;
    }
    int8_t* q8 = static_cast<int8_t*>(ws);
    const int st8 = run_rotate_quant(st, X, M, K, rot, 4, q8, scale, nullptr, static_cast<char*>(ws) + round256((size_t)M * K));
    if (st8 != LRQ_OK) return st8;
    return lrq::launch_pack_nibbles(st, q8, M, K, q4) == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_ars_rotate_quant_packed4(void* stream, const void* X, int M, int K, const lrq_rotation* rot, uint8_t* q4, float* scale,
                                 void* ws, size_t ws_bytes) {
    int st = check_act(X, M, K, rot, 4);
    if (st != LRQ_OK) return st;
    if (K % 16 != 0) return LRQ_EUNSUPPORTED;
    if (!q4 || !scale || !aligned16(q4)) return LRQ_EINVAL;
    const size_t need = lrq_ars_workspace_bytes_packed4(M, K, rot);
    if (need > 0 && (!ws || ws_bytes < need || !aligned16(ws))) return LRQ_EWORKSPACE;
    return rotate_quant_packed4(static_cast<hipStream_t>(stream), X, M, K, rot, q4, scale, ws);
}

static int check_gemm_common(const lrq_tlq_weight* w, int K, int out_dtype) {
    int st = check_weight(w);
    if (st != LRQ_OK) return st;
    if (w->K != K) return LRQ_EINVAL;
    if (out_dtype != LRQ_OUT_BF16 && out_dtype != LRQ_OUT_FP32) return LRQ_EUNSUPPORTED;
    return K % lrq::kGemmBlockK != 0 ? LRQ_EUNSUPPORTED : LRQ_OK;
}

int lrq_qgemm_packed4(void* stream, const uint8_t* q4, const float* scale, int M, int K, const lrq_tlq_weight* w,
                      const float* bias, int out_dtype, void* Y) {
    if (!q4 || !scale || !Y || M <= 0 || K <= 0 || !aligned16(q4) || !aligned16(Y)) return LRQ_EINVAL;
    const int st = check_gemm_common(w, K, out_dtype);
    if (st != LRQ_OK) return st;
    return lrq::launch_qgemm(static_cast<hipStream_t>(stream), reinterpret_cast<const int8_t*>(q4), scale, nullptr, M, K, *w, bias,
                             out_dtype, Y, true) == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

size_t lrq_workspace_bytes_packed4(int M, int N, int K, const lrq_rotation* rot) {
    (void)N;
    if (M <= 0 || K <= 0 || !rot) return 0;
    return round256((size_t)M * K / 2) + round256((size_t)M * sizeof(float)) + lrq_ars_workspace_bytes_packed4(M, K, rot);
}

int lrq_qlinear_packed4(void* stream, const void* X, int M, int K, const lrq_rotation* rot, const lrq_tlq_weight* w,
                        const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes) {
    int st = check_act(X, M, K, rot, 4);
    if (st != LRQ_OK) return st;
    if (!Y || !aligned16(Y)) return LRQ_EINVAL;
    st = check_gemm_common(w, K, out_dtype);
    if (st != LRQ_OK) return st;
    if (!ws || ws_bytes < lrq_workspace_bytes_packed4(M, w->N, K, rot) || !aligned16(ws)) return LRQ_EWORKSPACE;
    char* base = static_cast<char*>(ws);
    uint8_t* q4 = reinterpret_cast<uint8_t*>(base);
    float* scale = reinterpret_cast<float*>(base + round256((size_t)M * K / 2));
    void* rot_ws = base + round256((size_t)M * K / 2) + round256((size_t)M * sizeof(float));
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = rotate_quant_packed4(s, X, M, K, rot, q4, scale, rot_ws);
    if (st != LRQ_OK) return st;
    return lrq::launch_qgemm(s, reinterpret_cast<const int8_t*>(q4), scale, nullptr, M, K, *w, bias, out_dtype, Y, true) == hipSuccess
               ? LRQ_OK : LRQ_EHIP;
}

// ---- FP8 E4M3 operands on both sides --------------------------------------------------------------------------------
static int rotate_quant_fp8(hipStream_t st, const void* X, int M, int K, const lrq_rotation* rot, uint8_t* q8, float* scale,
                            void* ws) {
    if (packs_in_kernel(rot, K)) {
        const int h = rot->kind == LRQ_ROT_HADAMARD ? rot->had_block : 1;
        return lrq::launch_hadamard_quant(st, static_cast<const uint16_t*>(X), M, K, h, 4, reinterpret_cast<int8_t*>(q8), scale,
                                          nullptr, nullptr, false, true) == hipSuccess ? LRQ_OK : LRQ_EHIP;
    }
    // the other kinds write int8 codes, converted in place
    const int st8 = run_rotate_quant(st, X, M, K, rot, 4, reinterpret_cast<int8_t*>(q8), scale, nullptr, ws);
    if (st8 != LRQ_OK) return st8;
    return lrq::launch_codes_to_fp8(st, reinterpret_cast<int8_t*>(q8), (size_t)M * K) == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_ars_rotate_quant_fp8(void* stream, const void* X, int M, int K, const lrq_rotation* rot, uint8_t* q8, float* scale,
                             void* ws, size_t ws_bytes) {
    int st = check_act(X, M, K, rot, 4);
    if (st != LRQ_OK) return st;
    if (K % 16 != 0) return LRQ_EUNSUPPORTED;
    if (!q8 || !scale || !aligned16(q8)) return LRQ_EINVAL;
    const size_t need = ars_layout(M, K, rot).total;
    if (need > 0 && (!ws || ws_bytes < need || !aligned16(ws))) return LRQ_EWORKSPACE;
    return rotate_quant_fp8(static_cast<hipStream_t>(stream), X, M, K, rot, q8, scale, ws);
}

int lrq_qgemm_fp8(void* stream, const uint8_t* q8, const float* scale, int M, int K, const lrq_tlq_weight* w,
                  const float* bias, int out_dtype, void* Y) {
    if (!q8 || !scale || !Y || M <= 0 || K <= 0 || !aligned16(q8) || !aligned16(Y)) return LRQ_EINVAL;
    const int st = check_gemm_common(w, K, out_dtype);
    if (st != LRQ_OK) return st;
    if (!w->lut_fp8 || !w->wscale_fp8) return LRQ_EINVAL;
    return lrq::launch_qgemm_fp8(static_cast<hipStream_t>(stream), q8, scale, M, K, *w, bias, out_dtype, Y) == hipSuccess ? LRQ_OK
                                                                                                                         : LRQ_EHIP;
}

int lrq_qlinear_fp8(void* stream, const void* X, int M, int K, const lrq_rotation* rot, const lrq_tlq_weight* w,
                    const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes) {
    int st = check_act(X, M, K, rot, 4);
    if (st != LRQ_OK) return st;
    if (!Y || !aligned16(Y)) return LRQ_EINVAL;
    st = check_gemm_common(w, K, out_dtype);
    if (st != LRQ_OK) return st;
    if (!w->lut_fp8 || !w->wscale_fp8) return LRQ_EINVAL;
    if (!ws || ws_bytes < lrq_workspace_bytes(M, w->N, K, rot, 4) || !aligned16(ws)) return LRQ_EWORKSPACE;
    char* base = static_cast<char*>(ws);
    uint8_t* q8 = reinterpret_cast<uint8_t*>(base);
    float* scale = reinterpret_cast<float*>(base + round256((size_t)M * K));
    void* rot_ws = base + round256((size_t)M * K) + round256((size_t)M * sizeof(float));
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = rotate_quant_fp8(s, X, M, K, rot, q8, scale, rot_ws);
    if (st != LRQ_OK) return st;
    return lrq::launch_qgemm_fp8(s, q8, scale, M, K, *w, bias, out_dtype, Y) == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_init(void) {
    void* p = nullptr;
    return static_scratch(&p);
}

size_t lrq_static_scratch_bytes(void) { return kStaticScratchBytes; }

int lrq_qlinear_static(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                       const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y) {
    // sizes first: a layer that does not fit is refused before anything else is looked at or launched
    if (M <= 0 || K <= 0 || !w || w->N <= 0) return LRQ_EINVAL;
    if (lrq_workspace_bytes(M, w->N, K, rot, act_bits) > kStaticScratchBytes) return LRQ_ESCRATCH;
    void* ws = nullptr;
    const int st = static_scratch(&ws);
    if (st != LRQ_OK) return st;
    return qlinear_impl(stream, X, M, K, rot, act_bits, w, bias, out_dtype, Y, ws, kStaticScratchBytes, Gemm::kInt8);
}

int lrq_qlinear_asym(void* stream, const void* X, int M, int K, const lrq_rotation* rot, int act_bits,
                     const lrq_tlq_weight* w, const float* bias, int out_dtype, void* Y, void* ws, size_t ws_bytes) {
    return qlinear_impl(stream, X, M, K, rot, act_bits, w, bias, out_dtype, Y, ws, ws_bytes, Gemm::kInt8Zero);
}

size_t lrq_ars_build_workspace_bytes(int T, int K, int block) {
    if (T <= 0 || K <= 0 || block <= 0 || K % block != 0) return 0;
    return lrq::ars_build_workspace_bytes(T, K, block);
}

int lrq_ars_build_rotation(void* stream, const void* Xcal, int T, int K, int block, int n_steps, const double* Rtilde,
                           const double* Q1, const double* Q2, void* R1, int32_t* perm, void* R2, void* ws,
                           size_t ws_bytes) {
    if (!Xcal || !Rtilde || !Q1 || !Q2 || !R1 || !perm || !R2 || T <= 0 || K <= 0 || block <= 0 || n_steps <= 0)
        return LRQ_EINVAL;
    if (!aligned16(Xcal) || !aligned16(Rtilde) || !aligned16(Q1) || !aligned16(Q2) || !aligned16(R1) ||
        !aligned16(perm) || !aligned16(R2))
        return LRQ_EINVAL;
    if (block % 128 != 0 || block > 1024 || K % block != 0 || K > kMaxRowLds) return LRQ_EUNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < lrq::ars_build_workspace_bytes(T, K, block)) return LRQ_EWORKSPACE;
    const hipError_t e = lrq::launch_ars_build_rotation(
        static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(Xcal), T, K, block, n_steps, Rtilde, Q1, Q2,
        static_cast<uint16_t*>(R1), perm, static_cast<uint16_t*>(R2), ws);
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

size_t lrq_smooth_workspace_bytes(int K) { return K > 0 ? lrq::smooth_workspace_bytes(K) : 0; }

int lrq_smooth_factor(void* stream, const void* Xcal, int T, const float* W, int N, int K, double alpha, float* s,
                      float* inv_s, float* W_out, void* ws, size_t ws_bytes) {
    if (!Xcal || !W || !s || !inv_s || T <= 0 || N <= 0 || K <= 0 || alpha != alpha) return LRQ_EINVAL;
    if (!aligned16(Xcal) || !aligned16(W) || !aligned16(s) || !aligned16(inv_s) || !aligned16(W_out)) return LRQ_EINVAL;
    if (K % 8 != 0 || alpha < 0.0 || alpha > 1.0) return LRQ_EUNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < lrq::smooth_workspace_bytes(K)) return LRQ_EWORKSPACE;
    const hipError_t e = lrq::launch_smooth_factor(static_cast<hipStream_t>(stream), static_cast<const uint16_t*>(Xcal),
                                                   T, W, N, K, alpha, s, inv_s, W_out, ws);
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

size_t lrq_fluctuation_workspace_bytes(void) { return lrq::fluctuation_workspace_bytes(); }

int lrq_fluctuation_metric(void* stream, const void* X, int M, int K, double* J_out, void* ws, size_t ws_bytes) {
    if (!X || !J_out || M <= 0 || K <= 0 || !aligned16(X)) return LRQ_EINVAL;
    if (((size_t)M * K) % 8 != 0) return LRQ_EUNSUPPORTED;
    if (!ws || !aligned16(ws) || ws_bytes < lrq::fluctuation_workspace_bytes()) return LRQ_EWORKSPACE;
    const hipError_t e = lrq::launch_fluctuation_metric(static_cast<hipStream_t>(stream),
                                                        static_cast<const uint16_t*>(X), (size_t)M * K, J_out, ws);
    return e == hipSuccess ? LRQ_OK : LRQ_EHIP;
}

int lrq_ars_select(double J, double threshold) {
    if (J != J || threshold != threshold) return LRQ_EINVAL;
    return J < threshold ? LRQ_ROT_HADAMARD : LRQ_ROT_BLOCKPERM;
}

}  // extern "C"
#pragma GCC visibility pop
