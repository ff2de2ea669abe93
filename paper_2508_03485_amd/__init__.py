"""Thin Python binding of liblrq (the C ABI declared in include/lrq.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch is
used for device memory and streams.  There is no CPU or eager fallback: if liblrq.so has not been
built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LRQ_LIB", os.path.join(_HERE, "liblrq.so"))   # LRQ_LIB: developer override

LRQ_OK, LRQ_EINVAL, LRQ_EUNSUPPORTED, LRQ_EWORKSPACE, LRQ_EHIP, LRQ_ESCRATCH = 0, -1, -2, -3, -4, -5
LRQ_ROT_NONE, LRQ_ROT_HADAMARD, LRQ_ROT_DENSE, LRQ_ROT_BLOCKPERM, LRQ_ROT_DENSE_F64 = 0, 1, 2, 3, 4
LRQ_OUT_BF16, LRQ_OUT_FP32 = 0, 1

EXPORTS = ("lrq_status_string", "lrq_version", "lrq_tlq_codes_bytes", "lrq_tlq_gemm_codes_bytes",
           "lrq_tlq_workspace_bytes", "lrq_tlq_quantize_pack", "lrq_ars_workspace_bytes",
           "lrq_ars_rotate_quant", "lrq_workspace_bytes", "lrq_qlinear", "lrq_qgemm",
           "lrq_ars_rotate_quant_asym", "lrq_qgemm_asym", "lrq_workspace_bytes_asym",
           "lrq_qlinear_asym", "lrq_ars_build_workspace_bytes", "lrq_ars_build_rotation",
           "lrq_fluctuation_workspace_bytes", "lrq_fluctuation_metric", "lrq_ars_select",
           "lrq_smooth_workspace_bytes", "lrq_smooth_factor", "lrq_tlq_quantize_pack_clip", "lrq_qgemm_levels",
           "lrq_qlinear_levels", "lrq_ars_dense_diagnostics", "lrq_ars_dense_prepared_bytes", "lrq_ars_dense_prepare", "lrq_ars_workspace_bytes_packed4",
           "lrq_ars_rotate_quant_packed4", "lrq_qgemm_packed4", "lrq_workspace_bytes_packed4", "lrq_qlinear_packed4",
           "lrq_ars_rotate_quant_fp8", "lrq_qgemm_fp8", "lrq_qlinear_fp8", "lrq_init", "lrq_static_scratch_bytes", "lrq_qlinear_static")


class LrqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class _Rotation(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("had_block", ctypes.c_int), ("R", ctypes.c_void_p),
                ("block", ctypes.c_int), ("R1", ctypes.c_void_p), ("perm", ctypes.c_void_p), ("R2", ctypes.c_void_p),
                ("prescale", ctypes.c_void_p), ("R_prepared", ctypes.c_void_p)]


class _TlqWeight(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("K", ctypes.c_int), ("bits", ctypes.c_int), ("I", ctypes.c_int),
                ("codes", ctypes.c_void_p), ("s_pos", ctypes.c_void_p), ("s_neg", ctypes.c_void_p),
                ("z_pos", ctypes.c_void_p), ("z_neg", ctypes.c_void_p), ("alpha", ctypes.c_void_p),
                ("beta", ctypes.c_void_p), ("lut", ctypes.c_void_p), ("wscale", ctypes.c_void_p),
                ("gemm_codes", ctypes.c_void_p), ("colsum", ctypes.c_void_p), ("levels", ctypes.c_void_p),
                ("lut_fp8", ctypes.c_void_p), ("wscale_fp8", ctypes.c_void_p),
                ("err_pos", ctypes.c_void_p), ("err_neg", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load liblrq.so (once) and declare the signatures of include/lrq.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2508_03485_amd.build` "
                          "(hipcc, gfx950); there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.lrq_status_string.restype, L.lrq_status_string.argtypes = ctypes.c_char_p, [ci]
    L.lrq_version.restype, L.lrq_version.argtypes = ci, []
    for name in ("lrq_tlq_codes_bytes", "lrq_tlq_gemm_codes_bytes", "lrq_tlq_workspace_bytes"):
        f = getattr(L, name)
        f.restype, f.argtypes = sz, [ci, ci, ci]
    L.lrq_tlq_quantize_pack.restype = ci
    L.lrq_tlq_quantize_pack.argtypes = [vp, vp, ci, ci, ci, ci, vp, ci, vp, ci, ctypes.POINTER(_TlqWeight), vp, sz]
    L.lrq_tlq_quantize_pack_clip.restype = ci
    L.lrq_tlq_quantize_pack_clip.argtypes = [vp, vp, ci, ci, ci, ci, vp, ci, vp, ci, vp, ci, ctypes.POINTER(_TlqWeight),
                                             vp, vp, vp, sz]
    L.lrq_ars_workspace_bytes.restype = sz
    L.lrq_ars_workspace_bytes.argtypes = [ci, ci, ctypes.POINTER(_Rotation), ci]
    L.lrq_ars_rotate_quant.restype = ci
    L.lrq_ars_rotate_quant.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), ci, vp, vp, vp, sz]
    L.lrq_ars_dense_diagnostics.restype = ci
    L.lrq_ars_dense_diagnostics.argtypes = [ci, ci, ctypes.POINTER(sz * 4)]
    L.lrq_ars_dense_prepared_bytes.restype = sz
    L.lrq_ars_dense_prepared_bytes.argtypes = [ci]
    L.lrq_ars_dense_prepare.restype = ci
    L.lrq_ars_dense_prepare.argtypes = [vp, vp, ci, vp, sz]
    L.lrq_ars_workspace_bytes_packed4.restype = sz
    L.lrq_ars_workspace_bytes_packed4.argtypes = [ci, ci, ctypes.POINTER(_Rotation)]
    L.lrq_ars_rotate_quant_packed4.restype = ci
    L.lrq_ars_rotate_quant_packed4.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), vp, vp, vp, sz]
    L.lrq_qgemm_packed4.restype = ci
    L.lrq_qgemm_packed4.argtypes = [vp, vp, vp, ci, ci, ctypes.POINTER(_TlqWeight), vp, ci, vp]
    L.lrq_workspace_bytes_packed4.restype = sz
    L.lrq_workspace_bytes_packed4.argtypes = [ci, ci, ci, ctypes.POINTER(_Rotation)]
    L.lrq_qlinear_packed4.restype = ci
    L.lrq_qlinear_packed4.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), ctypes.POINTER(_TlqWeight), vp, ci, vp, vp, sz]
    L.lrq_ars_rotate_quant_fp8.restype = ci
    L.lrq_ars_rotate_quant_fp8.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), vp, vp, vp, sz]
    L.lrq_qgemm_fp8.restype = ci
    L.lrq_qgemm_fp8.argtypes = [vp, vp, vp, ci, ci, ctypes.POINTER(_TlqWeight), vp, ci, vp]
    L.lrq_qlinear_fp8.restype = ci
    L.lrq_qlinear_fp8.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), ctypes.POINTER(_TlqWeight), vp, ci, vp, vp, sz]
    L.lrq_workspace_bytes.restype = sz
    L.lrq_workspace_bytes.argtypes = [ci, ci, ci, ctypes.POINTER(_Rotation), ci]
    L.lrq_qlinear.restype = ci
    L.lrq_qlinear.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), ci, ctypes.POINTER(_TlqWeight), vp, ci,
                              vp, vp, sz]
    L.lrq_init.restype, L.lrq_init.argtypes = ci, []
    L.lrq_static_scratch_bytes.restype, L.lrq_static_scratch_bytes.argtypes = sz, []
    L.lrq_qlinear_static.restype = ci
    L.lrq_qlinear_static.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), ci, ctypes.POINTER(_TlqWeight), vp, ci, vp]
    L.lrq_qgemm.restype = ci
    L.lrq_qgemm.argtypes = [vp, vp, vp, ci, ci, ctypes.POINTER(_TlqWeight), vp, ci, vp]
    L.lrq_ars_rotate_quant_asym.restype = ci
    L.lrq_ars_rotate_quant_asym.argtypes = [vp, vp, ci, ci, ctypes.POINTER(_Rotation), ci, vp, vp, vp, vp, sz]
    L.lrq_qgemm_asym.restype = ci
    L.lrq_qgemm_asym.argtypes = [vp, vp, vp, vp, ci, ci, ctypes.POINTER(_TlqWeight), vp, ci, vp]
    L.lrq_workspace_bytes_asym.restype = sz
    L.lrq_workspace_bytes_asym.argtypes = [ci, ci, ci, ctypes.POINTER(_Rotation), ci]
    L.lrq_qlinear_asym.restype = ci
    L.lrq_qlinear_asym.argtypes = L.lrq_qlinear.argtypes
    L.lrq_qgemm_levels.restype, L.lrq_qgemm_levels.argtypes = ci, L.lrq_qgemm.argtypes
    L.lrq_qlinear_levels.restype, L.lrq_qlinear_levels.argtypes = ci, L.lrq_qlinear.argtypes
    L.lrq_ars_build_workspace_bytes.restype, L.lrq_ars_build_workspace_bytes.argtypes = sz, [ci, ci, ci]
    L.lrq_ars_build_rotation.restype = ci
    L.lrq_ars_build_rotation.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, sz]
    L.lrq_fluctuation_workspace_bytes.restype, L.lrq_fluctuation_workspace_bytes.argtypes = sz, []
    L.lrq_fluctuation_metric.restype = ci
    L.lrq_fluctuation_metric.argtypes = [vp, vp, ci, ci, vp, vp, sz]
    L.lrq_ars_select.restype, L.lrq_ars_select.argtypes = ci, [ctypes.c_double, ctypes.c_double]
    L.lrq_smooth_workspace_bytes.restype, L.lrq_smooth_workspace_bytes.argtypes = sz, [ci]
    L.lrq_smooth_factor.restype = ci
    L.lrq_smooth_factor.argtypes = [vp, vp, ci, vp, ci, ci, ctypes.c_double, vp, vp, vp, vp, sz]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().lrq_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != LRQ_OK:
        raise LrqError(status, where)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


@dataclass
class Rotation:
    """Per-layer rotation choice: kind in {"none", "hadamard", "dense", "blockperm", "dense_f64"}."""
    kind: str = "hadamard"
    had_block: int = 0
    R: object = None        # torch bf16 [K, K] on the device for kind == "dense" / "dense_f64"
    block: int = 0          # kind == "blockperm": block size of R1, R2
    R1: object = None       # torch bf16 [K/block, block, block] on the device
    perm: object = None     # torch int32 [K] on the device (gather form)
    R2: object = None       # torch bf16 [K/block, block, block] on the device
    prescale: object = None # any kind: torch fp32 [K] on the device multiplied into x before the rotation
    prepared: object = None # kind == "dense": torch uint8 buffer filled by ars_dense_prepare(R), or None

    def __setattr__(self, name, value):
        object.__setattr__(self, name, value)
        object.__setattr__(self, "_cs", None)       # any change drops the cached C struct

    def c_struct(self) -> _Rotation:
        """The C struct of this choice (built once per state: marshalling is most of a small call's host time)."""
        cs = self.__dict__.get("_cs")
        if cs is None:
            kinds = {"none": LRQ_ROT_NONE, "hadamard": LRQ_ROT_HADAMARD, "dense": LRQ_ROT_DENSE,
                     "blockperm": LRQ_ROT_BLOCKPERM, "dense_f64": LRQ_ROT_DENSE_F64}
            cs = _Rotation(kinds[self.kind], int(self.had_block), _ptr(self.R), int(self.block), _ptr(self.R1),
                           _ptr(self.perm), _ptr(self.R2), _ptr(self.prescale), _ptr(self.prepared))
            object.__setattr__(self, "_cs", cs)
        return cs


class TLQWeight:
    """Device arrays of one TLQ-quantized weight matrix (see lrq_tlq_weight in include/lrq.h)."""

    def __init__(self, N: int, K: int, bits: int, I: int, device):
        import torch
        L = lib()
        self.N, self.K, self.bits, self.I = N, K, bits, I
        nb, ng = L.lrq_tlq_codes_bytes(N, K, bits), L.lrq_tlq_gemm_codes_bytes(N, K, bits)
        if nb == 0 or ng == 0:
            raise LrqError(LRQ_EUNSUPPORTED, "TLQWeight sizes")
        kw = dict(device=device)
        self.codes = torch.empty(nb, dtype=torch.uint8, **kw).view(N, nb // N)
        self.s_pos = torch.empty(N, dtype=torch.float64, **kw)
        self.s_neg = torch.empty(N, dtype=torch.float64, **kw)
        self.z_pos = torch.empty(N, dtype=torch.int32, **kw)
        self.z_neg = torch.empty(N, dtype=torch.int32, **kw)
        self.alpha = torch.empty(N, dtype=torch.float32, **kw)
        self.beta = torch.empty(N, dtype=torch.float32, **kw)
        self.lut = torch.empty((N, 16), dtype=torch.int8, **kw)
        self.wscale = torch.empty(N, dtype=torch.float32, **kw)
        self.gemm_codes = torch.zeros(ng, dtype=torch.uint8, **kw)
        self.colsum = torch.empty(N, dtype=torch.int32, **kw)
        self.levels = torch.empty((N, 16), dtype=torch.bfloat16, **kw)
        self.lut_fp8 = torch.empty((N, 16), dtype=torch.uint8, **kw)
        self.wscale_fp8 = torch.empty(N, dtype=torch.float32, **kw)
        self.err_pos = torch.empty(N, dtype=torch.float64, **kw)
        self.err_neg = torch.empty(N, dtype=torch.float64, **kw)

    def __setattr__(self, name, value):
        object.__setattr__(self, name, value)
        object.__setattr__(self, "_cs", None)       # any change drops the cached C struct

    def c_struct(self) -> _TlqWeight:
        """The C struct over these arrays (built once per state)."""
        cs = self.__dict__.get("_cs")
        if cs is None:
            cs = _TlqWeight(self.N, self.K, self.bits, self.I, _ptr(self.codes), _ptr(self.s_pos), _ptr(self.s_neg),
                            _ptr(self.z_pos), _ptr(self.z_neg), _ptr(self.alpha), _ptr(self.beta), _ptr(self.lut),
                            _ptr(self.wscale), _ptr(self.gemm_codes), _ptr(self.colsum), _ptr(self.levels),
                            _ptr(self.lut_fp8), _ptr(self.wscale_fp8), _ptr(self.err_pos), _ptr(self.err_neg))
            object.__setattr__(self, "_cs", cs)
        return cs


def tlq_quantize_pack(W, bits: int, I: int = 7, alpha_grid=None, beta_grid=None, out: Optional[TLQWeight] = None,
                      gamma_grid=None):
    """lrq_tlq_quantize_pack: W fp32 [N, K] on the device -> TLQWeight.
    gamma_grid (fp32 device tensor): lrq_tlq_quantize_pack_clip, the search with a lower clip factor; the chosen
    factors land in w.gamma_pos / w.gamma_neg."""
    import torch
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous()
    N, K = W.shape
    if alpha_grid is None:
        alpha_grid = torch.tensor([1.0 + 0.05 * i for i in range(21)], dtype=torch.float32, device=W.device)
    if beta_grid is None:
        beta_grid = alpha_grid
    w = out if out is not None else TLQWeight(N, K, bits, I, W.device)
    cs = w.c_struct()
    if gamma_grid is None:
        st = lib().lrq_tlq_quantize_pack(_stream(), _ptr(W), N, K, bits, I, _ptr(alpha_grid), alpha_grid.numel(),
                                         _ptr(beta_grid), beta_grid.numel(), ctypes.byref(cs), None, 0)
        _check(st, "lrq_tlq_quantize_pack")
    else:
        assert gamma_grid.is_cuda and gamma_grid.dtype == torch.float32
        w.gamma_pos = torch.empty(N, dtype=torch.float32, device=W.device)
        w.gamma_neg = torch.empty(N, dtype=torch.float32, device=W.device)
        st = lib().lrq_tlq_quantize_pack_clip(_stream(), _ptr(W), N, K, bits, I, _ptr(alpha_grid), alpha_grid.numel(),
                                              _ptr(beta_grid), beta_grid.numel(), _ptr(gamma_grid), gamma_grid.numel(),
                                              ctypes.byref(cs), _ptr(w.gamma_pos), _ptr(w.gamma_neg), None, 0)
        _check(st, "lrq_tlq_quantize_pack_clip")
    return w


def ars_workspace_bytes(M: int, K: int, rot: Rotation, act_bits: int) -> int:
    r = rot.c_struct()
    return lib().lrq_ars_workspace_bytes(M, K, ctypes.byref(r), act_bits)


def workspace_bytes(M: int, N: int, K: int, rot: Rotation, act_bits: int, asym: bool = False) -> int:
    r = rot.c_struct()
    fn = lib().lrq_workspace_bytes_asym if asym else lib().lrq_workspace_bytes
    return fn(M, N, K, ctypes.byref(r), act_bits)


def ars_rotate_quant(X, rot: Rotation, act_bits: int, q=None, scale=None, workspace=None, asym: bool = False,
                     zero=None):
    """lrq_ars_rotate_quant: X bf16 [M, K] -> (q int8 [M, K], scale fp32 [M]);
    asym=True: lrq_ars_rotate_quant_asym -> (q, scale, zero int32 [M])."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    if q is None:
        q = torch.empty((M, K), dtype=torch.int8, device=X.device)
    if scale is None:
        scale = torch.empty(M, dtype=torch.float32, device=X.device)
    r = rot.c_struct()
    need = lib().lrq_ars_workspace_bytes(M, K, ctypes.byref(r), act_bits)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    nws = 0 if workspace is None else workspace.numel()
    if asym:
        if zero is None:
            zero = torch.empty(M, dtype=torch.int32, device=X.device)
        st = lib().lrq_ars_rotate_quant_asym(_stream(), _ptr(X), M, K, ctypes.byref(r), act_bits, _ptr(q), _ptr(scale),
                                             _ptr(zero), _ptr(workspace), nws)
        _check(st, "lrq_ars_rotate_quant_asym")
        return q, scale, zero
    st = lib().lrq_ars_rotate_quant(_stream(), _ptr(X), M, K, ctypes.byref(r), act_bits, _ptr(q), _ptr(scale),
                                    _ptr(workspace), nws)
    _check(st, "lrq_ars_rotate_quant")
    return q, scale


def ars_rotate_quant_packed4(X, rot: Rotation, q4=None, scale=None, workspace=None):
    """lrq_ars_rotate_quant_packed4: X bf16 [M, K] -> (q4 uint8 [M, K/2] packed 4-bit codes, scale fp32 [M])."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    if q4 is None:
        q4 = torch.empty((M, K // 2), dtype=torch.uint8, device=X.device)
    if scale is None:
        scale = torch.empty(M, dtype=torch.float32, device=X.device)
    r = rot.c_struct()
    need = lib().lrq_ars_workspace_bytes_packed4(M, K, ctypes.byref(r))
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    st = lib().lrq_ars_rotate_quant_packed4(_stream(), _ptr(X), M, K, ctypes.byref(r), _ptr(q4), _ptr(scale), _ptr(workspace),
                                            0 if workspace is None else workspace.numel())
    _check(st, "lrq_ars_rotate_quant_packed4")
    return q4, scale


def qgemm_packed4(q4, scale, w: TLQWeight, bias=None, out_dtype=None, out=None):
    """lrq_qgemm_packed4: the decode + GEMM + rescale stage on packed 4-bit activation codes [M, K/2]."""
    import torch
    assert q4.is_cuda and q4.dtype == torch.uint8 and q4.is_contiguous()
    M, K = q4.shape[0], q4.shape[1] * 2
    out_dtype = out_dtype or (out.dtype if out is not None else torch.bfloat16)
    if out is None:
        out = torch.empty((M, w.N), dtype=out_dtype, device=q4.device)
    cs = w.c_struct()
    st = lib().lrq_qgemm_packed4(_stream(), _ptr(q4), _ptr(scale), M, K, ctypes.byref(cs), _ptr(bias), _out_code(out_dtype), _ptr(out))
    _check(st, "lrq_qgemm_packed4")
    return out


def qlinear_packed4(X, rot: Rotation, w: TLQWeight, bias=None, out_dtype=None, out=None, workspace=None):
    """lrq_qlinear_packed4: the fused layer with 4-bit activation codes packed two per byte between its stages."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    out_dtype = out_dtype or (out.dtype if out is not None else torch.bfloat16)
    if out is None:
        out = torch.empty((M, w.N), dtype=out_dtype, device=X.device)
    r, cs = rot.c_struct(), w.c_struct()
    if workspace is None:
        workspace = torch.empty(lib().lrq_workspace_bytes_packed4(M, w.N, K, ctypes.byref(r)), dtype=torch.uint8, device=X.device)
    st = lib().lrq_qlinear_packed4(_stream(), _ptr(X), M, K, ctypes.byref(r), ctypes.byref(cs), _ptr(bias), _out_code(out_dtype),
                                   _ptr(out), _ptr(workspace), workspace.numel())
    _check(st, "lrq_qlinear_packed4")
    return out


def ars_rotate_quant_fp8(X, rot: Rotation, q8=None, scale=None, workspace=None):
    """lrq_ars_rotate_quant_fp8: X bf16 [M, K] -> (q8 uint8 [M, K] 4-bit codes as FP8 E4M3 bit patterns, scale fp32 [M])."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    if q8 is None:
        q8 = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    if scale is None:
        scale = torch.empty(M, dtype=torch.float32, device=X.device)
    r = rot.c_struct()
    need = lib().lrq_ars_workspace_bytes(M, K, ctypes.byref(r), 4)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    st = lib().lrq_ars_rotate_quant_fp8(_stream(), _ptr(X), M, K, ctypes.byref(r), _ptr(q8), _ptr(scale), _ptr(workspace),
                                        0 if workspace is None else workspace.numel())
    _check(st, "lrq_ars_rotate_quant_fp8")
    return q8, scale


def qgemm_fp8(q8, scale, w: TLQWeight, bias=None, out_dtype=None, out=None):
    """lrq_qgemm_fp8: decode + FP8 MFMA GEMM + rescale on activation codes held as E4M3 bytes [M, K]."""
    import torch
    assert q8.is_cuda and q8.dtype == torch.uint8 and q8.is_contiguous()
    M, K = q8.shape
    out_dtype = out_dtype or (out.dtype if out is not None else torch.bfloat16)
    if out is None:
        out = torch.empty((M, w.N), dtype=out_dtype, device=q8.device)
    cs = w.c_struct()
    st = lib().lrq_qgemm_fp8(_stream(), _ptr(q8), _ptr(scale), M, K, ctypes.byref(cs), _ptr(bias), _out_code(out_dtype), _ptr(out))
    _check(st, "lrq_qgemm_fp8")
    return out


def qlinear_fp8(X, rot: Rotation, w: TLQWeight, bias=None, out_dtype=None, out=None, workspace=None):
    """lrq_qlinear_fp8: the fused layer with FP8 E4M3 operands on both sides (4-bit activation codes)."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    out_dtype = out_dtype or (out.dtype if out is not None else torch.bfloat16)
    if out is None:
        out = torch.empty((M, w.N), dtype=out_dtype, device=X.device)
    r, cs = rot.c_struct(), w.c_struct()
    if workspace is None:
        workspace = torch.empty(lib().lrq_workspace_bytes(M, w.N, K, ctypes.byref(r), 4), dtype=torch.uint8, device=X.device)
    st = lib().lrq_qlinear_fp8(_stream(), _ptr(X), M, K, ctypes.byref(r), ctypes.byref(cs), _ptr(bias), _out_code(out_dtype),
                               _ptr(out), _ptr(workspace), workspace.numel())
    _check(st, "lrq_qlinear_fp8")
    return out


def ars_dense_prepare(R):
    """lrq_ars_dense_prepare: the preprocessing of a dense rotation matrix R (bf16 [K, K] on the device), to be kept in
    Rotation.prepared for as long as R's contents stay the same.  Returns a uint8 device tensor."""
    import torch
    K = R.shape[0]
    need = lib().lrq_ars_dense_prepared_bytes(K)
    if need == 0:
        raise LrqError(LRQ_EUNSUPPORTED, "lrq_ars_dense_prepared_bytes")
    out = torch.empty(need, dtype=torch.uint8, device=R.device)
    _check(lib().lrq_ars_dense_prepare(_stream(), _ptr(R), K, _ptr(out), need), "lrq_ars_dense_prepare")
    return out


def ars_dense_diagnostics(workspace, M: int, K: int):
    """Views into the workspace an LRQ_ROT_DENSE call of lrq_ars_rotate_quant used (lrq_ars_dense_diagnostics):
    (u~ fp32 [M, K], eps fp64 [M], undecided-element counts int32 [M], whole-row flags int32 [M])."""
    import torch
    offs = (ctypes.c_size_t * 4)()
    _check(lib().lrq_ars_dense_diagnostics(M, K, ctypes.byref(offs)), "lrq_ars_dense_diagnostics")
    u = workspace[offs[0]:offs[0] + M * K * 4].view(torch.float32).view(M, K)
    eps = workspace[offs[1]:offs[1] + M * 8].view(torch.float64)
    cnt = workspace[offs[2]:offs[2] + M * 4].view(torch.int32)
    whole = workspace[offs[3]:offs[3] + M * 4].view(torch.int32)
    return u, eps, cnt, whole


def _out_code(dtype) -> int:
    import torch
    return {torch.bfloat16: LRQ_OUT_BF16, torch.float32: LRQ_OUT_FP32}[dtype]


def qlinear(X, rot: Rotation, act_bits: int, w: TLQWeight, bias=None, out_dtype=None, out=None, workspace=None,
            asym: bool = False, levels: bool = False):
    """lrq_qlinear (asym=True: lrq_qlinear_asym; levels=True: lrq_qlinear_levels): fused rotate, quantize, decode,
    GEMM and rescale.  Returns Y [M, N]."""
    assert not (asym and levels)
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    out_dtype = out_dtype or (out.dtype if out is not None else torch.bfloat16)
    if out is None:
        out = torch.empty((M, w.N), dtype=out_dtype, device=X.device)
    r, cs = rot.c_struct(), w.c_struct()
    size_fn = lib().lrq_workspace_bytes_asym if asym else lib().lrq_workspace_bytes
    if workspace is None:
        workspace = torch.empty(size_fn(M, w.N, K, ctypes.byref(r), act_bits), dtype=torch.uint8, device=X.device)
    name = "lrq_qlinear_asym" if asym else ("lrq_qlinear_levels" if levels else "lrq_qlinear")
    st = getattr(lib(), name)(_stream(), _ptr(X), M, K, ctypes.byref(r), act_bits, ctypes.byref(cs), _ptr(bias),
                              _out_code(out_dtype), _ptr(out), _ptr(workspace), workspace.numel())
    _check(st, name)
    return out


def qlinear_static(X, rot: Rotation, act_bits: int, w: TLQWeight, out, bias=None):
    """lrq_qlinear_static: lrq_qlinear on the library's built-in scratch buffer (no workspace, no allocation: `out`
    must be given).  Returns `out`."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    assert out.shape == (M, w.N) and out.is_contiguous()
    r, cs = rot.c_struct(), w.c_struct()
    st = lib().lrq_qlinear_static(_stream(), _ptr(X), M, K, ctypes.byref(r), act_bits, ctypes.byref(cs), _ptr(bias),
                                  _out_code(out.dtype), _ptr(out))
    _check(st, "lrq_qlinear_static")
    return out


def qgemm(q, scale, w: TLQWeight, bias=None, out_dtype=None, out=None, zero=None, levels: bool = False):
    """lrq_qgemm (zero given: lrq_qgemm_asym; levels=True: lrq_qgemm_levels): the decode + GEMM + rescale stage on
    existing activation codes."""
    assert not (levels and zero is not None)
    import torch
    assert q.is_cuda and q.dtype == torch.int8 and q.is_contiguous()
    M, K = q.shape
    out_dtype = out_dtype or (out.dtype if out is not None else torch.bfloat16)
    if out is None:
        out = torch.empty((M, w.N), dtype=out_dtype, device=q.device)
    cs = w.c_struct()
    if zero is not None:
        st = lib().lrq_qgemm_asym(_stream(), _ptr(q), _ptr(scale), _ptr(zero), M, K, ctypes.byref(cs), _ptr(bias),
                                  _out_code(out_dtype), _ptr(out))
        _check(st, "lrq_qgemm_asym")
        return out
    name = "lrq_qgemm_levels" if levels else "lrq_qgemm"
    st = getattr(lib(), name)(_stream(), _ptr(q), _ptr(scale), M, K, ctypes.byref(cs), _ptr(bias), _out_code(out_dtype),
                              _ptr(out))
    _check(st, name)
    return out


def ars_build_rotation(Xcal, block: int, Rtilde, Q1, Q2) -> Rotation:
    """lrq_ars_build_rotation: calibration activations bf16 [T, K], Rtilde fp64 [B, B], Q1/Q2 fp64
    [K/B, n_steps, B, B] (all on the device) -> the "blockperm" Rotation (R1, perm, R2 device tensors)."""
    import torch
    assert Xcal.is_cuda and Xcal.dtype == torch.bfloat16 and Xcal.is_contiguous()
    T, K = Xcal.shape
    for a in (Rtilde, Q1, Q2):
        assert a.is_cuda and a.dtype == torch.float64 and a.is_contiguous()
    assert Q1.shape == Q2.shape and Q1.dim() == 4
    n_steps = Q1.shape[1]
    nb = K // block if block > 0 else 0
    R1 = torch.empty((max(nb, 1), block, block), dtype=torch.bfloat16, device=Xcal.device)
    R2 = torch.empty_like(R1)
    perm = torch.empty(K, dtype=torch.int32, device=Xcal.device)
    need = lib().lrq_ars_build_workspace_bytes(T, K, block)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=Xcal.device)
    _check(lib().lrq_ars_build_rotation(_stream(), _ptr(Xcal), T, K, block, n_steps, _ptr(Rtilde), _ptr(Q1), _ptr(Q2),
                                        _ptr(R1), _ptr(perm), _ptr(R2), _ptr(ws), ws.numel()), "lrq_ars_build_rotation")
    return Rotation("blockperm", block=block, R1=R1, perm=perm, R2=R2)


def smooth_factor(Xcal, W, alpha: float = 0.5, smooth_weights: bool = True):
    """lrq_smooth_factor: Xcal bf16 [T, K], W fp32 [N, K] on the device -> (s fp32 [K], inv_s fp32 [K],
    W * s fp32 [N, K] or None)."""
    import torch
    assert Xcal.is_cuda and Xcal.dtype == torch.bfloat16 and Xcal.is_contiguous()
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.shape[1] == Xcal.shape[1]
    T, K = Xcal.shape
    s = torch.empty(K, dtype=torch.float32, device=W.device)
    inv = torch.empty_like(s)
    Wout = torch.empty_like(W) if smooth_weights else None
    ws = torch.empty(max(lib().lrq_smooth_workspace_bytes(K), 16), dtype=torch.uint8, device=W.device)
    _check(lib().lrq_smooth_factor(_stream(), _ptr(Xcal), T, _ptr(W), W.shape[0], K, float(alpha), _ptr(s), _ptr(inv),
                                   _ptr(Wout), _ptr(ws), ws.numel()), "lrq_smooth_factor")
    return s, inv, Wout


def fluctuation_metric(X):
    """lrq_fluctuation_metric: X bf16 [M, K] on the device -> J as a device tensor double[1]."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    M, K = X.shape
    J = torch.empty(1, dtype=torch.float64, device=X.device)
    ws = torch.empty(lib().lrq_fluctuation_workspace_bytes(), dtype=torch.uint8, device=X.device)
    _check(lib().lrq_fluctuation_metric(_stream(), _ptr(X), M, K, _ptr(J), _ptr(ws), ws.numel()), "lrq_fluctuation_metric")
    return J


def ars_select(J: float, threshold: float = 1.0) -> str:
    """lrq_ars_select: "hadamard" if J < threshold else "blockperm"."""
    k = lib().lrq_ars_select(float(J), float(threshold))
    _check(min(k, 0), "lrq_ars_select")
    return {LRQ_ROT_HADAMARD: "hadamard", LRQ_ROT_BLOCKPERM: "blockperm"}[k]
