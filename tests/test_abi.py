"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything would be launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2508_03485_amd as lrq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(lrq.LIB_PATH):
        from paper_2508_03485_amd.build import build
        build()
    return lrq.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "lrq.h")).read()
    declared = set(re.findall(r"\b(lrq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(lrq.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.lrq_version() >= 100
    assert lrq.status_string(0) == "ok" and "workspace" in lrq.status_string(lrq.LRQ_EWORKSPACE)


def test_sizes(L):
    assert L.lrq_tlq_codes_bytes(1152, 1152, 4) == 1152 * 1152 // 2
    assert L.lrq_tlq_codes_bytes(1152, 1152, 3) == 1152 * 1152 * 3 // 8
    assert L.lrq_tlq_codes_bytes(8, 12, 4) == 0 and L.lrq_tlq_codes_bytes(8, 16, 5) == 0
    assert L.lrq_tlq_gemm_codes_bytes(1152, 1152, 4) == 1152 * 1152 // 2
    assert L.lrq_tlq_gemm_codes_bytes(33, 64, 3) == 64 * 64 // 2              # channels padded to 32; a nibble per code
    had = lrq.Rotation("hadamard", 128).c_struct()
    assert L.lrq_ars_workspace_bytes(256, 1152, ctypes.byref(had), 8) == 0
    dense = lrq._Rotation(lrq.LRQ_ROT_DENSE, 0, 4096)
    assert L.lrq_ars_workspace_bytes(256, 1152, ctypes.byref(dense), 8) >= 256 * 1152 * 8
    assert L.lrq_workspace_bytes(256, 64, 1152, ctypes.byref(had), 8) >= 256 * 1152 + 256 * 4


def test_rotate_quant_rejects_bad_arguments_on_the_host(L):
    P = 4096   # any aligned non-null value: validation must fail before the pointer is ever used
    had = lambda h: ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_HADAMARD, h, None))
    f = L.lrq_ars_rotate_quant
    assert f(None, None, 4, 128, had(128), 8, P, P, None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 0, 128, had(128), 8, P, P, None, 0) == lrq.LRQ_EINVAL
    assert f(None, P + 2, 4, 128, had(128), 8, P, P, None, 0) == lrq.LRQ_EINVAL          # misaligned
    assert f(None, P, 4, 128, None, 8, P, P, None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 4, 128, had(128), 5, P, P, None, 0) == lrq.LRQ_EUNSUPPORTED        # act bits
    assert f(None, P, 4, 132, had(4), 8, P, P, None, 0) == lrq.LRQ_EUNSUPPORTED          # K % 8
    assert f(None, P, 4, 1152, had(96), 8, P, P, None, 0) == lrq.LRQ_EUNSUPPORTED        # not a power of two
    assert f(None, P, 4, 1152, had(256), 8, P, P, None, 0) == lrq.LRQ_EUNSUPPORTED       # does not divide K
    assert f(None, P, 4, 1152, had(0), 8, P, P, None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 4, 1152, had(128), 8, None, P, None, 0) == lrq.LRQ_EINVAL
    dense = ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_DENSE, 0, P))
    assert f(None, P, 4, 1152, dense, 8, P, P, None, 0) == lrq.LRQ_EWORKSPACE
    assert f(None, P, 4, 1152, dense, 8, P, P, P, 16) == lrq.LRQ_EWORKSPACE
    assert f(None, P, 4, 1152, ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_DENSE, 0, None)), 8, P, P, P, 1 << 30) == lrq.LRQ_EINVAL
    assert f(None, P, 4, 1152, ctypes.byref(lrq._Rotation(7, 0, None)), 8, P, P, None, 0) == lrq.LRQ_EINVAL


def _weight(N=64, K=128, bits=4, I=7, p=4096, **over):
    kw = dict(N=N, K=K, bits=bits, I=I, codes=p, s_pos=p, s_neg=p, z_pos=p, z_neg=p, alpha=p, beta=p, lut=p,
              wscale=p, gemm_codes=p, colsum=p)
    kw.update(over)
    return lrq._TlqWeight(**kw)


def test_quantize_pack_rejects_bad_arguments_on_the_host(L):
    P = 4096
    f = L.lrq_tlq_quantize_pack
    ok = _weight()
    assert f(None, None, 64, 128, 4, 7, P, 21, P, 21, ctypes.byref(ok), None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 64, 128, 4, 7, P, 0, P, 21, ctypes.byref(ok), None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 64, 128, 4, 7, P, 65, P, 21, ctypes.byref(ok), None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 64, 128, 5, 7, P, 21, P, 21, ctypes.byref(_weight(bits=5)), None, 0) == lrq.LRQ_EUNSUPPORTED
    assert f(None, P, 64, 128, 4, 7, P, 21, P, 21, ctypes.byref(_weight(N=32)), None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 64, 128, 4, 7, P, 21, P, 21, ctypes.byref(_weight(lut=None)), None, 0) == lrq.LRQ_EINVAL
    assert f(None, P, 64, 72, 4, 7, P, 21, P, 21, ctypes.byref(_weight(K=72)), None, 0) == lrq.LRQ_EUNSUPPORTED
    assert f(None, P, 64, 32768, 4, 7, P, 21, P, 21, ctypes.byref(_weight(K=32768)), None, 0) == lrq.LRQ_EUNSUPPORTED
    assert f(None, P, 64, 128, 4, 7, P, 21, P, 21, None, None, 0) == lrq.LRQ_EINVAL


def test_qlinear_rejects_bad_arguments_on_the_host(L):
    P = 4096
    had = ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_HADAMARD, 128, None))
    f = L.lrq_qlinear
    w = ctypes.byref(_weight())
    big = 1 << 30
    assert f(None, P, 16, 128, had, 8, w, None, 0, None, P, big) == lrq.LRQ_EINVAL            # Y null
    assert f(None, P, 16, 256, had, 8, w, None, 0, P, P, big) == lrq.LRQ_EINVAL               # K mismatch
    assert f(None, P, 16, 128, had, 8, w, None, 3, P, P, big) == lrq.LRQ_EUNSUPPORTED         # out dtype
    assert f(None, P, 16, 128, had, 8, w, None, 0, P, None, 0) == lrq.LRQ_EWORKSPACE
    assert f(None, P, 16, 128, had, 8, w, None, 0, P, P, 100) == lrq.LRQ_EWORKSPACE
    assert f(None, P, 16, 128, had, 8, None, None, 0, P, P, big) == lrq.LRQ_EINVAL
    assert f(None, P, 16, 128, had, 8, ctypes.byref(_weight(bits=2)), None, 0, P, P, big) == lrq.LRQ_EUNSUPPORTED
    g = L.lrq_qgemm
    assert g(None, None, P, 16, 128, w, None, 0, P) == lrq.LRQ_EINVAL
    assert g(None, P, P, 16, 128, w, None, 9, P) == lrq.LRQ_EUNSUPPORTED
    w96 = ctypes.byref(_weight(K=96))
    assert g(None, P, P, 16, 96, w96, None, 0, P) == lrq.LRQ_EUNSUPPORTED                    # K % 64


def test_levels_entry_points_validate_on_the_host(L):
    P = 4096
    had = ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_HADAMARD, 128, None))
    big = 1 << 30
    g, f = L.lrq_qgemm_levels, L.lrq_qlinear_levels
    no_table = ctypes.byref(_weight())                                # levels == NULL
    assert g(None, P, P, 16, 128, no_table, None, 0, P) == lrq.LRQ_EINVAL
    assert f(None, P, 16, 128, had, 8, no_table, None, 0, P, P, big) == lrq.LRQ_EINVAL
    for I in (8, -1):                                                 # levels that are not bf16 values
        w = ctypes.byref(_weight(I=I, levels=P))
        assert g(None, P, P, 16, 128, w, None, 0, P) == lrq.LRQ_EUNSUPPORTED
        assert f(None, P, 16, 128, had, 8, w, None, 0, P, P, big) == lrq.LRQ_EUNSUPPORTED
    w = ctypes.byref(_weight(levels=P))
    assert g(None, None, P, 16, 128, w, None, 0, P) == lrq.LRQ_EINVAL                       # q null
    assert g(None, P, P, 16, 128, w, None, 7, P) == lrq.LRQ_EUNSUPPORTED                    # out dtype
    assert g(None, P, P, 16, 128, ctypes.byref(_weight(levels=P + 2)), None, 0, P) == lrq.LRQ_EINVAL   # misaligned table
    assert f(None, P, 16, 128, had, 8, w, None, 0, P, None, 0) == lrq.LRQ_EWORKSPACE
    assert f(None, P, 16, 256, had, 8, w, None, 0, P, P, big) == lrq.LRQ_EINVAL             # K mismatch


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(lrq, "_lib", None)
    monkeypatch.setattr(lrq, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError, match="no fallback"):
        lrq.lib()


def test_zero_point_variants_reject_bad_arguments_on_the_host(L):
    P = 4096
    had = ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_HADAMARD, 128, None))
    w = ctypes.byref(_weight())
    big = 1 << 30
    assert L.lrq_ars_rotate_quant_asym(None, P, 4, 128, had, 8, P, P, None, None, 0) == lrq.LRQ_EINVAL      # zero null
    assert L.lrq_ars_rotate_quant_asym(None, P, 4, 128, had, 5, P, P, P, None, 0) == lrq.LRQ_EUNSUPPORTED
    assert L.lrq_qgemm_asym(None, P, P, None, 16, 128, w, None, 0, P) == lrq.LRQ_EINVAL
    assert L.lrq_qgemm_asym(None, P, P, P, 16, 128, ctypes.byref(_weight(colsum=None)), None, 0, P) == lrq.LRQ_EINVAL
    need = L.lrq_workspace_bytes_asym(16, 64, 128, had, 8)
    assert need >= L.lrq_workspace_bytes(16, 64, 128, had, 8) + 16 * 4
    assert L.lrq_qlinear_asym(None, P, 16, 128, had, 8, w, None, 0, P, P, need - 1) == lrq.LRQ_EWORKSPACE
    assert L.lrq_qlinear_asym(None, P, 16, 128, had, 8, w, None, 0, None, P, big) == lrq.LRQ_EINVAL


def test_structured_rotation_is_validated_on_the_host(L):
    P = 4096
    def rot(block=128, R1=P, perm=P, R2=P):
        return ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_BLOCKPERM, 0, None, block, R1, perm, R2))
    need = L.lrq_ars_workspace_bytes(16, 256, rot(), 8)
    assert need >= 16 * 256 * (8 + 4)                    # fp64 U plus the permuted fp32 intermediate
    assert L.lrq_ars_rotate_quant(None, P, 16, 256, rot(), 8, P, P, P, need - 1) == lrq.LRQ_EWORKSPACE
    assert L.lrq_ars_rotate_quant(None, P, 16, 256, rot(R1=None), 8, P, P, P, need) == lrq.LRQ_EINVAL
    assert L.lrq_ars_rotate_quant(None, P, 16, 256, rot(perm=None), 8, P, P, P, need) == lrq.LRQ_EINVAL
    assert L.lrq_ars_rotate_quant(None, P, 16, 256, rot(R2=P + 2), 8, P, P, P, need) == lrq.LRQ_EINVAL   # misaligned
    assert L.lrq_ars_rotate_quant(None, P, 16, 256, rot(block=0), 8, P, P, P, need) == lrq.LRQ_EINVAL
    assert L.lrq_ars_rotate_quant(None, P, 16, 256, rot(block=64), 8, P, P, P, need) == lrq.LRQ_EUNSUPPORTED
    assert L.lrq_ars_rotate_quant(None, P, 16, 384, rot(block=256), 8, P, P, P, 1 << 30) == lrq.LRQ_EUNSUPPORTED


def test_calibration_entry_points_validate_on_the_host(L):
    P = 4096
    need = L.lrq_ars_build_workspace_bytes(64, 256, 128)
    assert need >= 2 * 64 * 256 * 8 + 256 * 128 * 8
    assert L.lrq_ars_build_workspace_bytes(64, 250, 128) == 0
    ok_args = (None, P, 64, 256, 128, 2, P, P, P, P, P, P, P, need)
    def call(**kw):
        a = list(ok_args)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return L.lrq_ars_build_rotation(*a)
    assert call(_1=None) == lrq.LRQ_EINVAL               # Xcal
    assert call(_6=None) == lrq.LRQ_EINVAL               # Rtilde
    assert call(_10=None) == lrq.LRQ_EINVAL              # perm
    assert call(_5=0) == lrq.LRQ_EINVAL                  # n_steps
    assert call(_4=64) == lrq.LRQ_EUNSUPPORTED           # block not a multiple of 128
    assert call(_3=384, _4=256) == lrq.LRQ_EUNSUPPORTED  # block does not divide K
    assert call(_13=need - 1) == lrq.LRQ_EWORKSPACE
    nj = L.lrq_fluctuation_workspace_bytes()
    assert nj > 0
    assert L.lrq_fluctuation_metric(None, None, 4, 64, P, P, nj) == lrq.LRQ_EINVAL
    assert L.lrq_fluctuation_metric(None, P, 3, 3, P, P, nj) == lrq.LRQ_EUNSUPPORTED
    assert L.lrq_fluctuation_metric(None, P, 4, 64, P, P, nj - 1) == lrq.LRQ_EWORKSPACE


def test_threshold_rule_runs_on_the_host(L):
    # Method, ARS case equation: Hadamard below the threshold, the dual transformation at or above it
    assert L.lrq_ars_select(0.5, 1.0) == lrq.LRQ_ROT_HADAMARD
    assert L.lrq_ars_select(1.0, 1.0) == lrq.LRQ_ROT_BLOCKPERM
    assert L.lrq_ars_select(7.0, 1.0) == lrq.LRQ_ROT_BLOCKPERM
    assert L.lrq_ars_select(float("nan"), 1.0) == lrq.LRQ_EINVAL
    assert lrq.ars_select(0.2) == "hadamard" and lrq.ars_select(1.5) == "blockperm"


def test_smoothing_entry_point_validates_on_the_host(L):
    P = 4096
    need = L.lrq_smooth_workspace_bytes(256)
    assert need >= 2 * 256 * 4
    ok = [None, P, 32, P, 16, 256, 0.5, P, P, None, P, need]
    def call(i=None, v=None):
        a = list(ok)
        if i is not None:
            a[i] = v
        return L.lrq_smooth_factor(*a)
    assert call(1, None) == lrq.LRQ_EINVAL
    assert call(7, None) == lrq.LRQ_EINVAL
    assert call(6, float("nan")) == lrq.LRQ_EINVAL
    assert call(6, 1.5) == lrq.LRQ_EUNSUPPORTED
    assert call(5, 250) == lrq.LRQ_EUNSUPPORTED
    assert call(11, need - 1) == lrq.LRQ_EWORKSPACE
    # a misaligned pre-scale vector in the rotation struct
    rot = ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_HADAMARD, 128, None, 0, None, None, None, P + 4))
    assert L.lrq_ars_rotate_quant(None, P, 4, 128, rot, 8, P, P, None, 0) == lrq.LRQ_EINVAL


def test_lower_clip_entry_point_validates_on_the_host(L):
    P = 4096
    w = ctypes.byref(_weight())
    ok = [None, P, 64, 128, 4, 7, P, 3, P, 3, P, 5, w, None, None, None, 0]
    def call(i=None, v=None):
        a = list(ok)
        if i is not None:
            a[i] = v
        return L.lrq_tlq_quantize_pack_clip(*a)
    assert call(10, None) == lrq.LRQ_EINVAL          # gamma grid missing
    assert call(11, 0) == lrq.LRQ_EINVAL
    assert call(11, 65) == lrq.LRQ_EINVAL
    assert call(1, None) == lrq.LRQ_EINVAL
    assert call(4, 5) == lrq.LRQ_EUNSUPPORTED


def test_dense_prepare_validates_on_the_host(L):
    P = 4096
    assert L.lrq_ars_dense_prepared_bytes(3072) >= 2 * 3072 * 3072 + 4 * 3072
    assert L.lrq_ars_dense_prepared_bytes(192) == 0          # K % 128 != 0: the fp64 evaluation serves it, nothing to prepare
    assert L.lrq_ars_dense_prepared_bytes(32768) == 0
    f = L.lrq_ars_dense_prepare
    big = 1 << 30
    assert f(None, None, 256, P, big) == lrq.LRQ_EINVAL
    assert f(None, P, 256, None, big) == lrq.LRQ_EINVAL
    assert f(None, P, 0, P, big) == lrq.LRQ_EINVAL
    assert f(None, P, 192, P, big) == lrq.LRQ_EUNSUPPORTED
    assert f(None, P, 256, P, 100) == lrq.LRQ_EINVAL          # short buffer
    assert f(None, P, 256, P + 16, big) == lrq.LRQ_EINVAL     # not 256-byte aligned
    # a rotation that carries a misaligned prepared buffer is refused before anything is launched
    bad = ctypes.byref(lrq._Rotation(lrq.LRQ_ROT_DENSE, 0, P, 0, None, None, None, None, P + 16))
    assert L.lrq_ars_rotate_quant(None, P, 128, 256, bad, 8, P, P, P, big) == lrq.LRQ_EINVAL


def test_header_is_plain_c(tmp_path):
    """include/lrq.h is a C header: it compiles as C99 with no torch, HIP or C++ types in its signatures."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler on this host")
    src = tmp_path / "use_header.c"
    src.write_text('#include "lrq.h"\nint main(void) { lrq_rotation r = {0}; lrq_tlq_weight w = {0}; (void)r; (void)w; return 0; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I" + inc, "-fsyntax-only", str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    # the ctypes mirrors used by the binding have the C structs' sizes
    probe = tmp_path / "sizes.c"
    probe.write_text('#include <stdio.h>\n#include "lrq.h"\nint main(void) { printf("%zu %zu\\n", sizeof(lrq_rotation), sizeof(lrq_tlq_weight)); return 0; }\n')
    exe = tmp_path / "sizes"
    r = subprocess.run([gcc, "-std=c99", "-I" + inc, str(probe), "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    a, b = (int(v) for v in subprocess.run([str(exe)], capture_output=True, text=True).stdout.split())
    assert a == ctypes.sizeof(lrq._Rotation) and b == ctypes.sizeof(lrq._TlqWeight)
