"""lrq_qlinear_static: the entry point that allocates nothing (its activation codes, scales and rotation scratch live
in a fixed buffer inside the library) against lrq_qlinear, through the C ABI.  Two calls in a row on the same buffer,
the second on a smaller input; same kernels, so the outputs must be identical bit for bit."""
import ctypes

import numpy as np
import pytest

import synth
from gpu_util import bf16_to_dev, to_dev

pytestmark = pytest.mark.gpu
GRID = synth.DEFAULT_GRID


@pytest.fixture(scope="module")
def lrq():
    import torch
    assert torch.cuda.is_available()
    import paper_2508_03485_amd as m
    m.lib()
    return m


def _layer(lrq, M, K, N, w_bits, seed):
    X = bf16_to_dev(synth.make_activations(M, K, (940, seed, 0), 0.05, 6, 40.0))
    W = to_dev(synth.make_weights(N, K, (940, seed, 1)))
    gd = to_dev(GRID)
    return X, lrq.tlq_quantize_pack(W, w_bits, 7, gd, gd), to_dev(synth.make_bias(N, (940, seed, 2)))


def test_static_scratch_entry_point_matches_the_workspace_one(lrq):
    import torch
    L = lrq.lib()
    assert L.lrq_init() == lrq.LRQ_OK
    cap = L.lrq_static_scratch_bytes()
    assert cap == 64 << 20
    st = torch.cuda.current_stream().cuda_stream
    cases = [(700, 1152, 416, 4, 8, lrq.Rotation("hadamard", 128), torch.bfloat16),       # first call
             (129, 512, 200, 3, 4, lrq.Rotation("hadamard", 512), torch.float32)]         # smaller, other kernels
    R = bf16_to_dev(synth.make_rotation(256, (940, 9, 0)))
    cases.append((90, 256, 96, 4, 8, lrq.Rotation("dense", 0, R), torch.bfloat16))         # rotation scratch in the buffer too
    for i, (M, K, N, wb, ab, rot, dt) in enumerate(cases):
        print(f"case static M={M} K={K} N={N} W{wb}A{ab} {rot.kind}", flush=True)
        X, w, bias = _layer(lrq, M, K, N, wb, i)
        ref = lrq.qlinear(X, rot, ab, w, bias=bias, out_dtype=dt)
        out = torch.full((M, N), float("nan"), dtype=dt, device="cuda")
        r, cs = rot.c_struct(), w.c_struct()
        code = L.lrq_qlinear_static(st, X.data_ptr(), M, K, ctypes.byref(r), ab, ctypes.byref(cs), bias.data_ptr(),
                                    lrq.LRQ_OUT_BF16 if dt == torch.bfloat16 else lrq.LRQ_OUT_FP32, out.data_ptr())
        assert code == lrq.LRQ_OK, lrq.status_string(code)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
    # a layer that does not fit the buffer is refused before anything is launched
    M, K = 35100, 3072
    w = lrq._TlqWeight(N=64, K=K, bits=4, I=7, codes=4096, s_pos=4096, s_neg=4096, z_pos=4096, z_neg=4096, alpha=4096,
                       beta=4096, lut=4096, wscale=4096, gemm_codes=4096, colsum=4096)
    had = lrq.Rotation("hadamard", 1024).c_struct()
    assert L.lrq_workspace_bytes(M, 64, K, ctypes.byref(had), 8) > cap
    assert L.lrq_qlinear_static(st, 4096, M, K, ctypes.byref(had), 8, ctypes.byref(w), None, 0, 4096) == lrq.LRQ_ESCRATCH
    assert "built-in" in lrq.status_string(lrq.LRQ_ESCRATCH)
