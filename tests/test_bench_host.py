"""Host-side logic of bench.py that needs no GPU: the one-GPU rule, the flags, the oracle baseline leg."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_defaults_follow_the_contract(monkeypatch):
    monkeypatch.setattr(sys, "argv", ["bench.py"])
    a = bench.parse()
    assert a.gpus == 1 and a.workload == "c4"             # the largest configuration: the one the metric is quoted on
    assert a.steps == 0 and a.warmup == -1                # sized from a pilot run
    monkeypatch.setattr(sys, "argv", ["bench.py", "--gpus", "1", "--steps", "7", "--warmup", "3"])
    a = bench.parse()
    assert (a.steps, a.warmup) == (7, 3)


def test_published_peaks():
    assert bench.INT8_MFMA_PEAK_TOPS == 5000.0 and bench.BF16_MFMA_PEAK_TFLOPS == 2500.0
    assert bench.HBM_PEAK_GBS == 8000.0 and bench.FP64_VEC_PEAK_TFLOPS == 78.6


def test_oracle_baseline_leg_on_a_tiny_sample():
    specs = synth.config_layers(1)
    out = bench.cpu_baseline(specs, rows=32, channels=48)
    assert out["kind"] == "oracle" and out["unit"] == "TOPS" and out["cores"] >= 1
    assert out["value"] > 0 and "32 token rows" in out["sample"] and "48 output channels" in out["sample"]
    # ops are counted as 2 M N K of the sample actually run: a bound that holds whatever the host's speed
    # (a few milliseconds of work at most a second long on any host)
    s = specs[0]
    assert out["value"] >= 2 * 32 * 48 * s.K / 1.0 / 1e12
