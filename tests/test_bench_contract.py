"""CPU-side checks of bench.py's contract: the algorithmic work it divides by
(pinned to the per-minibatch totals derived from the configurations' shapes:
24*N*D^2 per layer for the linear layers with d_ffn = 4*d_model, 4*N*s_eff*D
for attention, 2*N*D*V for the LM head, backward twice forward), the published
peaks, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


@pytest.mark.parametrize("k,expected", [(2, 1.34e12), (3, 1.95e12), (4, 7.89e12), (5, 1.03e13)])
def test_algorithmic_flops_per_minibatch(k, expected):
    got = bench.algorithmic_flops_per_minibatch(W.CONFIGS[k])
    assert abs(got - expected) / expected < 5e-3, got


def test_flops_by_hand_for_the_smallest_configuration():
    w = W.CONFIGS[1]                   # one causal layer, d_model 128, d_ffn 512, 2 sequences of 64
    N, D, F, s = 128, 128, 512, 64
    fwd = 2 * N * (4 * D * D + 2 * D * F) + 4 * N * ((s + 1) / 2) * D
    assert bench.algorithmic_flops_per_minibatch(w) == pytest.approx(3 * fwd, rel=1e-12)


def test_published_peaks():
    assert bench.PEAK_BF16_TFLOPS == 2500.0 and bench.PEAK_HBM_GBS == 8000.0 and bench.PEAK_FP32_TFLOPS == 157.3


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_default_workload_is_the_largest_configuration_and_nothing_comes_from_tests():
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert 'default="5"' in src
    assert "from tests" not in src and "import tests" not in src
    # the oracle is imported inside cpu_baseline() only
    head, tail = src.split("def cpu_baseline", 1)
    assert "oracle" not in head.replace("CPU oracle", "").replace("the oracle", "") and "from oracle" in tail
