"""The byte accounting behind bench.py's roofline figures, checked against hand-computed values.

Algorithmic bytes of a decode step = weights of the active layers + the valid KV entries those layers read + the
LM head (bf16).  The expected figures below were worked out by hand from the shapes (OPT-6.7B: d = 4096, f = 16384,
V = 50272; per-layer matrices 12 d^2 * 2 bytes = 402.65 MB, LM head 411.83 MB) and the Section 2.3 schedule.
"""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import synth_inputs as S  # noqa: E402
from oracle import oracle as ORA  # noqa: E402


def _totals(name):
    shape, B, P, T, n_min, n_max, ragged, *rest = bench.WORKLOADS[name]
    assert ragged is None and not rest
    n = [ORA.schedule(P + k, P, P + T, n_min, n_max, shape.L) for k in range(T)]
    sum_len = [(P + k + 1) * B for k in range(T)]
    skip = sum(bench.step_bytes(shape, n[k], sum_len[k]) for k in range(T))
    full = sum(bench.step_bytes(shape, shape.L, sum_len[k]) for k in range(T))
    return shape, T, n, skip, full


def test_matrix_bytes_per_layer_and_head():
    s = S.OPT_6_7B
    assert bench.class_bytes(s, "gemm_qkv", 0) == 100_663_296
    assert bench.class_bytes(s, "gemm_out", 0) == 33_554_432
    assert bench.class_bytes(s, "gemm_ffn1", 0) == 134_217_728 == bench.class_bytes(s, "gemm_ffn2", 0)
    assert bench.class_bytes(s, "lm_head", 0) == 411_828_224
    # one key and one value vector of d bf16 elements per cached position and row
    assert bench.class_bytes(s, "attention", 32 * 513) == 32 * 513 * 2 * 4096 * 2
    # a step with no layers is the LM head alone; one more layer adds its matrices (+ fp32 vectors) and its KV
    assert bench.step_bytes(s, 0, 12345) == 411_828_224
    per_layer = bench.step_bytes(s, 1, 0) - bench.step_bytes(s, 0, 0)
    assert per_layer == 402_653_184 + 4 * (9 * 4096 + 16384)  # biases and LayerNorm vectors stay fp32
    assert bench.step_bytes(s, 3, 1000) - bench.step_bytes(s, 3, 0) == 3 * 1000 * 2 * 4096 * 2


@pytest.mark.parametrize("name,sum_n,skip_gb,full_gb,layer_ratio", [
    ("opt6.7b_b32_p512_t256_32to6", 4878, 14.19, 24.05, 1.679),
    ("opt6.7b_b8_p2048_t512_32to12", 11276, 15.82, 22.97, 1.453),
    ("opt1.3b_b16_p256_t256_24to12", 4616, 2.90, 3.83, 1.331),
])
def test_step_bytes_of_the_contract_workloads(name, sum_n, skip_gb, full_gb, layer_ratio):
    shape, T, n, skip, full = _totals(name)
    assert sum(n) == sum_n
    assert abs(skip / T / 1e9 - skip_gb) < 0.01
    assert abs(full / T / 1e9 - full_gb) < 0.01
    assert abs(shape.L * T / sum(n) - layer_ratio) < 5e-4


def test_more_than_one_gpu_is_refused():
    import subprocess
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.parametrize("name", ["opt6.7b_b32_p512_t256_32to6", "opt6.7b_b8_p2048_t512_32to12",
                                  "opt1.3b_b16_p256_t256_24to12", "opt6.7b_b128_p64-512_t128_24to8"])
@pytest.mark.parametrize("steps", [5, 20, 33])
def test_timed_sample_has_the_schedules_mean_depth(name, steps):
    # with fewer timed steps than the generation has, the timed positions are the mid-points of equal strata: strictly
    # increasing, inside the generation, and their mean layer count is the schedule's (not that of its first steps)
    shape, B, P, T, n_min, n_max, *_ = bench.WORKLOADS[name]
    ks = bench.sample_positions(T, steps)
    assert len(ks) == steps and ks == sorted(set(ks)) and 0 <= ks[0] and ks[-1] < T
    n_all = [ORA.schedule(P + k, P, P + T, n_min, n_max, shape.L) for k in range(T)]
    mean_all, mean_sample = np.mean(n_all), np.mean([n_all[k] for k in ks])
    assert abs(mean_sample - mean_all) <= 0.02 * mean_all + 0.5 / steps * (n_max - n_min)
    assert bench.sample_positions(T, T) == list(range(T)) == bench.sample_positions(T, T + 7)
