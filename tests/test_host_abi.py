"""CPU-side checks of the C ABI: every declared symbol is exported, the
library's schedule equals the oracle's on every position (two independent
implementations of Section 2.3 / 2.4), and configuration errors are reported
before any device work."""
import ctypes as C
import os
import random
import re

import pytest

from oracle import oracle as O
from paper_2307_02628_amd import _build, skd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(skd.LIB_PATH):
        _build.build(force=True)


def test_header_symbols_exported():
    text = open(os.path.join(ROOT, "include", "skd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(skd_[a-z_0-9]+)\s*\(", text)))
    assert len(names) >= 12
    lib = C.CDLL(skd.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in skd.h but not exported"
    assert sorted(skd.EXPORTS) == names


def test_schedule_matches_oracle_everywhere():
    rng = random.Random(5)
    cases = [(4, 16, 32, 2, 4), (24, 256, 512, 12, 24), (32, 512, 768, 6, 32), (32, 2048, 2560, 12, 32),
             (32, 512, 640, 8, 24), (12, 20, 100, 2, 8)]
    for _ in range(200):
        L = rng.randint(1, 48)
        n_max = rng.randint(1, L)
        n_min = rng.randint(1, n_max)
        P = rng.randint(0, 200)
        cases.append((L, P, P + rng.randint(1, 400), n_min, n_max))
    for L, P, N, n_min, n_max in cases:
        for i in range(-1, N + 2):
            assert skd.skd_schedule(i, P, N, n_min, n_max, L) == O.schedule_rc(i, P, N, n_min, n_max, L)


def test_active_layers_match_oracle():
    class Sh:
        pass
    rng = random.Random(6)
    for _ in range(100):
        L = rng.randint(1, 40)
        n_max = rng.randint(1, L)
        n_min = rng.randint(1, n_max)
        w = rng.randint(0, n_min)
        P = rng.randint(1, 50)
        N = P + rng.randint(1, 120)
        cfg = skd.Config(L, 64, 1, 64, 10, N, 1, P, N, n_min, n_max, w, 0, 0, 0)
        for i in range(N + 1):
            assert skd.skd_active_layers(i, cfg) == O.active_layers(i, P, N, n_min, n_max, w, L)


def test_error_codes():
    assert skd.skd_schedule(0, 10, 10, 1, 2, 4) == skd.ERR_SHAPE
    assert skd.skd_schedule(0, 10, 20, 0, 2, 4) == skd.ERR_SHAPE
    assert skd.skd_schedule(0, 10, 20, 3, 2, 4) == skd.ERR_SHAPE
    assert skd.skd_schedule(0, 10, 20, 1, 5, 4) == skd.ERR_SHAPE
    assert skd.skd_schedule(21, 10, 20, 1, 2, 4) == skd.ERR_RANGE
    assert skd.skd_schedule(-1, 10, 20, 1, 2, 4) == skd.ERR_RANGE
    assert skd.skd_schedule(20, 10, 20, 1, 2, 4) == 1
    lib = skd.lib()
    assert lib.skd_active_layers(0, None, None) == skd.ERR_NULL
    assert lib.skd_strerror(skd.ERR_ORDER).decode() == "call out of sequence"
    h = C.c_void_p()
    w = skd.Weights()
    bad = [
        skd.Config(4, 250, 4, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.FP32, 0),    # d % heads
        skd.Config(4, 256, 4, 64, 10, 32, 1, 8, 8, 1, 2, 0, 0, skd.FP32, 0),    # N == P
        skd.Config(4, 256, 4, 64, 10, 7, 1, 4, 8, 1, 2, 0, 0, skd.FP32, 0),     # max_pos < N
        skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 3, 2, 0, 0, skd.FP32, 0),    # n_min > n_max
        skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 5, 0, 0, skd.FP32, 0),    # n_max > L
        skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 2, 2, 0, skd.FP32, 0),    # warmup > n_min
        skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 2, 0, 48, skd.FP32, 0),   # page_tokens % 32
        skd.Config(4, 256, 8, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.BF16, 0),    # bf16 path: head_dim 32
        skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, 7, 0),           # unknown dtype
        skd.Config(4, 256, 4, 64, 10, 32, 129, 4, 8, 1, 2, 0, 0, skd.BF16, 0),  # bf16 path: batch above 128
        skd.Config(4, 256, 4, 80, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.BF16, 0),    # bf16 path: FFN width % 32
        skd.Config(4, 32768, 256, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.BF16, 0),  # bf16 path: d_model above 16384
        skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.FP32, 2),    # io_on_device is 0 or 1
    ]
    for cfg in bad:
        assert lib.skd_create(C.byref(cfg), C.byref(w), None, C.byref(h)) == skd.ERR_SHAPE
    assert lib.skd_create(None, C.byref(w), None, C.byref(h)) == skd.ERR_NULL
    ok = skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.FP32, 0)
    assert lib.skd_create(C.byref(ok), C.byref(w), None, C.byref(h)) == skd.ERR_NULL   # weight pointers missing
    assert lib.skd_prefill(None, None, None) == skd.ERR_NULL
    assert lib.skd_decode_step(None, 0, None) == skd.ERR_NULL
    assert lib.skd_logits_argmax(None, None, None) == skd.ERR_NULL
    assert lib.skd_kv_len(None, 0) == skd.ERR_NULL


def test_schedule_table_validation():
    # caller-supplied layer counts: monotone non-increasing, within [max(1, warmup), L]; checked before any device work
    lib = skd.lib()
    h = C.c_void_p()
    w = skd.Weights()
    cfg = skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 1, 2, 0, 0, skd.FP32, 0)

    def rc(table, cfg=cfg):
        import numpy as np
        t = np.asarray(table, dtype=np.int32)
        return lib.skd_create_with_schedule(C.byref(cfg), C.byref(w), None, t.ctypes.data, C.byref(h))

    assert rc([4, 4, 4, 4, 3, 3, 2, 1]) == skd.ERR_NULL            # valid table: fails later, on the missing weights
    assert rc([4, 4, 4, 4, 3, 2, 3, 1]) == skd.ERR_SCHEDULE        # a layer would re-enter
    assert rc([4, 4, 4, 4, 3, 3, 2, 0]) == skd.ERR_RANGE
    assert rc([5, 4, 4, 4, 3, 3, 2, 1]) == skd.ERR_RANGE
    cfgw = skd.Config(4, 256, 4, 64, 10, 32, 1, 4, 8, 2, 3, 2, 0, skd.FP32, 0)
    assert rc([4, 4, 4, 4, 3, 3, 2, 1], cfgw) == skd.ERR_SHAPE     # falls below the warm-up layers
    assert lib.skd_create_with_schedule(C.byref(cfg), C.byref(w), None, None, C.byref(h)) == skd.ERR_NULL
    assert lib.skd_state_active_layers(None, 0, None) == skd.ERR_NULL
