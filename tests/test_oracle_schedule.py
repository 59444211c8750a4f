"""Pins for the oracle's schedule (Section 2.3) and active-layer set (Section 2.4).

Nothing here re-types the oracle's integer formula: the checks are the values
the paper prints (Fig. 3, Table 2), exact rational arithmetic with
fractions.Fraction on the paper's real-valued equation, and the properties the
text states (bounds, monotone decrease, end points, predefined total cost).
"""
import os
import random
from fractions import Fraction

import pytest

from oracle import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_fig3():
    params, rows = {}, []
    for line in open(os.path.join(GOLD, "fig3_schedule.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a = line.split()
        if a[0].isalpha() or "_" in a[0]:
            params[a[0]] = int(a[1])
        else:
            rows.append((int(a[0]), Fraction(a[1]), int(a[2])))
    return params, rows


def _read_table2():
    rows = []
    for line in open(os.path.join(GOLD, "table2_configs.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a = line.split()
        rows.append((int(a[0]), int(a[1]), Fraction(a[2]), int(a[3]), int(a[4]), int(a[5])))
    return rows


def paper_real_value(i, P, N, n_min, n_max, L):
    """The paper's token_idx equation in exact rationals (Section 2.3)."""
    if i < P:
        return Fraction(L)
    t = Fraction(i - P, N - P)
    return (1 - t) * n_max + t * n_min


def test_fig3_worked_example():
    p, rows = _read_fig3()
    for pos, real, integer in rows:
        assert paper_real_value(pos, p["P"], p["N"], p["n_min"], p["n_max"], p["L"]) == real
        assert O.schedule(pos, p["P"], p["N"], p["n_min"], p["n_max"], p["L"]) == integer


def test_table2_target_average():
    # The mean of the layer counts over a full-length generation is the
    # table's "#Target Avg Layer" = (min + max) / 2, up to the rounding of
    # individual positions (bounded by 1/2 layer each, and nearly cancelling).
    for L, _speedup, printed_avg, _w, n_min, n_max in _read_table2():
        for P, N in ((60, 160), (512, 1024), (1024, 2048)):   # the paper's three length settings
            T = N - P
            ns = [O.schedule(P + k, P, N, n_min, n_max, L) for k in range(T)]
            mean = Fraction(sum(ns), T)
            mid = Fraction(n_min + n_max, 2)
            assert abs(mean - mid) <= Fraction(n_max - n_min, 2 * T) + Fraction(1, 2)
            assert abs(printed_avg - mid) <= Fraction(1, 2)


def _random_params(rng):
    L = rng.randint(1, 48)
    n_max = rng.randint(1, L)
    n_min = rng.randint(1, n_max)
    P = rng.randint(0, 300)
    N = P + rng.randint(1, 600)
    return L, n_min, n_max, P, N


def test_properties_random():
    rng = random.Random(1234)
    for _ in range(300):
        L, n_min, n_max, P, N = _random_params(rng)
        T = N - P
        ns = [O.schedule(i, P, N, n_min, n_max, L) for i in range(N + 1)]
        assert all(n == L for n in ns[:P])                       # prompt at full depth
        gen = ns[P:]
        assert gen[0] == n_max                                    # first generated position gets max
        assert gen[-1] == n_min                                   # position max-length gets min
        assert all(n_min <= n <= n_max for n in gen)              # never above max nor below min
        assert all(a >= b for a, b in zip(gen, gen[1:]))          # monotonically decreasing
        # nearest integer to the paper's real value, halves up
        for k in (0, T // 3, T // 2, T - 1, T):
            r = paper_real_value(P + k, P, N, n_min, n_max, L)
            n = gen[k]
            assert Fraction(-1, 2) <= r - n < Fraction(1, 2)
            assert n == (r + Fraction(1, 2)).__floor__()
        # predefined total cost: closed form of the real sum over k = 0..T-1
        real_sum = Fraction(T * n_max) - Fraction((n_max - n_min) * (T - 1), 2)
        assert real_sum == sum(paper_real_value(P + k, P, N, n_min, n_max, L) for k in range(T))
        assert abs(sum(gen[:T]) - real_sum) <= Fraction(T, 2)
        assert sum(gen[:T]) <= T * n_max                          # worst case strictly bounded


def test_contract_config_sums():
    # Σ n over the decode steps of the five benchmark configurations
    # (integers that follow from the half-up rounding of the linear decay).
    cases = [
        (4, 16, 32, 2, 4, 50),
        (24, 256, 512, 12, 24, 4616),
        (32, 512, 768, 6, 32, 4878),
        (32, 2048, 2560, 12, 32, 11276),
        (32, 512, 640, 8, 24, 2064),
    ]
    for L, P, N, n_min, n_max, total in cases:
        ns = [O.schedule(P + k, P, N, n_min, n_max, L) for k in range(N - P)]
        assert sum(ns) == total
        assert ns[-1] == n_min


def test_errors():
    assert O.schedule_rc(0, 10, 10, 1, 2, 4) == O.ERR_SHAPE      # N == P
    assert O.schedule_rc(0, 10, 20, 0, 2, 4) == O.ERR_SHAPE      # n_min < 1
    assert O.schedule_rc(0, 10, 20, 3, 2, 4) == O.ERR_SHAPE      # n_min > n_max
    assert O.schedule_rc(0, 10, 20, 1, 5, 4) == O.ERR_SHAPE      # n_max > L
    assert O.schedule_rc(21, 10, 20, 1, 2, 4) == O.ERR_RANGE     # i > N
    assert O.schedule_rc(-1, 10, 20, 1, 2, 4) == O.ERR_RANGE
    assert O.schedule_rc(20, 10, 20, 1, 2, 4) == 1               # i == N allowed, gives n_min
    with pytest.raises(O.OracleError):
        O.active_layers(12, 10, 20, 1, 2, 2, 4)                  # warmup > n_min


def test_active_set_is_top_window_and_warmup():
    rng = random.Random(7)
    for _ in range(200):
        L, n_min, n_max, P, N = _random_params(rng)
        w = rng.randint(0, n_min)
        prev = None
        for i in range(P, N + 1):
            n = O.schedule(i, P, N, n_min, n_max, L)
            A = O.active_layers(i, P, N, n_min, n_max, w, L)
            assert len(A) == n and A == sorted(set(A))
            assert A[:w] == list(range(w))                        # warm-up layers are the bottom ones
            assert A[w:] == list(range(L - (n - w), L))           # the rest is a top window ending at L-1
            if prev is not None:
                assert set(A) <= set(prev)                        # nested: a layer never re-enters
            prev = A
        if P > 0:
            assert O.active_layers(P - 1, P, N, n_min, n_max, w, L) == list(range(L))


def test_f32_build_agrees():
    rng = random.Random(99)
    for _ in range(50):
        L, n_min, n_max, P, N = _random_params(rng)
        for i in (0, P, (P + N) // 2, N):
            assert O.schedule(i, P, N, n_min, n_max, L, "f32") == O.schedule(i, P, N, n_min, n_max, L, "f64")
