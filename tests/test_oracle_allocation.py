"""Pins for the oracle's layer-budget allocation (Sec. 3.2 allocation eq., App. A.3, Sec. 4.3)."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import meda_oracle as O


def test_budgets_sum_to_total_and_stay_in_bounds():
    r = np.random.default_rng(0)
    for trial in range(200):
        L = int(r.integers(1, 40))
        T = int(r.integers(64, 5000))
        W = int(r.integers(1, 64))
        lo, hi = min(W, T), T
        B = int(r.integers(L * lo, L * hi + 1))
        E = r.uniform(0, 12, size=L)
        S, M, N, off = O.allocate_budgets(E, B, T, W)
        assert S.sum() == B and off[-1] == B and off[0] == 0
        assert np.all(S >= lo) and np.all(S <= hi)
        assert np.all(np.diff(off) == S)
        assert np.all(M + N == S) and np.all(N >= 0) and np.all(M >= np.minimum(W, S))


def test_equal_entropies_split_evenly_extras_on_lowest_layers():
    S, M, N, off = O.allocate_budgets(np.full(5, 3.3), 1003, 1000, 16)
    assert list(S) == [201, 201, 201, 200, 200]


def test_two_layers_ln2_apart_split_two_to_one():
    # no clamp active: S_l proportional to exp(E_l)  ->  exactly 2 : 1
    S, *_ = O.allocate_budgets(np.array([1.0 + math.log(2.0), 1.0]), 3000, 4000, 8)
    assert list(S) == [2000, 1000]


def test_matches_paper_formula_when_no_clamp_binds():
    # S_l = softmax(E)_l * L * rho * T (App. A.3) up to the integer rounding
    E = np.array([5.1, 4.7, 5.6, 4.9, 5.3, 5.0])
    L, T, rho = 6, 10000, 0.2
    B = int(L * rho * T)
    S, *_ = O.allocate_budgets(E, B, T, 16)
    alpha = np.exp(E) / np.exp(E).sum() * L * rho
    assert np.all(np.abs(S - alpha * T) < 1.0)
    assert S.sum() == B


def test_largest_remainder_with_exact_rationals():
    # weights 1:2:4 (entropies 0, ln2, 2ln2), B = 100 -> reals 100/7, 200/7, 400/7
    E = np.array([0.0, math.log(2.0), 2 * math.log(2.0)])
    S, *_ = O.allocate_budgets(E, 100, 1000, 1)
    reals = [Fraction(100, 7), Fraction(200, 7), Fraction(400, 7)]   # fracs 2/7, 4/7, 1/7
    floors = [int(x) for x in reals]                                   # 14, 28, 57 -> rest 1
    assert sum(floors) == 99
    assert list(S) == [14, 29, 57]


def test_full_budget_is_identity_allocation_for_any_entropies():
    E = np.array([0.1, 9.0, 3.0, 7.5])
    S, M, N, off = O.allocate_budgets(E, 4 * 777, 777, 32)
    assert np.all(S == 777)


def test_floor_budget_gives_every_layer_the_window():
    E = np.array([0.1, 9.0, 3.0, 7.5])
    S, M, N, off = O.allocate_budgets(E, 4 * 32, 777, 32)
    assert np.all(S == 32) and np.all(M == 32) and np.all(N == 0)


def test_monotone_in_entropy():
    r = np.random.default_rng(1)
    for _ in range(50):
        E = r.uniform(0, 10, size=12)
        S, *_ = O.allocate_budgets(E, 12 * 300, 2000, 16)
        order = np.argsort(E)
        # integer rounding can only reorder by one unit
        assert np.all(np.diff(S[order]) >= -1)


def test_clamps_redistribute_exactly():
    # layer 0 would get almost everything; it is capped at T and the rest is shared 1:1
    E = np.array([30.0, 1.0, 1.0])
    S, *_ = O.allocate_budgets(E, 1000 + 2 * 150, 1000, 10)
    assert list(S) == [1000, 150, 150]
    # layers 1, 2 would get nothing; they are floored at W and layer 0 takes the rest
    S, *_ = O.allocate_budgets(E, 500, 1000, 10)
    assert list(S) == [480, 10, 10]


def test_water_filling_against_bisection():
    # an independent solver for sum clamp(lam*w) = B
    r = np.random.default_rng(2)
    for _ in range(100):
        L = int(r.integers(2, 33))
        T, W = 4096, 32
        E = r.uniform(0, 9, size=L)
        B = int(r.integers(L * W + 1, L * T))
        x = O.allocation_reals(E, B, W, T)
        w = np.exp(E - E.max())
        a, b = 0.0, 1e12
        for _ in range(200):
            mid = 0.5 * (a + b)
            if np.clip(mid * w, W, T).sum() < B:
                a = mid
            else:
                b = mid
        np.testing.assert_allclose(x, np.clip(b * w, W, T), rtol=1e-9, atol=1e-6)
        assert x.sum() == pytest.approx(B, rel=1e-12)


def test_recent_to_important_ratio_is_three_to_one():
    S, M, N, off = O.allocate_budgets(np.zeros(1), 400, 1000, 32)
    assert (int(M[0]), int(N[0])) == (300, 100)
    # window larger than 3/4 of the budget: the window wins
    S, M, N, off = O.allocate_budgets(np.zeros(1), 40, 1000, 32)
    assert (int(M[0]), int(N[0])) == (32, 8)
    # other split (recent = window only)
    S, M, N, off = O.allocate_budgets(np.zeros(1), 400, 1000, 32, recent_num=0, recent_den=1)
    assert (int(M[0]), int(N[0])) == (32, 368)


def test_kv_memory_formula_golden():
    # tests/golden/kv_memory_formula.txt holds the constants of the paper's App. A.2 formula
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "kv_memory_formula.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split("=")
                vals[key.strip()] = float(val)
    per_token = O.kv_cache_bytes(1, int(vals["layers"]), int(vals["heads"]), int(vals["head_dim"]),
                                 int(vals["bytes_per_element"]))
    assert per_token == 2 * 32 * 32 * 128 * 2
    # the full-cache figure printed in the latency/memory table corresponds to a whole number of tokens
    tokens = vals["full_cache_gib"] * 1024 ** 3 / per_token
    assert abs(tokens - round(tokens)) < 0.5 and 4900 < tokens < 5000


def test_budget_margins_predict_which_perturbation_flips_a_budget():
    """The margin report of the parity helper: shifting one layer's entropy by clearly less than its reported
    relative margin leaves every budget as it is, shifting it by clearly more changes some budget."""
    from parity import budget_margins
    from workloads import get_workload, variant
    wl = variant(get_workload("tiny"), n_layers=6, total_budget=6 * 300)
    rng = np.random.default_rng(3)
    e = rng.uniform(3.0, 5.0, size=6)
    S0 = O.allocate_budgets(e, wl.total_budget, wl.seq_len, wl.window)[0]
    margin, rel = budget_margins(wl, e)
    assert np.all(margin > 0) and np.isfinite(margin).all()
    l = int(np.argmin(rel))
    for sign in (+1.0, -1.0):
        small = e.copy(); small[l] *= 1.0 + sign * 0.2 * rel[l]
        assert np.array_equal(O.allocate_budgets(small, wl.total_budget, wl.seq_len, wl.window)[0], S0)
    flipped = False
    for sign in (+1.0, -1.0):
        big = e.copy(); big[l] *= 1.0 + sign * 5.0 * rel[l]
        flipped |= not np.array_equal(O.allocate_budgets(big, wl.total_budget, wl.seq_len, wl.window)[0], S0)
    assert flipped
