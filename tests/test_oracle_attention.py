"""Pins for the oracle's window attention, column scores and cross-modal entropy.

Each test checks the oracle against something other than itself: a closed form, a library
routine (scipy), or a brute-force loop written here from the paper's formula.
"""
import math

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax
from scipy.stats import entropy as sp_entropy

from oracle import meda_oracle as O


def rng(seed=0):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- logits / softmax

def test_logits_scale_and_ratio_closed_form():
    # one query, two keys: p0/p1 = exp((q.k0 - q.k1)/sqrt(d))   (Sec. 3.2, Softmax(QK^T/sqrt(D)))
    d = 16
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 2.0
    k = np.zeros((1, 2, d)); k[0, 0, 0] = 3.0; k[0, 1, 0] = 1.0
    s = O.window_logits(q, k)
    assert s.shape == (1, 1, 2)
    assert s[0, 0, 0] == pytest.approx(6.0 / 4.0) and s[0, 0, 1] == pytest.approx(2.0 / 4.0)
    p = O.masked_softmax(s, np.ones((1, 2), bool))
    assert p[0, 0, 0] / p[0, 0, 1] == pytest.approx(math.exp(4.0 / 4.0))


def test_logits_not_transposed():
    # asymmetric operands: s[h, i, j] must pair query row i with key row j
    r = rng(1)
    q = r.standard_normal((2, 3, 8)); k = r.standard_normal((2, 5, 8))
    s = O.window_logits(q, k, scale=1.0)
    for h in range(2):
        for i in range(3):
            for j in range(5):
                assert s[h, i, j] == pytest.approx(float(np.dot(q[h, i], k[h, j])))


def test_gqa_head_mapping():
    # kv head g has a single dominant key at position g: query head h must peak at h // G
    Hq, Hkv, T, d, W = 6, 3, 12, 8, 2
    k = np.zeros((Hkv, T, d))
    for g in range(Hkv):
        k[g, g, :] = 10.0
    q = np.ones((Hq, W, d))
    p = O.masked_softmax(O.window_logits(q, k), O.causal_allowed(T, W))
    for h in range(Hq):
        assert np.all(np.argmax(p[h], axis=1) == h // 2)


def test_softmax_matches_scipy_on_unmasked_rows():
    r = rng(2)
    s = r.standard_normal((3, 4, 50)) * 5
    p = O.masked_softmax(s, np.ones((4, 50), bool))
    np.testing.assert_allclose(p, sp_softmax(s, axis=-1), rtol=1e-13, atol=0)


def test_causal_uniform_closed_form():
    # zero queries: row i at position T-W+i is uniform over its T-W+i+1 visible keys
    Hq, Hkv, T, W, d = 4, 2, 40, 8, 4
    q = np.zeros((Hq, W, d)); k = rng(3).standard_normal((Hkv, T, d))
    allowed = O.causal_allowed(T, W)
    p = O.masked_softmax(O.window_logits(q, k), allowed)
    for i in range(W):
        n = T - W + i + 1
        np.testing.assert_allclose(p[:, i, :n], 1.0 / n, rtol=1e-14)
        assert np.all(p[:, i, n:] == 0.0)
    # column scores: A_s[j] = G * sum_{i : j visible} 1/(T-W+i+1), and sum_j A_s = G*W
    a = O.column_scores(p, Hkv)
    G = Hq // Hkv
    for j in range(T):
        want = G * sum(1.0 / (T - W + i + 1) for i in range(W) if j <= T - W + i)
        assert a[0, j] == pytest.approx(want, rel=1e-13)
    np.testing.assert_allclose(a.sum(axis=1), G * W, rtol=1e-13)


def test_column_scores_group_sum_bruteforce():
    r = rng(4)
    Hq, Hkv, T, W, d = 6, 2, 30, 5, 8
    q = r.standard_normal((Hq, W, d)); k = r.standard_normal((Hkv, T, d))
    p = O.masked_softmax(O.window_logits(q, k), O.causal_allowed(T, W))
    a = O.column_scores(p, Hkv)
    G = Hq // Hkv
    for g in range(Hkv):
        for j in range(T):
            want = sum(p[h, i, j] for h in range(g * G, (g + 1) * G) for i in range(W))
            assert a[g, j] == pytest.approx(want, rel=1e-13)


# ---------------------------------------------------------------- entropy

def test_row_entropy_uniform_onehot_binary():
    n = 37
    assert O.row_entropy(np.full((1, n), 1.0 / n))[0] == pytest.approx(math.log(n), rel=1e-14)
    one = np.zeros((1, n)); one[0, 5] = 1.0
    assert O.row_entropy(one)[0] == 0.0
    pb = 0.3
    assert O.row_entropy(np.array([[pb, 1 - pb]]))[0] == pytest.approx(
        -(pb * math.log(pb) + (1 - pb) * math.log(1 - pb)), rel=1e-14)


def test_row_entropy_matches_scipy():
    p = sp_softmax(rng(5).standard_normal((6, 64)) * 3, axis=-1)
    np.testing.assert_allclose(O.row_entropy(p), sp_entropy(p, axis=-1), rtol=1e-13)


def _layout_mask(T, vis_ranges):
    m = np.zeros(T, dtype=np.uint8)
    for a, b in vis_ranges:
        m[a:b] = 1
    return m


def test_cross_modal_entropy_uniform_is_log_of_cross_set():
    # zero logits: a text row's cross-modal distribution is uniform over the visible vision keys
    Hq, Hkv, T, W, d = 2, 1, 64, 8, 4
    mask = _layout_mask(T, [(10, 40)])                 # 30 vision keys, window all text
    s = np.zeros((Hq, W, T))
    h_tv, h_vt, e = O.cross_modal_entropy(s, mask)
    assert h_tv == pytest.approx(math.log(30), rel=1e-14)
    assert h_vt == 0.0 and e == pytest.approx(math.log(30), rel=1e-14)


def test_cross_modal_entropy_both_directions_and_causality():
    # window = 4 vision rows then 4 text rows; zero logits -> each row is uniform over the
    # visible keys of the other modality, so E_CM = mean log|C_i| (text rows) + mean log|C_i| (vision rows)
    T, W = 48, 8
    mask = _layout_mask(T, [(8, 20), (T - 8, T - 4)])  # vision: 12 keys + the first 4 window rows
    s = np.zeros((3, W, T))
    h_tv, h_vt, e = O.cross_modal_entropy(s, mask)
    n_text_before = lambda p: int((mask[:p + 1] == 0).sum())
    n_vis_before = lambda p: int((mask[:p + 1] == 1).sum())
    want_vt = np.mean([math.log(n_text_before(T - 8 + i)) for i in range(4)])
    want_tv = np.mean([math.log(n_vis_before(T - 4 + i)) for i in range(4)])
    assert h_vt == pytest.approx(want_vt, rel=1e-14)
    assert h_tv == pytest.approx(want_tv, rel=1e-14)
    assert e == pytest.approx(want_tv + want_vt, rel=1e-14)
    # vision rows inside the window are causal: row 0 (first vision row) sees only the text before it
    assert n_text_before(T - 8) == 8 + (T - 8 - 20)


def test_entropy_is_of_head_mean_not_mean_of_entropies():
    # two heads, each one-hot on a different vision key: the head-averaged row is {1/2, 1/2},
    # entropy log 2; averaging per-head entropies would give 0 (Sec. 3.2: A is the head average)
    T, W = 16, 1
    mask = _layout_mask(T, [(2, 6)])
    s = np.full((2, W, T), -1e4)
    s[0, 0, 2] = 0.0
    s[1, 0, 4] = 0.0
    h_tv, h_vt, e = O.cross_modal_entropy(s, mask)
    assert e == pytest.approx(math.log(2.0), rel=1e-12)


def test_cross_modal_softmax_is_renormalised_over_the_sub_block():
    # a huge same-modality logit must not change the cross-modal distribution
    T, W = 12, 1
    mask = _layout_mask(T, [(3, 6)])
    r = rng(6)
    s = r.standard_normal((1, W, T))
    s2 = s.copy(); s2[0, 0, 0] += 50.0                  # key 0 is text, row is text
    assert O.cross_modal_entropy(s, mask)[2] == pytest.approx(O.cross_modal_entropy(s2, mask)[2], rel=1e-12)
    # and equals scipy's entropy of the softmax restricted to the vision keys
    want = sp_entropy(sp_softmax(s[0, 0, 3:6]))
    assert O.cross_modal_entropy(s, mask)[2] == pytest.approx(want, rel=1e-12)


def test_cross_modal_entropy_bruteforce_loops():
    r = rng(7)
    Hq, T, W = 3, 20, 6
    mask = _layout_mask(T, [(4, 9), (15, 17)])
    s = r.standard_normal((Hq, W, T)) * 2
    h_tv, h_vt, e = O.cross_modal_entropy(s, mask)
    ent_t, ent_v = [], []
    for i in range(W):
        p_i = T - W + i
        cols = [j for j in range(p_i + 1) if mask[j] != mask[p_i]]
        pbar = np.zeros(len(cols))
        for h in range(Hq):
            z = sum(math.exp(s[h, i, j]) for j in cols)
            pbar += np.array([math.exp(s[h, i, j]) / z for j in cols]) / Hq
        hrow = -sum(p * math.log(p) for p in pbar if p > 0)
        (ent_t if mask[p_i] == 0 else ent_v).append(hrow)
    assert h_tv == pytest.approx(np.mean(ent_t), rel=1e-12)
    assert h_vt == pytest.approx(np.mean(ent_v), rel=1e-12)
    assert e >= 0.0


def test_row_with_empty_cross_set_counts_in_denominator():
    # no vision key at all: every text row has an empty cross-modal set -> entropy 0
    s = rng(8).standard_normal((2, 4, 10))
    assert O.cross_modal_entropy(s, np.zeros(10, np.uint8)) == (0.0, 0.0, 0.0)
