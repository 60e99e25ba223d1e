"""Pins of the decoding-step oracle (Section 3.1 of the paper) against library routines, closed forms and
invariants.  CPU only."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import decode_oracle as D
from oracle import meda_oracle as O


def rng(seed):
    return np.random.Generator(np.random.Philox(key=[seed, 77]))


def test_attend_matches_scipy_softmax_and_loops():
    r = rng(1)
    q, k, v = r.normal(size=16), r.normal(size=(37, 16)), r.normal(size=(37, 16))
    got = D.attend(q, k, v)
    p = softmax(k @ q / 4.0)                       # 1/sqrt(16)
    assert np.allclose(got, p @ v, rtol=1e-13, atol=1e-15)
    # the definition written as loops
    logits = [sum(q[e] * k[j, e] for e in range(16)) / 4.0 for j in range(37)]
    z = sum(np.exp(x) for x in logits)
    ref = [sum(np.exp(logits[j]) / z * v[j, e] for j in range(37)) for e in range(16)]
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-14)


def test_equal_logits_give_the_mean_value():
    r = rng(2)
    v = r.normal(size=(9, 8))
    assert np.allclose(D.attend(np.zeros(8), r.normal(size=(9, 8)), v), v.mean(axis=0), rtol=1e-14)
    k = np.tile(r.normal(size=(1, 8)), (9, 1))     # identical keys: any query sees equal logits
    assert np.allclose(D.attend(r.normal(size=8), k, v), v.mean(axis=0), rtol=1e-13)


def test_dominant_key_returns_its_value_and_two_keys_are_logistic():
    r = rng(3)
    d = 4
    q = np.array([1.0, 0, 0, 0])
    k = np.zeros((5, d)); k[3, 0] = 400.0          # logit 200 against zeros
    v = r.normal(size=(5, d))
    assert np.allclose(D.attend(q, k, v), v[3], rtol=1e-12, atol=1e-14)
    # two keys with logits a, b: weights sigma(a-b), 1-sigma(a-b)
    k2 = np.array([[3.0, 0, 0, 0], [1.0, 0, 0, 0]])
    v2 = r.normal(size=(2, d))
    w = 1.0 / (1.0 + np.exp(-(3.0 - 1.0) / np.sqrt(d)))
    assert np.allclose(D.attend(q, k2, v2), w * v2[0] + (1 - w) * v2[1], rtol=1e-14)


def test_scale_argument_and_logit_shift_invariance():
    r = rng(4)
    q, k, v = r.normal(size=8), r.normal(size=(20, 8)), r.normal(size=(20, 8))
    assert np.allclose(D.attend(q, k, v, scale=0.5), softmax(k @ q * 0.5) @ v, rtol=1e-13)
    # adding a vector c to every key shifts all logits by q.c and cannot change the output
    c = r.normal(size=8)
    assert np.allclose(D.attend(q, k + c, v), D.attend(q, k, v), rtol=1e-11, atol=1e-13)


def test_row_order_of_the_cache_does_not_matter_and_append_is_concatenation():
    r = rng(5)
    q, k, v = r.normal(size=8), r.normal(size=(30, 8)), r.normal(size=(30, 8))
    perm = r.permutation(30)
    assert np.allclose(D.attend(q, k[perm], v[perm]), D.attend(q, k, v), rtol=1e-12, atol=1e-14)
    q_l = r.normal(size=(2, 8))
    k_l, v_l = r.normal(size=(2, 11, 8)), r.normal(size=(2, 11, 8))
    k_n, v_n = r.normal(size=(2, 3, 8)), r.normal(size=(2, 3, 8))
    got = D.decode_layer(q_l, k_l, v_l, k_n, v_n)
    ref = D.decode_layer(q_l, np.concatenate([k_l, k_n], axis=1), np.concatenate([v_l, v_n], axis=1))
    assert np.array_equal(got, ref)
    assert np.array_equal(D.append_rows(k_l[0], None), k_l[0])
    assert np.array_equal(D.append_rows(k_l[0], k_n[0])[11:], k_n[0])


def test_grouped_heads_read_their_kv_head():
    r = rng(6)
    Hq, Hkv, d = 6, 2, 8
    q_l = r.normal(size=(Hq, d))
    k_l, v_l = r.normal(size=(Hkv, 13, d)), r.normal(size=(Hkv, 13, d))
    out = D.decode_layer(q_l, k_l, v_l)
    for h in range(Hq):
        assert np.array_equal(out[h], D.attend(q_l[h], k_l[h // 3], v_l[h // 3]))
    # changing kv head 1 must not touch the query heads 0..2
    k2 = k_l.copy(); k2[1, 0] += 1.0
    out2 = D.decode_layer(q_l, k2, v_l)
    assert np.array_equal(out2[:3], out[:3]) and not np.allclose(out2[3:], out[3:])


def test_ragged_layout_and_full_budget_equals_full_cache():
    r = rng(7)
    L, Hq, Hkv, d, T, W = 3, 4, 2, 8, 40, 4
    f32 = lambda x: x.astype(np.float32).astype(np.float64)      # storage type of this test: binary32
    q_win = f32(r.normal(size=(L, Hq, W, d)))
    k = f32(r.normal(size=(L, Hkv, T, d))); v = f32(r.normal(size=(L, Hkv, T, d)))
    mask = (np.arange(T) % 3 == 0).astype(np.uint8)
    q = r.normal(size=(L, Hq, d))
    def flat(res):      # the ragged layout the compression pass writes: layer after layer, [Hkv][S_l][d] inside
        return (np.concatenate([x.reshape(-1, d) for x in res["k_out"]]),
                np.concatenate([x.reshape(-1, d) for x in res["v_out"]]))
    # budget 100 %: the compression oracle returns the cache itself, so decoding over it is decoding over k, v
    res = O.meda_compress(q_win, k, v, mask, total_budget=L * T, window=W, dtype="f32")
    kc, vc = flat(res)
    out = D.decode_step(q, kc, vc, res["S"], res["off"], Hkv)
    for l in range(L):
        assert np.allclose(out[l], D.decode_layer(q[l], k[l], v[l]), rtol=1e-13, atol=1e-15)
    # a smaller budget: every layer is read at its own offset and length
    res = O.meda_compress(q_win, k, v, mask, total_budget=L * 12 + 1, window=W, dtype="f32")
    kc, vc = flat(res)
    assert kc.shape[0] == (L * 12 + 1) * Hkv
    out = D.decode_step(q, kc, vc, res["S"], res["off"], Hkv)
    for l in range(L):
        assert np.array_equal(out[l], D.decode_layer(q[l], res["k_out"][l], res["v_out"][l]))
    # a layer read at a wrong offset gives a different result (the offsets are used)
    if res["S"][0] != res["S"][1]:
        bad = D.decode_step(q, kc, vc, res["S"][::-1].copy(), res["off"], Hkv)
        assert not np.allclose(bad, out)


def test_merging_duplicate_pairs_leaves_the_decoding_output_of_those_keys_consistent():
    # two identical (k, v) pairs carry twice the weight of one: attention over [a, a, b] equals
    # attention over [a, b] with a's logit raised by log 2
    r = rng(8)
    d = 8
    q = r.normal(size=d)
    a_k, b_k, a_v, b_v = r.normal(size=d), r.normal(size=d), r.normal(size=d), r.normal(size=d)
    out3 = D.attend(q, np.stack([a_k, a_k, b_k]), np.stack([a_v, a_v, b_v]))
    sa, sb = a_k @ q / np.sqrt(d), b_k @ q / np.sqrt(d)
    w = 2 * np.exp(sa) / (2 * np.exp(sa) + np.exp(sb))
    assert np.allclose(out3, w * a_v + (1 - w) * b_v, rtol=1e-13)
