"""Pins of the oracle when every prompt position scores the keys (Section 3.3: A_s sums A_p over all prompt rows;
Section 3.2: A_TV / A_VT over all text / vision queries) instead of an observation window.  CPU only."""
import numpy as np

from oracle import meda_oracle as O


def rng(seed):
    return np.random.Generator(np.random.Philox(key=[seed, 99]))


def test_uniform_causal_attention_gives_harmonic_column_scores_and_log_counts():
    # Q = 0: row i is uniform over its i+1 visible keys, so A_s[j] = sum_{i>=j} 1/(i+1) = H_T - H_j
    T, d = 50, 8
    q = np.zeros((2, T, d)); k = rng(1).normal(size=(1, T, d))
    s = O.window_logits(q, k)
    a_s = O.column_scores(O.masked_softmax(s, O.causal_allowed(T, T)), 1)
    harm = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, T + 1))])
    assert np.allclose(a_s[0], 2 * (harm[T] - harm[:T]), rtol=1e-13)        # two query heads share the kv head
    # entropy: a text row with n visible vision keys has entropy log n (0 keys -> 0), and vice versa
    mask = (np.arange(T) % 5 < 2).astype(np.uint8)
    h_tv, h_vt, e = O.cross_modal_entropy(s, mask)
    nv = np.cumsum(mask); nt = np.cumsum(1 - mask)
    ent_rows = np.where(mask == 0, np.log(np.maximum(nv, 1)), np.log(np.maximum(nt, 1)))
    assert np.isclose(h_tv, ent_rows[mask == 0].mean(), rtol=1e-13)
    assert np.isclose(h_vt, ent_rows[mask == 1].mean(), rtol=1e-13) and np.isclose(e, h_tv + h_vt)


def test_all_rows_against_plain_loops():
    r = rng(2)
    T, d, Hq, Hkv = 12, 4, 4, 2
    q, k = r.normal(size=(Hq, T, d)), r.normal(size=(Hkv, T, d))
    mask = np.array([0, 1, 1, 0, 1, 0, 0, 1, 1, 1, 0, 0], dtype=np.uint8)
    s = O.window_logits(q, k)
    a_s = O.column_scores(O.masked_softmax(s, O.causal_allowed(T, T)), Hkv)
    ref = np.zeros((Hkv, T))
    pbar = np.zeros((T, T))
    for h in range(Hq):
        g = h // 2
        for i in range(T):
            lg = [q[h, i] @ k[g, j] / 2.0 for j in range(i + 1)]
            z = sum(np.exp(x) for x in lg)
            for j in range(i + 1):
                ref[g, j] += np.exp(lg[j]) / z
            cross = [j for j in range(i + 1) if mask[j] != mask[i]]
            zc = sum(np.exp(lg[j]) for j in cross)
            for j in cross:
                pbar[i, j] += np.exp(lg[j]) / zc / Hq
    assert np.allclose(a_s, ref, rtol=1e-12)
    ent = [-sum(p * np.log(p) for p in pbar[i] if p > 0) for i in range(T)]
    h_tv, h_vt, e = O.cross_modal_entropy(s, mask)
    assert np.isclose(h_tv, np.mean([ent[i] for i in range(T) if mask[i] == 0]), rtol=1e-12)
    assert np.isclose(h_vt, np.mean([ent[i] for i in range(T) if mask[i] == 1]), rtol=1e-12)


def test_scores_of_all_rows_are_the_sum_over_row_blocks_with_truncated_keys():
    # the rows [a, b) only see keys < b: their contribution is a window computation on the first b keys
    r = rng(3)
    T, d, Hq, Hkv, blk = 45, 8, 4, 2, 16
    q, k = r.normal(size=(Hq, T, d)), r.normal(size=(Hkv, T, d))
    mask = (r.random(T) < 0.6).astype(np.uint8)
    s = O.window_logits(q, k)
    full = O.column_scores(O.masked_softmax(s, O.causal_allowed(T, T)), Hkv)
    ent_full = O.row_entropy(O.cross_modal_probs(s, mask))
    acc = np.zeros_like(full)
    ent_rows = np.zeros(T)
    b = T
    while b > 0:
        a = max(0, b - blk)
        sb = O.window_logits(q[:, a:b], k[:, :b])
        acc[:, :b] += O.column_scores(O.masked_softmax(sb, O.causal_allowed(b, b - a)), Hkv)
        ent_rows[a:b] = O.row_entropy(O.cross_modal_probs(sb, mask[:b]))
        b = a
    assert np.allclose(acc, full, rtol=1e-12, atol=1e-15)
    assert np.allclose(ent_rows, ent_full, rtol=1e-12, atol=1e-15)


def test_compress_accepts_all_rows_and_keeps_the_window_as_the_recent_floor():
    r = rng(4)
    L, Hq, Hkv, T, d, W = 2, 2, 2, 40, 8, 4
    f32 = lambda x: x.astype(np.float32).astype(np.float64)
    q, k, v = f32(r.normal(size=(L, Hq, T, d))), f32(r.normal(size=(L, Hkv, T, d))), f32(r.normal(size=(L, Hkv, T, d)))
    mask = (np.arange(T) % 4 == 1).astype(np.uint8)
    res = O.meda_compress(q, k, v, mask, total_budget=L * 12, window=W, dtype="f32")
    assert int(res["S"].sum()) == L * 12 and (res["S"] >= W).all()
    assert (res["M"] == np.maximum(np.minimum(W, res["S"]), res["S"] * 3 // 4)).all()
    win = O.meda_compress(q[:, :, T - W:], k, v, mask, total_budget=L * 12, window=W, dtype="f32")
    assert not np.allclose(res["entropy"], win["entropy"])      # the other rows do enter the entropy
    # the vision -> text direction is present: some vision rows see text keys
    assert res["h_vt"].min() > 0
