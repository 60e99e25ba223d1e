"""Pins for the oracle's selection, nearest-neighbour matching, average merging and the whole pass
(Section 3.3), plus the storage rounding helper."""
import numpy as np
import pytest
import torch

from oracle import meda_oracle as O
from workloads import generate, get_workload, variant
from workloads.gen import to_float64


def rng(seed=0):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- selection

def brute_force_top(a_s, mask, n_top, n_recent):
    """Python sort written from the text: boost text by the max, drop the recent tail, take the best."""
    T = len(a_s)
    mx = max(a_s)
    boosted = [a_s[j] + (mx if mask[j] == 0 else 0.0) for j in range(T)]
    cand = list(range(T - n_recent))
    cand.sort(key=lambda j: (-boosted[j], j))
    return sorted(cand[:n_top])


@pytest.mark.parametrize("seed", range(6))
def test_select_matches_brute_force_sort(seed):
    r = rng(seed)
    T = int(r.integers(8, 60))
    n_recent = int(r.integers(0, T // 2))
    n_top = int(r.integers(0, T - n_recent + 1))
    a_s = r.random(T)
    a_s[r.integers(0, T, size=T // 3)] = 0.25          # exact ties
    mask = (r.random(T) < 0.6).astype(np.uint8)
    idx_c, idx_less = O.select_tokens(a_s, mask, n_top, n_recent)
    top = brute_force_top(list(a_s), list(mask), n_top, n_recent)
    assert list(idx_c) == top + list(range(T - n_recent, T))
    assert sorted(set(idx_c) | set(idx_less)) == list(range(T))
    assert len(idx_c) == n_top + n_recent and not (set(idx_c) & set(idx_less))
    assert list(idx_less) == sorted(idx_less)


def test_ties_go_to_the_smaller_position():
    a_s = np.array([0.5, 0.5, 0.5, 0.5, 0.1, 0.9])
    mask = np.ones(6, np.uint8)
    idx_c, _ = O.select_tokens(a_s, mask, 2, 1)
    assert list(idx_c) == [0, 1, 5]


def test_text_outranks_vision_after_boost():
    # every text candidate must be selected before any vision candidate (A_s[T] += max(A_s))
    r = rng(3)
    T = 40
    mask = (np.arange(T) % 3 != 0).astype(np.uint8)     # every third position is text
    a_s = r.random(T)
    a_s[mask == 0] *= 1e-3                              # text scores tiny
    n_recent = 4
    n_text_cand = int((mask[:T - n_recent] == 0).sum())
    idx_c, _ = O.select_tokens(a_s, mask, n_text_cand, n_recent)
    assert set(idx_c[:n_text_cand]) == set(np.flatnonzero(mask[:T - n_recent] == 0))
    # one more slot goes to the best vision candidate
    idx_c2, _ = O.select_tokens(a_s, mask, n_text_cand + 1, n_recent)
    extra = set(idx_c2[:n_text_cand + 1]) - set(idx_c[:n_text_cand])
    vis_c = np.flatnonzero(mask[:T - n_recent] == 1)
    assert extra == {int(vis_c[np.argmax(a_s[vis_c])])}


def test_boost_uses_max_over_all_positions():
    a_s = np.array([0.1, 0.2, 0.3, 5.0])
    mask = np.array([0, 1, 1, 1], np.uint8)
    np.testing.assert_allclose(O.boosted_scores(a_s, mask), [5.1, 0.2, 0.3, 5.0])


def test_select_everything_and_nothing():
    a_s = rng(4).random(10); mask = np.zeros(10, np.uint8)
    idx_c, idx_less = O.select_tokens(a_s, mask, 7, 3)
    assert list(idx_c) == list(range(10)) and len(idx_less) == 0
    idx_c, idx_less = O.select_tokens(a_s, mask, 0, 3)
    assert list(idx_c) == [7, 8, 9] and list(idx_less) == list(range(7))


# ---------------------------------------------------------------- nearest conserved key

def test_nn_assign_matches_brute_force_loops():
    r = rng(5)
    T, d = 30, 6
    k = r.standard_normal((T, d))
    idx_c = np.array(sorted(r.choice(T, 8, replace=False)))
    idx_less = np.array([t for t in range(T) if t not in set(idx_c)])
    got = O.nn_assign(k, idx_c, idx_less, chunk=7)
    for n, i in enumerate(idx_less):
        best, best_u = -1, -np.inf
        for slot, j in enumerate(idx_c):
            u = float(np.dot(k[i], k[j]) / (np.linalg.norm(k[i]) * np.linalg.norm(k[j])))
            if u > best_u:
                best, best_u = slot, u
        assert got[n] == best


def test_cosine_is_scale_invariant_and_bounded():
    r = rng(6)
    a = r.standard_normal((5, 8)); b = r.standard_normal((7, 8))
    u = O.cosine_matrix(a, b)
    u2 = O.cosine_matrix(a * r.uniform(0.1, 9, (5, 1)), b * r.uniform(0.1, 9, (7, 1)))
    np.testing.assert_allclose(u, u2, rtol=1e-12, atol=1e-14)
    assert np.all(np.abs(u) <= 1 + 1e-12)
    e = np.eye(4)
    np.testing.assert_allclose(O.cosine_matrix(e, 3 * e), e, atol=1e-15)


def test_duplicate_of_a_conserved_key_maps_to_its_lowest_copy():
    r = rng(7)
    k = r.standard_normal((12, 8))
    k[9] = k[3] * 2.5           # same direction as conserved 3 and 5
    k[5] = k[3]
    idx_c = np.array([1, 3, 5, 11]); idx_less = np.array([0, 2, 4, 6, 7, 8, 9, 10])
    got = O.nn_assign(k, idx_c, idx_less)
    assert got[list(idx_less).index(9)] == 1     # slot of position 3, the lower of the duplicates


def test_identical_conserved_keys_always_resolve_to_the_lowest_slot():
    # many columns and rows, so that a blocked float64 matrix product rounds identical columns differently:
    # the tie rule must not depend on that noise
    r = rng(8)
    T, d = 900, 64
    k = r.standard_normal((T, d)).astype(np.float32).astype(np.float64)
    heavy = 3.0 * k[5] / np.linalg.norm(k[5])
    dup_pos = [7, 130, 131, 395, 640]
    k[dup_pos] = heavy
    idx_c = np.array(sorted(set(range(0, T, 3)) | set(dup_pos)))
    idx_less = np.array([t for t in range(T) if t not in set(idx_c)])
    k[idx_less[::4]] = heavy * r.uniform(0.5, 2.0, size=(len(idx_less[::4]), 1))   # rows whose best is the duplicate
    got = O.nn_assign(k, idx_c, idx_less, chunk=257)
    lowest = int(np.flatnonzero(idx_c == 7)[0])
    assert np.all(got[::4] == lowest)
    # brute force on a sample of the other rows
    for n in range(1, len(idx_less), 37):
        u = [float(np.dot(k[idx_less[n]], k[j]) / (np.linalg.norm(k[idx_less[n]]) * np.linalg.norm(k[j]))) for j in idx_c]
        assert abs(u[got[n]] - max(u)) <= 1e-12


def test_heavy_hitter_duplicates_in_a_workload_resolve_to_the_lowest_slot():
    # the workloads hold exact duplicate keys (heavy hitters): whatever slot a row is assigned to, no
    # lower conserved slot may hold a bit-identical key (fails with a plain argmax over the float64 product)
    wl = variant(get_workload("tiny"), tau_lo=1.5, tau_hi=1.5, n_layers=3, total_budget=700)
    d = generate(wl)
    res = O.meda_compress(to_float64(d["q"]), to_float64(d["k"]), to_float64(d["v"]), d["mask"].numpy(),
                          wl.total_budget, wl.window, wl.dtype)
    k = to_float64(d["k"])[0]
    n_dup_rows = 0
    for g, h in enumerate(res["heads"][0]):
        kc = k[g][h["idx_c"]]
        _, first = np.unique(kc, axis=0, return_index=True)
        lowest_copy = {kc[i].tobytes(): i for i in sorted(first, reverse=True)}
        for i in sorted(first):
            lowest_copy[kc[i].tobytes()] = min(lowest_copy[kc[i].tobytes()], i)
        canon = np.array([lowest_copy[row.tobytes()] for row in kc])
        n_dup_rows += int((canon[h["assign"]] != np.arange(len(kc))[h["assign"]]).sum())
        assert np.array_equal(canon[h["assign"]], h["assign"])
    assert n_dup_rows == 0


def test_rounding_noise_between_equal_similarities_does_not_pick_a_higher_slot(monkeypatch):
    # emulate a matrix product that rounds two identical columns differently by one unit in the last place
    k = np.array([[1.0, 2.0], [3.0, 1.0], [1.0, 2.0], [0.5, 1.0], [-1.0, 0.3]])
    exact = O.cosine_matrix

    def noisy(a, b):
        u = exact(a, b)
        u[:, 0] -= 2.3e-16          # column 0 and column 2 are the same key; make the lower one look smaller
        return u
    monkeypatch.setattr(O, "cosine_matrix", noisy)
    got = O.nn_assign(k, np.array([0, 1, 2]), np.array([3, 4]))
    assert got[0] == 0              # [0.5, 1] is parallel to slots 0 and 2: the lower slot wins
    # a real gap far above the noise is still respected
    assert got[1] == int(np.argmax(exact(k[[4]], k[[0, 1, 2]])[0]))


def test_margin_reporting():
    k = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 0.1]])
    a, best, gap = O.nn_assign(k, np.array([0, 1]), np.array([2]), return_margin=True)
    c0 = 1.0 / np.hypot(1.0, 0.1); c1 = 0.1 / np.hypot(1.0, 0.1)
    assert a[0] == 0 and best[0] == pytest.approx(c0) and gap[0] == pytest.approx(c0 - c1)


# ---------------------------------------------------------------- merging

def _random_case(seed, T=50, d=8, S=12):
    r = rng(seed)
    k = r.standard_normal((T, d)); v = r.standard_normal((T, d))
    idx_c = np.array(sorted(r.choice(T, S, replace=False)))
    idx_less = np.array([t for t in range(T) if t not in set(idx_c)])
    return k, v, idx_c, idx_less


@pytest.mark.parametrize("seed", range(4))
def test_merge_conserves_mass_for_any_assignment(seed):
    k, v, idx_c, idx_less = _random_case(seed)
    assign = rng(seed + 100).integers(0, len(idx_c), size=len(idx_less))
    k_m, v_m, members = O.average_merge(k, v, idx_c, idx_less, assign)
    w = (members + 1)[:, None]
    np.testing.assert_allclose((w * k_m).sum(0), k.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose((w * v_m).sum(0), v.sum(0), rtol=1e-12, atol=1e-12)
    assert (members + 1).sum() == len(k)


def test_merge_matches_loop_from_the_formula():
    k, v, idx_c, idx_less = _random_case(9)
    assign = O.nn_assign(k, idx_c, idx_less)
    k_m, v_m, members = O.average_merge(k, v, idx_c, idx_less, assign)
    for slot, j in enumerate(idx_c):
        nb = [i for n, i in enumerate(idx_less) if assign[n] == slot]
        np.testing.assert_allclose(k_m[slot], (k[j] + sum(k[i] for i in nb)) / (len(nb) + 1), rtol=1e-13)
        np.testing.assert_allclose(v_m[slot], (v[j] + sum(v[i] for i in nb)) / (len(nb) + 1), rtol=1e-13)
        assert members[slot] == len(nb)


def test_values_follow_the_keys_assignment():
    # V of a less-important token lands in the slot its KEY chose, whatever the values are
    k = np.array([[1.0, 0.0], [0.0, 1.0], [0.9, 0.1]])
    v = np.array([[10.0, 0.0], [0.0, 20.0], [0.0, 300.0]])   # V of token 2 is closest to V of token 1
    idx_c, idx_less = np.array([0, 1]), np.array([2])
    assign = O.nn_assign(k, idx_c, idx_less)
    k_m, v_m, _ = O.average_merge(k, v, idx_c, idx_less, assign)
    np.testing.assert_allclose(v_m[0], [5.0, 150.0])
    np.testing.assert_allclose(v_m[1], [0.0, 20.0])


def test_merging_duplicate_pairs_preserves_them():
    r = rng(10)
    base_k = r.standard_normal((3, 8)); base_v = r.standard_normal((3, 8))
    reps = [0, 1, 2, 0, 0, 1, 2, 2, 1, 0]
    k = base_k[reps]; v = base_v[reps]
    idx_c = np.array([0, 1, 2]); idx_less = np.arange(3, 10)
    assign = O.nn_assign(k, idx_c, idx_less)
    assert list(assign) == reps[3:]
    k_m, v_m, members = O.average_merge(k, v, idx_c, idx_less, assign)
    np.testing.assert_allclose(k_m, base_k, rtol=1e-14)
    np.testing.assert_allclose(v_m, base_v, rtol=1e-14)


# ---------------------------------------------------------------- storage rounding

def test_round_to_bf16_matches_torch_and_rounds_once():
    r = rng(11)
    x32 = (r.standard_normal(20000) * np.exp(r.uniform(-6, 6, 20000))).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_storage(x32.astype(np.float64), "bf16"), want)
    # a float64 just above a bf16 midpoint: rounding through float32 first would land on the
    # midpoint and then go to even (down); direct rounding goes up
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert O.round_to_storage(np.array([x]), "bf16")[0] == 1.0 + 2.0 ** -7
    assert O.round_to_storage(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 1.0          # tie -> even
    assert O.round_to_storage(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 1.0 + 2.0 ** -6
    assert O.round_to_storage(np.array([0.0, -2.5]), "bf16").tolist() == [0.0, -2.5]


def test_round_to_f32():
    x = np.array([0.1, 1.0 + 2.0 ** -30])
    np.testing.assert_array_equal(O.round_to_storage(x, "f32"), x.astype(np.float32).astype(np.float64))


# ---------------------------------------------------------------- whole pass

@pytest.fixture(scope="module")
def tiny():
    wl = get_workload("tiny")
    d = generate(wl)
    return wl, d


def _run(wl, d, budget=None):
    return O.meda_compress(to_float64(d["q"]), to_float64(d["k"]), to_float64(d["v"]), d["mask"].numpy(),
                           wl.total_budget if budget is None else budget, wl.window, wl.dtype)


def test_full_budget_is_the_identity_cache(tiny):
    wl, d = tiny
    res = _run(wl, d, budget=wl.n_layers * wl.seq_len)
    k = to_float64(d["k"]); v = to_float64(d["v"])
    for l in range(wl.n_layers):
        assert res["S"][l] == wl.seq_len
        np.testing.assert_array_equal(res["k_out"][l], k[l])
        np.testing.assert_array_equal(res["v_out"][l], v[l])
        for h in res["heads"][l]:
            assert len(h["idx_less"]) == 0 and np.all(h["members"] == 0)


def test_whole_pass_invariants(tiny):
    wl, d = tiny
    res = _run(wl, d)
    k = to_float64(d["k"]); v = to_float64(d["v"])
    T = wl.seq_len
    assert res["S"].sum() == wl.total_budget
    assert np.all(res["entropy"] >= 0) and np.all(res["h_vt"] == 0)      # window is all text
    for l in range(wl.n_layers):
        np.testing.assert_allclose(res["a_s"][l].sum(axis=1), wl.group_size * wl.window, rtol=1e-12)
        assert res["k_out"][l].shape == (wl.n_kv_heads, res["S"][l], wl.head_dim)
        for g, h in enumerate(res["heads"][l]):
            assert list(h["idx_c"][-res["M"][l]:]) == list(range(T - res["M"][l], T))
            w = (h["members"] + 1)[:, None]
            np.testing.assert_allclose((w * h["k_exact"]).sum(0), k[l, g].sum(0), rtol=1e-10, atol=1e-9)
            np.testing.assert_allclose((w * h["v_exact"]).sum(0), v[l, g].sum(0), rtol=1e-10, atol=1e-9)
            # slots nobody merged into are exact copies
            alone = h["members"] == 0
            np.testing.assert_array_equal(h["k_out"][alone], k[l, g][h["idx_c"][alone]])
    # output bytes scale with the budget (App. A.2: memory is proportional to the kept length)
    total_rows = sum(o.shape[1] for o in res["k_out"])
    assert total_rows == wl.total_budget


def test_higher_temperature_layer_gets_smaller_budget(tiny):
    # a sharper (higher temperature) layer has lower cross-modal entropy, hence a smaller share
    from workloads.gen import layer_taus
    wl, d = tiny
    res = _run(wl, d)
    taus = layer_taus(wl)
    assert (taus[0] < taus[1]) == (res["S"][0] > res["S"][1])


def test_vision_rows_in_window_give_vt_entropy():
    base = get_workload("tiny")
    layout = (("t", 64, -1), ("v", 256, 0), ("v", 256, 1), ("v", 256, 2), ("t", 160, -1),
              ("v", 16, 2), ("t", 16, -1))
    wl = variant(base, name="tiny_vt", layout=layout)
    assert wl.seq_len == 1024
    d = generate(wl)
    res = _run(wl, d)
    assert np.all(res["h_vt"] > 0) and np.all(res["h_tv"] > 0)
    np.testing.assert_allclose(res["entropy"], res["h_tv"] + res["h_vt"], rtol=1e-15)
