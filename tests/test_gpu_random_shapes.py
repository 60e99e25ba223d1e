"""Seeded sweep over small shapes (sequence length, window, group size, head dimension, storage type, layout,
budget, recent share, scoring with the window or with every prompt row) through the whole pass and one decoding
step, against the oracles; a second sweep runs such shapes with the ablation flags."""
import numpy as np
import pytest

from workloads import generate, get_workload, variant

from parity import check_all, run_gpu

pytestmark = pytest.mark.gpu
TINY = get_workload("tiny")


def _random_layout(r, T):
    """Alternating text / vision segments of random lengths that sum to T; ends with text or vision at random."""
    segs, left, kind, grp = [], T, ("t" if r.random() < 0.5 else "v"), 0
    while left > 0:
        n = int(min(left, r.integers(1, max(2, T // 3))))
        if kind == "v":
            segs.append(("v", n, grp)); grp += 1
        else:
            segs.append(("t", n, -1))
        left -= n
        kind = "v" if kind == "t" else "t"
    return tuple(segs)


def _configs():
    r = np.random.Generator(np.random.Philox(key=[2024, 5]))
    out = []
    for i in range(14):
        T = int(r.choice([40, 63, 64, 65, 127, 129, 200, 257, 300, 511, 640]))
        W = int(min(T, r.choice([1, 2, 7, 31, 32, 33, 64, 100, 128])))
        hkv = int(r.choice([1, 2, 3]))
        G = int(r.choice([1, 2, 3, 4, 5, 8]))
        while G * ((W + 31) // 32) > 32:
            G //= 2
        d = int(r.choice([64, 128]))
        dtype = str(r.choice(["f32", "bf16"]))
        L = int(r.integers(1, 5))
        lo, hi = L * W, L * T
        B = int(r.integers(lo, hi + 1)) if r.random() < 0.8 else int(r.choice([lo, hi]))
        num, den = [(3, 4), (0, 1), (1, 1), (1, 2)][int(r.integers(0, 4))]
        out.append(variant(TINY, name=f"rand{i}", n_layers=L, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                           layout=_random_layout(r, T), window=W, total_budget=B, seed=100 + i, recent_num=num,
                           recent_den=den, tau_lo=0.3, tau_hi=3.0, heavy_frac=float(r.choice([0.0, 0.02, 0.1]))))
    # a second draw with longer sequences (several sort tiles, both similarity kernels' regimes), windows of up to
    # four 32-row blocks, group sizes up to 8 and more kv heads
    r = np.random.Generator(np.random.Philox(key=[2024, 6]))
    for i in range(14, 40):
        T = int(r.choice([33, 100, 128, 129, 255, 256, 300, 513, 777, 1024, 1500, 2049, 3000]))
        W = int(min(T, r.choice([1, 5, 31, 32, 33, 63, 64, 65, 96, 97, 127, 128])))
        hkv = int(r.choice([1, 2, 3, 5]))
        G = int(r.choice([1, 2, 3, 4, 6, 7, 8]))
        while G * ((W + 31) // 32) > 32:
            G -= 1
        d = int(r.choice([64, 128]))
        dtype = str(r.choice(["f32", "bf16"]))
        L = int(r.integers(1, 4))
        lo, hi = L * W, L * T
        B = int(r.integers(lo, hi + 1)) if r.random() < 0.85 else int(r.choice([lo, hi]))
        num, den = [(3, 4), (0, 1), (1, 1), (1, 2), (1, 3)][int(r.integers(0, 5))]
        out.append(variant(TINY, name=f"rand{i}", n_layers=L, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                           layout=_random_layout(r, T), window=W, total_budget=B, seed=100 + i, recent_num=num,
                           recent_den=den, tau_lo=0.3, tau_hi=3.0, heavy_frac=float(r.choice([0.0, 0.02, 0.1]))))
    # a third draw for the row-block mode of the scoring kernels: windows of more than 128 rows, up to 32 query heads
    # per kv head, and every prompt row scoring (three cases in ten)
    r = np.random.Generator(np.random.Philox(key=[2024, 7]))
    for i in range(40, 64):
        T = int(r.choice([64, 129, 200, 256, 300, 513, 777, 1024, 1500, 2049]))
        W = int(min(T, r.choice([16, 32, 64, 96, 128, 129, 150, 200, 256, 257, 300, 400, 512, 640])))
        hkv = int(r.choice([1, 2, 3]))
        G = int(r.choice([1, 2, 3, 4, 7, 8, 12, 16, 32]))
        d = int(r.choice([64, 128]))
        dtype = str(r.choice(["f32", "bf16"]))
        L = int(r.integers(1, 3))
        lo, hi = L * W, L * T
        B = int(r.integers(lo, hi + 1)) if r.random() < 0.85 else int(r.choice([lo, hi]))
        kw = dict(score_rows=T) if r.random() < 0.3 else {}
        out.append(variant(TINY, name=f"rand{i}", n_layers=L, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                           layout=_random_layout(r, T), window=W, total_budget=B, seed=100 + i, tau_lo=0.3, tau_hi=3.0,
                           heavy_frac=float(r.choice([0.0, 0.02, 0.1])), **kw))
    return out


@pytest.mark.parametrize("wl", _configs(), ids=lambda w: w.name)
def test_random_shape(wl):
    print(f"\n[random case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} T={wl.seq_len} "
          f"W={wl.window} B={wl.total_budget} {wl.dtype} recent={wl.recent_num}/{wl.recent_den} layout={wl.layout}", flush=True)
    data = generate(wl)
    comp, gpu = run_gpu(wl, data)
    check_all(wl, data, gpu)
    # one decoding step over the cache this shape produces, with a few appended rows (the step takes up to 8 query
    # heads per kv head and has no notion of scoring rows)
    if wl.n_q_heads // wl.n_kv_heads <= 8 and wl.n_score_rows == wl.window:
        from test_gpu_decode import _check as check_decode
        check_decode(wl, n_new=wl.seed % 4)


def _flag_configs():
    """Shapes of both scoring modes, each with one of the three flag combinations."""
    r = np.random.Generator(np.random.Philox(key=[2024, 8]))
    out = []
    for i in range(18):
        T = int(r.choice([40, 64, 129, 200, 300, 513, 777, 1024, 1500]))
        W = int(min(T, r.choice([1, 7, 32, 33, 64, 96, 128, 129, 200, 300])))
        hkv = int(r.choice([1, 2, 3]))
        G = int(r.choice([1, 2, 3, 4, 8, 16]))
        d = int(r.choice([64, 128]))
        dtype = str(r.choice(["f32", "bf16"]))
        L = int(r.integers(1, 5))
        lo, hi = L * W, L * T
        B = int(r.integers(lo, hi + 1)) if r.random() < 0.85 else int(r.choice([lo, hi]))
        num, den = [(3, 4), (0, 1), (1, 1), (1, 2)][int(r.integers(0, 4))]
        kw = dict(score_rows=T) if r.random() < 0.25 else {}
        wl = variant(TINY, name=f"flags{i}", n_layers=L, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                     layout=_random_layout(r, T), window=W, total_budget=B, seed=300 + i, recent_num=num, recent_den=den,
                     tau_lo=0.3, tau_hi=3.0, heavy_frac=float(r.choice([0.0, 0.02, 0.1])), **kw)
        out.append((wl, 1 + i % 3))
    return out


@pytest.mark.parametrize("wl,flags", _flag_configs(), ids=lambda x: x.name if hasattr(x, "name") else f"flags={x}")
def test_random_shape_with_flags(wl, flags):
    """Uniform budgets (1): the layer lengths are B/L whatever the entropies are, and everything downstream matches the
    oracle run with them.  No merge (2): the same conserved sets as the plain run, their rows copied bit for bit.
    Both (3): the conserved sets of the uniform-budget run, copied."""
    import paper_2502_17599_amd as pkg
    from oracle import meda_oracle as O
    from parity import check_head, gpu_head, oracle_scores
    from workloads.gen import to_float64
    assert (pkg.FLAG_UNIFORM_BUDGET, pkg.FLAG_NO_MERGE) == (1, 2)
    print(f"\n[flag case] {wl.name} flags={flags}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} W={wl.window} rows={wl.n_score_rows} B={wl.total_budget} {wl.dtype} "
          f"recent={wl.recent_num}/{wl.recent_den}", flush=True)
    data = generate(wl)
    _, gpu = run_gpu(wl, data, flags=flags)
    L, Hkv, T = wl.n_layers, wl.n_kv_heads, wl.seq_len
    assert int(gpu["S"].sum()) == wl.total_budget and np.array_equal(np.diff(gpu["off"]), gpu["S"])
    if flags & pkg.FLAG_UNIFORM_BUDGET:
        S, M, N, off = O.allocate_budgets(np.zeros(L), wl.total_budget, T, wl.window, wl.recent_num, wl.recent_den)
        assert gpu["S"].tolist() == S.tolist() and max(S) - min(S) <= 1 and list(S) == sorted(S, reverse=True)
        assert np.array_equal(gpu["alloc"][:, 1], M) and np.array_equal(gpu["alloc"][:, 2], N)
    if flags == pkg.FLAG_UNIFORM_BUDGET:
        a_s, _ = oracle_scores(wl, data)
        stats = {"heads": 0, "rows": 0, "ambiguous_rows": 0, "sets_differing_in_tie_band": 0,
                 "max_kv_err": 0.0, "kv_elems_not_bit_exact": 0}
        for l in range(L):
            for g in range(Hkv):
                check_head(wl, data, gpu, a_s[l], l, g, int(N[l]), int(M[l]), stats)
        print(f"[flag case] {stats}", flush=True)
        return
    # no merge: the sets of the run that merges (same budget rule), the rows as stored
    _, ref = run_gpu(wl, data, flags=flags & ~pkg.FLAG_NO_MERGE)
    assert np.array_equal(gpu["S"], ref["S"]) and np.array_equal(gpu["sel_idx"], ref["sel_idx"])
    assert np.array_equal(gpu["entropy"], ref["entropy"]) and np.array_equal(gpu["col_scores"], ref["col_scores"])
    for l in range(L):
        for g in range(Hkv):
            idx, k_out, v_out = gpu_head(wl, gpu, l, g)
            assert np.array_equal(k_out, to_float64(data["k"][l, g])[idx]), f"layer {l} head {g}: keys not copied"
            assert np.array_equal(v_out, to_float64(data["v"][l, g])[idx]), f"layer {l} head {g}: values not copied"
            ma = gpu["merge_assign"][l, g]
            assert np.array_equal(ma[idx], np.arange(len(idx)))
            assert np.all(ma[np.setdiff1d(np.arange(T), idx)] == -1)


def _many_pairs_configs():
    """At least 256 (layer, kv head) pairs, which is when the similarity search sends layers whose conserved set fits
    into LDS to its resident-set kernel; average budgets on both sides of that capacity (576 rows of 256 bytes, 1184
    rows of 128 bytes), so that most cases run both kernels."""
    r = np.random.Generator(np.random.Philox(key=[2024, 9]))
    out = []
    for i in range(6):
        L, hkv = [(8, 32), (16, 16), (32, 8), (64, 4), (16, 32), (64, 8)][i]
        G = int(r.choice([1, 2, 4]))
        T = int(r.choice([640, 1000, 1537, 2048]))
        W = int(r.choice([8, 32, 64]))
        d = (64, 128)[i % 2]
        dtype = ("bf16", "bf16", "f32")[i % 3]
        avg = int(r.choice([100, 300, 560, 600, 1000]))
        B = int(max(L * W, L * min(avg, 3 * T // 4)))
        out.append(variant(TINY, name=f"pairs{i}", n_layers=L, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                           layout=_random_layout(r, T), window=W, total_budget=B, seed=400 + i, tau_lo=0.3, tau_hi=3.0,
                           heavy_frac=float(r.choice([0.0, 0.02]))))
    return out


@pytest.mark.parametrize("wl", _many_pairs_configs(), ids=lambda w: w.name)
def test_random_shape_with_many_layer_head_pairs(wl):
    print(f"\n[many-pairs case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} W={wl.window} B={wl.total_budget} {wl.dtype}", flush=True)
    data = generate(wl)
    comp, gpu = run_gpu(wl, data)
    order = np.argsort(gpu["S"])
    layers = sorted({int(order[0]), int(order[-1]), int(order[len(order) // 2]), int(order[len(order) // 3])})
    # entropies and budgets of all layers; selection, matching and merged rows of one head of the layers with the
    # smallest, the largest and two middle budgets
    check_all(wl, data, gpu, heads=[(l, (l * 7) % wl.n_kv_heads) for l in layers], threads=8)
