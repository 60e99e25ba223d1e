"""HIP path vs fp64 oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from workloads import generate, get_workload, variant

from parity import check_all, run_gpu

pytestmark = pytest.mark.gpu


def _case(wl, **kw):
    print(f"\n[case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} W={wl.window} B={wl.total_budget} {wl.dtype} seed={wl.seed}", flush=True)
    data = generate(wl)
    comp, gpu = run_gpu(wl, data)
    return check_all(wl, data, gpu, **kw)


TINY = get_workload("tiny")
VT_LAYOUT = (("t", 64, -1), ("v", 256, 0), ("v", 256, 1), ("v", 256, 2), ("t", 160, -1), ("v", 16, 2), ("t", 16, -1))


def test_tiny_fp32():
    stats = _case(TINY)
    assert stats["budgets_strictly_equal"]


def test_tiny_window_with_vision_rows():
    _case(variant(TINY, name="tiny_vt", layout=VT_LAYOUT))


def test_tiny_full_budget_is_identity():
    wl = variant(TINY, name="tiny_identity", total_budget=TINY.n_layers * TINY.seq_len)
    data = generate(wl)
    comp, gpu = run_gpu(wl, data)
    assert np.all(gpu["S"] == wl.seq_len)
    k = data["k"].to(torch.float64).numpy().reshape(-1, wl.head_dim)
    v = data["v"].to(torch.float64).numpy().reshape(-1, wl.head_dim)
    assert np.array_equal(gpu["k_out"], k) and np.array_equal(gpu["v_out"], v)
    check_all(wl, data, gpu)


def test_tiny_floor_budget():
    _case(variant(TINY, name="tiny_floor", total_budget=TINY.n_layers * TINY.window))


def test_tiny_equal_temperatures_split_evenly():
    wl = variant(TINY, name="tiny_equal_tau", tau_lo=1.5, tau_hi=1.5, n_layers=3, total_budget=700)
    _case(wl)


@pytest.mark.parametrize("seed", [1, 2])
def test_small_bf16_gqa_ragged(seed):
    # several column tiles and a ragged tail (T = 1000 is no multiple of 128), grouped heads, 3 layers
    layout = (("t", 40, -1), ("v", 300, 0), ("t", 30, -1), ("v", 300, 1), ("t", 10, -1), ("v", 200, 2), ("t", 120, -1))
    wl = variant(TINY, name=f"small_bf16_s{seed}", n_layers=3, n_q_heads=8, n_kv_heads=2, head_dim=128,
                 dtype="bf16", layout=layout, window=32, total_budget=3 * 230, seed=seed)
    assert wl.seq_len == 1000
    _case(wl)


def test_small_bf16_window_48_mixed_rows():
    # window that is no multiple of 32 and holds vision rows; group size 3
    layout = (("t", 33, -1), ("v", 400, 0), ("t", 77, -1), ("v", 350, 1), ("t", 100, -1), ("v", 20, 1), ("t", 20, -1))
    wl = variant(TINY, name="small_w48", n_layers=2, n_q_heads=6, n_kv_heads=2, head_dim=128, dtype="bf16",
                 layout=layout, window=48, total_budget=2 * 300, seed=3)
    _case(wl)


def test_small_fp32_d128_and_bf16_d64():
    layout = (("t", 50, -1), ("v", 500, 0), ("t", 150, -1))
    _case(variant(TINY, name="f32_d128", n_layers=2, n_q_heads=2, n_kv_heads=2, head_dim=128, dtype="f32",
                  layout=layout, window=32, total_budget=2 * 200, seed=4))
    _case(variant(TINY, name="bf16_d64", n_layers=2, n_q_heads=4, n_kv_heads=1, head_dim=64, dtype="bf16",
                  layout=layout, window=64, total_budget=2 * 200, seed=5))


def test_window_equals_sequence():
    layout = (("v", 40, 0), ("t", 24, -1))
    _case(variant(TINY, name="w_eq_t", n_layers=2, n_q_heads=2, n_kv_heads=1, layout=layout, window=64,
                  total_budget=2 * 64, seed=6))


def test_deterministic_across_runs():
    wl = variant(TINY, name="det", n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=128, dtype="bf16",
                 layout=(("t", 60, -1), ("v", 700, 0), ("t", 140, -1)), total_budget=2 * 180, seed=7)
    data = generate(wl)
    _, a = run_gpu(wl, data)
    _, b = run_gpu(wl, data)
    for key in ("k_out", "v_out", "sel_idx", "merge_assign", "entropy", "col_scores"):
        assert np.array_equal(a[key], b[key]), key


def test_flag_uniform_budget_ignores_the_entropies():
    # ablation "without dynamic allocation" (Table 5 of the paper): every layer gets B/L, extras on the lowest layers
    import paper_2502_17599_amd as pkg
    from oracle import meda_oracle as O
    wl = variant(TINY, name="uniform_budget", n_layers=3, total_budget=3 * 200 + 2)
    data = generate(wl)
    comp, gpu = run_gpu(wl, data, flags=pkg.FLAG_UNIFORM_BUDGET)
    S, M, N, off = O.allocate_budgets(np.zeros(wl.n_layers), wl.total_budget, wl.seq_len, wl.window,
                                      wl.recent_num, wl.recent_den)
    assert gpu["S"].tolist() == S.tolist() == [201, 201, 200]
    assert np.array_equal(gpu["alloc"][:, 1], M) and np.array_equal(gpu["alloc"][:, 2], N)
    # downstream stages still match the oracle run with these budgets
    from parity import check_head, oracle_scores
    a_s, _ = oracle_scores(wl, data)
    stats = {"heads": 0, "rows": 0, "ambiguous_rows": 0, "sets_differing_in_tie_band": 0,
             "max_kv_err": 0.0, "kv_elems_not_bit_exact": 0}
    for l in range(wl.n_layers):
        for g in range(wl.n_kv_heads):
            check_head(wl, data, gpu, a_s[l], l, g, int(N[l]), int(M[l]), stats)
    assert stats["kv_elems_not_bit_exact"] == 0


def test_flag_no_merge_copies_the_conserved_rows():
    # ablation "without average merging": eviction, the kept rows are bit-exact copies
    import paper_2502_17599_amd as pkg
    from parity import gpu_head
    wl = variant(TINY, name="no_merge")
    data = generate(wl)
    comp, ref = run_gpu(wl, data)
    comp, gpu = run_gpu(wl, data, flags=pkg.FLAG_NO_MERGE)
    assert np.array_equal(gpu["S"], ref["S"]) and np.array_equal(gpu["sel_idx"], ref["sel_idx"])
    k = data["k"].to(torch.float64).numpy(); v = data["v"].to(torch.float64).numpy()
    for l in range(wl.n_layers):
        for g in range(wl.n_kv_heads):
            idx, k_out, v_out = gpu_head(wl, gpu, l, g)
            assert np.array_equal(k_out, k[l, g][idx]) and np.array_equal(v_out, v[l, g][idx])
            ma = gpu["merge_assign"][l, g]
            assert np.array_equal(ma[idx], np.arange(len(idx)))
            rest = np.setdiff1d(np.arange(wl.seq_len), idx)
            assert np.all(ma[rest] == -1)


def test_large_window_and_large_groups():
    # window of 128 rows (four 32-row blocks) with 8 query heads per kv head, and a 96-row window with
    # vision rows: the largest (head, row block) counts the scoring kernels are built for
    layout = (("t", 30, -1), ("v", 500, 0), ("t", 100, -1), ("v", 300, 1), ("t", 94, -1))
    _case(variant(TINY, name="w128_g8", n_layers=2, n_q_heads=8, n_kv_heads=1, head_dim=128, dtype="bf16",
                  layout=layout, window=128, total_budget=2 * 300, seed=8))
    layout = (("t", 30, -1), ("v", 500, 0), ("t", 100, -1), ("v", 340, 1), ("t", 54, -1))
    _case(variant(TINY, name="w96_g4_f32", n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=64, dtype="f32",
                  layout=layout, window=96, total_budget=2 * 260, seed=9))


def test_windows_of_more_than_128_rows_take_the_row_block_mode():
    # 200 rows (fp32, one query head per kv head: a 256-row block whose second half is short), 300 rows with grouped
    # heads and vision rows inside the window (bf16: 96-row blocks of 32 in pass A, two 256-row blocks in pass B),
    # and a window as long as the sequence
    layout = (("t", 40, -1), ("v", 300, 0), ("t", 30, -1), ("v", 300, 1), ("t", 10, -1), ("v", 200, 2), ("t", 120, -1))
    _case(variant(TINY, name="w200_f32", n_layers=2, n_q_heads=4, n_kv_heads=4, layout=layout, window=200,
                  total_budget=2 * 320, seed=31))
    _case(variant(TINY, name="w300_g4", n_layers=3, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16",
                  layout=layout, window=300, total_budget=3 * 420, seed=32))
    short = (("v", 140, 0), ("t", 60, -1), ("v", 100, 1), ("t", 50, -1))
    _case(variant(TINY, name="w350_eq_t", n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="bf16",
                  layout=short, window=350, total_budget=2 * 350, seed=33))


def test_sixteen_query_heads_per_kv_head_with_a_96_row_window():
    # 48 (head, 32-row block) pairs per kv head: more than a workgroup of the window kernels holds, so the scoring
    # runs in the row-block mode although the window has fewer than 128 rows
    layout = (("t", 30, -1), ("v", 500, 0), ("t", 100, -1), ("v", 340, 1), ("t", 54, -1))
    _case(variant(TINY, name="w96_g16", n_layers=2, n_q_heads=16, n_kv_heads=1, head_dim=128, dtype="bf16",
                  layout=layout, window=96, total_budget=2 * 260, seed=34))


def test_argmax_when_another_slot_of_the_block_trails_the_best_by_exactly_two():
    """Crafted keys for the search of the winning slot inside a block of 32 (Section 3.3, merging: each key that is
    not conserved goes to the conserved key it is most similar to).  The conserved keys are unit vectors along the
    axes, so the scaled product of a row with slot s is the row's component s, exactly.  Row 0 has 1 on axis 0 and 3
    on axis 1: its best slot is 1, and slot 0, which sits in a lower register of the same lane, trails it by exactly
    2.0, a float whose low 28 bits are zero.  (A search that packs the difference and the register into one 32-bit
    key and drops high bits of the float sends this row to slot 0.)  The other rows probe differences of 0.5, 2^-31,
    8 and an exact tie."""
    T, S, d = 96, 32, 64
    layout = (("v", 32, 0), ("t", 64, -1))
    wl = variant(TINY, name="argmax_exact_two", n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=d, dtype="f32",
                 layout=layout, window=1, total_budget=S, recent_num=1, recent_den=1, seed=41)
    print(f"\n[case] {wl.name}: crafted keys, T={T} S={S}", flush=True)
    data = generate(wl)
    k = torch.zeros(1, 1, T, d, dtype=torch.float32)
    g = torch.Generator().manual_seed(3)
    k[0, 0, :T - S] = 0.01 * torch.randn(T - S, d, generator=g)
    for s_ in range(S):                         # the recent part (all of the budget): one axis each
        k[0, 0, T - S + s_, s_] = 1.0
    rows = {0: {0: 1.0, 1: 3.0}, 1: {4: 2.5, 9: 3.0}, 2: {2: 1.0, 3: 1.0 + 2.0 ** -31, 7: 1.0},
            3: {8: 1.0, 21: 9.0}, 4: {5: 2.0, 6: 2.0, 30: 2.0}, 5: {31: 4.0, 15: 2.0}, 6: {16: 3.0, 0: 1.0}}
    for r_, comps in rows.items():
        k[0, 0, r_] = 0.0
        for axis, val in comps.items():
            k[0, 0, r_, axis] = val
    data = dict(data, k=k)
    comp, gpu = run_gpu(wl, data)
    assert list(gpu["sel_idx"][:S]) == list(range(T - S, T))      # the conserved keys are the last S positions
    ma = gpu["merge_assign"][0, 0]
    want = {0: 1, 1: 9, 2: 2, 3: 21, 4: 5, 5: 31, 6: 16}           # ties (rows 2 and 4) go to the lowest slot
    got = {r_: int(ma[r_]) for r_ in want}
    assert got == want, got
    check_all(wl, data, gpu)


def test_single_window_row_with_scores_below_the_fp32_range():
    # one query row, a sharp softmax and a budget of three quarters of the sequence: the heavy keys take all the
    # probability and most columns have a score below 1e-40, which fp32 cannot rank; the conserved sets may differ
    # from the fp64 oracle's only inside that band (parity.py), everything downstream is checked on the GPU's set
    layout = (("t", 20, -1), ("v", 300, 0), ("t", 30, -1), ("v", 300, 1), ("t", 127, -1))
    stats = _case(variant(TINY, name="w1_sharp", n_layers=2, n_q_heads=2, n_kv_heads=2, head_dim=128, dtype="bf16",
                          layout=layout, window=1, total_budget=2 * 580, recent_num=1, recent_den=2, seed=26004,
                          tau_lo=2.5, tau_hi=3.0, heavy_frac=0.02))
    print("  conserved sets that differ inside the tie band:", stats["sets_differing_in_tie_band"])


def test_phase_timers_all_and_single():
    import paper_2502_17599_amd as pkg
    wl = variant(TINY, name="timers")
    data = generate(wl)
    names = [pkg.meda_phase_name(i) for i in range(pkg.N_PHASES)]
    try:
        pkg.meda_profile_enable(True)
        pkg.meda_profile_read(reset=True)
        _, ref = run_gpu(wl, data)
        ms, calls = pkg.meda_profile_read(reset=True)
        assert calls == 1 and all(m > 0.0 for m in ms)
        p = names.index("similarity")
        pkg.meda_profile_enable(True, p)
        _, a = run_gpu(wl, data)
        _, b = run_gpu(wl, data)
        ms, calls = pkg.meda_profile_read(reset=True)
        assert calls == 2 and ms[p] > 0.0 and all(m == 0.0 for i, m in enumerate(ms) if i != p)
    finally:
        pkg.meda_profile_enable(False)
    assert np.array_equal(a["k_out"], ref["k_out"]) and np.array_equal(b["v_out"], ref["v_out"])


def test_many_heads_small_context_both_similarity_kernels():
    # 8 layers x 32 kv heads = 256 (layer, head) pairs: enough for the resident-set similarity kernel to be used;
    # the temperature spread puts some layer budgets below and some above what fits into LDS (576 slots), so
    # both similarity kernels run in this one call
    layout = (("t", 40, -1), ("v", 576, 0), ("t", 30, -1), ("v", 576, 1), ("t", 58, -1), ("v", 576, 2), ("t", 192, -1))
    wl = variant(TINY, name="res_and_tiled", n_layers=8, n_q_heads=32, n_kv_heads=32, head_dim=128, dtype="bf16",
                 layout=layout, window=32, total_budget=8 * 600, tau_lo=0.5, tau_hi=3.0, seed=12)
    assert wl.seq_len == 2048
    data = generate(wl)
    comp, gpu = run_gpu(wl, data)
    S = gpu["S"]
    print("budgets", S.tolist(), flush=True)
    assert (S <= 576).any() and (S > 576).any(), S
    check_all(wl, data, gpu, heads=[(l, g) for l in range(wl.n_layers) for g in (0, 13, 31)])


def test_sequences_of_16384_positions_and_more_in_the_selection_kernel():
    # from 16384 positions on, a thread of the selection kernel takes four consecutive positions per iteration of its
    # output pass: a ragged length (the last thread's four positions straddle the end), a length that is a multiple of
    # the 4096 positions of an iteration, identical heavy-hitter keys (exact score ties at the cut), a recent part
    # that is not a multiple of four, text and vision candidates on both sides of the cut
    layout = (("t", 100, -1), ("v", 9000, 0), ("t", 1200, -1), ("v", 6000, 1), ("t", 89, -1))      # 16389 positions
    _case(variant(TINY, name="t16389", n_layers=2, n_q_heads=2, n_kv_heads=2, head_dim=64, dtype="f32", layout=layout,
                  window=32, total_budget=2 * 2001, seed=61, heavy_frac=0.02), threads=8)
    layout = (("v", 10000, 0), ("t", 300, -1), ("v", 10000, 1), ("t", 180, -1))                      # 20480 positions
    _case(variant(TINY, name="t20480", n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="bf16", layout=layout,
                  window=64, total_budget=2 * 333, seed=62, heavy_frac=0.02, recent_num=1, recent_den=3), threads=8)
