"""Every prompt position scores the keys (MEDA_FLAG_FULL_PROMPT; Sections 3.2 / 3.3 as the paper writes them):
HIP path against the fp64 oracle, same rules as the observation-window tests."""
import numpy as np
import pytest

from workloads import generate, get_workload, variant

from parity import check_all, run_gpu

pytestmark = pytest.mark.gpu
TINY = get_workload("tiny")
VT_LAYOUT = (("t", 64, -1), ("v", 256, 0), ("v", 256, 1), ("v", 256, 2), ("t", 160, -1), ("v", 16, 2), ("t", 16, -1))


def _case(wl, **kw):
    print(f"\n[full-prompt case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} W={wl.window} B={wl.total_budget} {wl.dtype}", flush=True)
    assert wl.n_score_rows == wl.seq_len
    data = generate(wl)
    assert data["q"].shape[2] == wl.seq_len
    comp, gpu = run_gpu(wl, data)
    return check_all(wl, data, gpu, **kw), gpu


def test_full_prompt_tiny_fp32_eight_row_blocks():
    stats, gpu = _case(variant(TINY, name="fp_tiny", score_rows=TINY.seq_len))
    assert stats["budgets_strictly_equal"]


def test_full_prompt_differs_from_the_window_variant():
    wl = variant(TINY, name="fp_vs_window", layout=VT_LAYOUT)
    _, win = run_gpu(wl, generate(wl))
    stats, full = _case(variant(wl, score_rows=wl.seq_len))
    # same keys (the generator draws them from the same streams), other rows: other scores and entropies
    assert not np.allclose(full["entropy"], win["entropy"], rtol=1e-3)


def test_full_prompt_ragged_bf16_grouped_heads():
    # T = 1000 = 7 blocks of 128 rows + one of 104; 4 query heads per kv head
    layout = (("t", 40, -1), ("v", 300, 0), ("t", 30, -1), ("v", 300, 1), ("t", 10, -1), ("v", 200, 2), ("t", 120, -1))
    wl = variant(TINY, name="fp_bf16_g4", n_layers=3, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16",
                 layout=layout, window=32, total_budget=3 * 230, seed=1, score_rows=1000)
    _case(wl)


def test_full_prompt_group_of_eight_and_short_sequence():
    layout = (("t", 30, -1), ("v", 500, 0), ("t", 100, -1), ("v", 300, 1), ("t", 94, -1))
    _case(variant(TINY, name="fp_g8", n_layers=2, n_q_heads=8, n_kv_heads=1, head_dim=128, dtype="bf16",
                  layout=layout, window=64, total_budget=2 * 300, seed=8, score_rows=1024))
    # one block only, shorter than a full block
    short = (("v", 40, 0), ("t", 24, -1), ("v", 20, 1), ("t", 12, -1))
    _case(variant(TINY, name="fp_short", n_layers=2, n_q_heads=2, n_kv_heads=1, layout=short, window=16,
                  total_budget=2 * 40, seed=6, score_rows=96))


def test_full_prompt_sixteen_query_heads_per_kv_head():
    # pass A then holds one 32-row block of each of the 16 heads per workgroup; T = 300 leaves ragged row blocks in both
    # scoring passes (32-row blocks in the first, 128-row blocks in the second)
    layout = (("t", 20, -1), ("v", 120, 0), ("t", 30, -1), ("v", 90, 1), ("t", 40, -1))
    _case(variant(TINY, name="fp_g16", n_layers=2, n_q_heads=16, n_kv_heads=1, head_dim=128, dtype="bf16",
                  layout=layout, window=32, total_budget=2 * 100, seed=12, score_rows=300))


def test_full_prompt_three_query_heads_per_kv_head_d64():
    # 5 row blocks of 32 rows per pass-A workgroup (15 (head, row block) pairs), head dimension 64
    layout = (("t", 33, -1), ("v", 200, 0), ("t", 17, -1), ("v", 150, 1), ("t", 50, -1))
    _case(variant(TINY, name="fp_g3", n_layers=2, n_q_heads=6, n_kv_heads=2, head_dim=64, dtype="bf16",
                  layout=layout, window=16, total_budget=2 * 120, seed=13, score_rows=450))


def test_full_prompt_fp32_head_dim_128_takes_the_row_block_mode_of_the_window_kernel():
    # rows of 512 bytes do not fit the two-stage LDS ring of the dedicated kernel: pass B falls back to the window
    # kernel walking the row blocks itself; T = 700 = 5 blocks of 128 rows + one of 60
    layout = (("t", 50, -1), ("v", 250, 0), ("t", 40, -1), ("v", 260, 1), ("t", 100, -1))
    _case(variant(TINY, name="fp_f32_d128", n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=128, dtype="f32",
                  layout=layout, window=32, total_budget=2 * 150, seed=17, score_rows=700))


def test_full_prompt_mid_size_bf16_one_head_per_kv_head():
    # 16 row blocks, 8 heads without grouping, several layers with different temperatures
    layout = (("t", 40, -1), ("v", 576, 0), ("t", 30, -1), ("v", 576, 1), ("t", 58, -1), ("v", 576, 2), ("t", 192, -1))
    wl = variant(TINY, name="fp_mid", n_layers=4, n_q_heads=8, n_kv_heads=8, head_dim=128, dtype="bf16",
                 layout=layout, window=32, total_budget=4 * 400, seed=21, score_rows=2048)
    _case(wl, heads=[(l, g) for l in range(4) for g in (0, 5)])


def test_full_prompt_llava7b_shape_two_layers():
    # the shape the full-prompt mode is benchmarked on (32 heads without grouping, 4096 positions, 32 row blocks),
    # two layers with different temperatures; the oracle takes a few minutes for them, run side by side
    base = get_workload("llava7b_multi_image")
    wl = variant(base, name="fp_llava7b_2_layers", n_layers=2, total_budget=2 * 512, score_rows=base.seq_len)
    print(f"\n[full-prompt case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} W={wl.window} B={wl.total_budget} {wl.dtype}", flush=True)
    data = generate(wl)
    comp, gpu = run_gpu(wl, data)
    stats = check_all(wl, data, gpu, heads=[(0, 0), (0, 17), (1, 31)], threads=2)
    assert stats["layers_passing_only_by_entropy_floor"] == 0
