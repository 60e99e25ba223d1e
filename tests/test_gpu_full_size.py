"""Full-size workloads in the launch configuration the benchmark times: scores, entropies and budgets of
every layer against the oracle, and selection / assignment / merged rows of sampled (layer, head) pairs."""
import numpy as np
import pytest

from workloads import generate, get_workload

from parity import check_all, run_gpu

pytestmark = pytest.mark.gpu


def _sample_heads(wl, n, seed=0):
    r = np.random.default_rng(seed)
    pairs = {(0, 0), (wl.n_layers - 1, wl.n_kv_heads - 1)}
    while len(pairs) < n:
        pairs.add((int(r.integers(wl.n_layers)), int(r.integers(wl.n_kv_heads))))
    return sorted(pairs)


def test_llava7b_multi_image_full_size():
    wl = get_workload("llava7b_multi_image")
    print(f"\n[case] {wl.name} T={wl.seq_len} B={wl.total_budget}", flush=True)
    data = generate(wl, threads=16)
    comp, gpu = run_gpu(wl, data)
    stats = check_all(wl, data, gpu, heads=_sample_heads(wl, 24))
    assert stats["ambiguous_rows"] <= 1e-3 * max(stats["rows"], 1)


def _full_size(name, n_heads, score_layers=None):
    wl = get_workload(name)
    print(f"\n[case] {wl.name} T={wl.seq_len} B={wl.total_budget}", flush=True)
    data = generate(wl, threads=16)
    comp, gpu = run_gpu(wl, data)
    heads = _sample_heads(wl, n_heads)
    if score_layers is not None:
        heads = [(l, g) for l, g in heads if l in score_layers]
    stats = check_all(wl, data, gpu, heads=heads, score_layers=score_layers)
    assert stats["ambiguous_rows"] <= 1e-3 * max(stats["rows"], 1)
    return stats


def test_long_multi_image_full_size():
    _full_size("long_multi_image", 6)


def test_long_video_full_size():
    _full_size("long_video", 4)


def test_extreme_full_size_sampled_layers():
    # 131072 positions: the oracle scores two layers (first and last); selection, matching and merging are
    # checked for one head of each against the oracle run with the budgets validated in check_all
    wl = get_workload("extreme")
    _full_size("extreme", 2, score_layers=[0, wl.n_layers - 1])
