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
    stats = check_all(wl, data, gpu, heads=_sample_heads(wl, 24), threads=4)
    assert stats["ambiguous_rows"] <= 1e-3 * max(stats["rows"], 1)
    assert stats["layers_passing_only_by_entropy_floor"] == 0


def _full_size(name, n_heads, threads=1, extremes=False):
    wl = get_workload(name)
    print(f"\n[case] {wl.name} T={wl.seq_len} B={wl.total_budget}", flush=True)
    data = generate(wl, threads=16)
    comp, gpu = run_gpu(wl, data)

    def heads(S):
        pairs = _sample_heads(wl, n_heads)
        if extremes:   # the layers with the largest and the smallest budget (cap / floor of the allocation active)
            pairs = sorted(set(pairs) | {(int(np.argmax(S)), 0), (int(np.argmin(S)), wl.n_kv_heads - 1)})
        return pairs

    stats = check_all(wl, data, gpu, heads=heads, threads=threads)
    assert stats["ambiguous_rows"] <= 1e-3 * max(stats["rows"], 1)
    assert stats["layers_passing_only_by_entropy_floor"] == 0
    return stats


def test_long_multi_image_full_size():
    _full_size("long_multi_image", 6, threads=4, extremes=True)


def test_long_video_full_size():
    _full_size("long_video", 4, threads=4, extremes=True)


def test_extreme_full_size_all_layers():
    # 131072 positions: the oracle scores every layer (four side by side), so all 32 entropies and budgets are
    # compared; selection, matching and merging of ten (layer, head) pairs, among them the layer with the largest
    # and the one with the smallest budget
    stats = _full_size("extreme", 8, threads=4, extremes=True)
    assert stats["budgets_strictly_equal"]
