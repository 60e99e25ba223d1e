"""The synthetic workloads have the stated shapes, layouts and budgets, and are reproducible."""
import numpy as np
import torch

from workloads import WORKLOADS, generate, get_workload, modality_mask, variant
from workloads.gen import generate_layer, layer_taus


def test_shapes_and_budgets_of_the_named_workloads():
    want = {
        "tiny": (2, 4, 4, 64, "f32", 1024, 768, 32, 512),
        "llava7b_multi_image": (32, 32, 32, 128, "bf16", 4096, 3456, 32, 16384),
        "long_multi_image": (32, 32, 8, 128, "bf16", 16384, 13824, 64, 104857),
        "long_video": (28, 28, 4, 128, "bf16", 37376, 36864, 64, 156979),
        "extreme": (32, 32, 8, 128, "bf16", 131072, 126720, 64, 419430),
    }
    for name, (L, Hq, Hkv, d, dt, T, nv, W, B) in want.items():
        wl = WORKLOADS[name]
        assert (wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype) == (L, Hq, Hkv, d, dt)
        assert (wl.seq_len, wl.n_vision, wl.window, wl.total_budget) == (T, nv, W, B)
        mask = modality_mask(wl)
        assert mask.shape == (T,) and int(mask.sum()) == nv
        assert np.all(mask[-W:] == 0)                # the observation window is text


def test_generation_is_reproducible_and_layerwise():
    wl = variant(get_workload("tiny"), n_layers=3)
    a = generate(wl, threads=1)
    b = generate(wl, threads=3)
    for key in ("q", "k", "v"):
        assert torch.equal(a[key], b[key])
    only1 = generate(wl, layers=[1])
    assert torch.equal(only1["k"][0], a["k"][1])


def test_structure_of_keys():
    wl = get_workload("tiny")
    q, k, v = generate_layer(wl, 0)
    tau = layer_taus(wl)[0]
    assert 0.5 <= tau <= 3.0
    assert abs(q.std() / tau - 1.0) < 0.05
    # heavy hitters: floor(2 % of T) identical keys of norm 3*sqrt(d) per head
    for g in range(wl.n_kv_heads):
        norms = np.linalg.norm(k[g], axis=1)
        heavy = np.flatnonzero(np.abs(norms - 3 * np.sqrt(wl.head_dim)) < 1e-3)
        assert len(heavy) == int(0.02 * wl.seq_len)
        assert np.all(k[g, heavy] == k[g, heavy[0]])
    # vision keys sit within ~sigma of one of 16 centres: nearest-neighbour distances are small
    mask = modality_mask(wl)
    vis = np.flatnonzero(mask == 1)[:256]
    kk = k[0, vis]
    d2 = ((kk[:, None, :] - kk[None, :, :]) ** 2).sum(-1) + np.eye(len(vis)) * 1e9
    assert np.median(np.sqrt(d2.min(axis=1))) < 0.3 * np.sqrt(2 * wl.head_dim) * 1.2


def test_bf16_storage_is_exact_in_float32():
    wl = variant(get_workload("llava7b_multi_image"), n_layers=1, n_q_heads=2, n_kv_heads=2)
    d = generate(wl)
    assert d["k"].dtype == torch.bfloat16 and d["k"].shape == (1, 2, 4096, 128)
