"""Decoding step over the ragged compressed cache: HIP path against the fp64 oracle, through the C ABI.

The cache the step reads is the HIP compression pass's own output (device tensors, never copied through the
oracle); the oracle gets the same bytes widened to fp64.  Tolerance: the kernel accumulates exact products in
fp32 and rounds the output once to the storage type, so the error is a few fp32 roundings of sums of d and of
S_l terms (observed 1e-8; allowed 1e-6 of the largest |v|) plus, for bf16, half an ulp of the value itself
(parity.decode_error).
"""
import numpy as np
import pytest
import torch

from oracle import decode_oracle as D
from workloads import generate, get_workload, variant
from workloads.gen import to_float64

from parity import decode_error

pytestmark = pytest.mark.gpu
TINY = get_workload("tiny")


def _compress(wl, data, dev):
    import paper_2502_17599_amd as pkg
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, data["q"].dtype, wl.recent_num, wl.recent_den)
    comp = pkg.Compressor(params, dev)
    return comp, comp(data["q"].to(dev), data["k"].to(dev), data["v"].to(dev), data["mask"].to(dev))


def _queries(wl, dtype, seed, n_new):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(wl.n_layers, wl.n_q_heads, wl.head_dim, generator=g).to(dtype)
    k_new = v_new = None
    if n_new:
        k_new = torch.randn(wl.n_layers, wl.n_kv_heads, n_new, wl.head_dim, generator=g).to(dtype)
        v_new = torch.randn(wl.n_layers, wl.n_kv_heads, n_new, wl.head_dim, generator=g).to(dtype)
    return q, k_new, v_new


def _check(wl, n_new=0, seed=11, layers=None):
    import paper_2502_17599_amd as pkg
    print(f"\n[decode case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} B={wl.total_budget} {wl.dtype} n_new={n_new}", flush=True)
    dev = torch.device("cuda:0")
    data = generate(wl)
    comp, cache = _compress(wl, data, dev)
    dt = data["q"].dtype
    q, k_new, v_new = _queries(wl, dt, seed, n_new)
    dparams = pkg.make_decode_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.total_budget, dt, n_new)
    dec = pkg.Decoder(dparams, dev)
    out = dec(q.to(dev), cache.k_out, cache.v_out, cache.layer_len, cache.layer_off,
              None if k_new is None else k_new.to(dev), None if v_new is None else v_new.to(dev))
    torch.cuda.synchronize()
    got = out.to(torch.float64).cpu().numpy()
    kc = cache.k_out.to(torch.float64).cpu().numpy(); vc = cache.v_out.to(torch.float64).cpu().numpy()
    S = cache.layer_len.cpu().numpy(); off = cache.layer_off.cpu().numpy()
    qn = to_float64(q)
    Hkv, d = wl.n_kv_heads, wl.head_dim
    worst = 0.0
    for l in (range(wl.n_layers) if layers is None else layers):
        a = int(off[l]) * Hkv
        k_l = kc[a:a + Hkv * S[l]].reshape(Hkv, S[l], d); v_l = vc[a:a + Hkv * S[l]].reshape(Hkv, S[l], d)
        ref = D.decode_layer(qn[l], k_l, v_l, None if k_new is None else to_float64(k_new[l]),
                             None if v_new is None else to_float64(v_new[l]))
        # the output is a convex combination of the cached and the appended value rows
        scale = max(np.abs(v_l).max(), 0.0 if v_new is None else float(v_new[l].abs().max()), 1e-30)
        worst = max(worst, decode_error(got[l], ref, scale, dt == torch.bfloat16))
    print(f"  max error / max|v| = {worst:.3e} (bound per element: 1e-6 max|v|"
          + (" + half a bf16 ulp of the value)" if dt == torch.bfloat16 else ")"), flush=True)
    # the second call with the same inputs is bit-identical
    out2 = dec(q.to(dev), cache.k_out, cache.v_out, cache.layer_len, cache.layer_off,
               None if k_new is None else k_new.to(dev), None if v_new is None else v_new.to(dev)).clone()
    torch.cuda.synchronize()
    assert torch.equal(out2, out)


def test_decode_tiny_fp32():
    _check(TINY)


def test_decode_tiny_with_appended_rows():
    _check(TINY, n_new=5)
    _check(TINY, n_new=300)          # more appended rows than one workgroup takes


def test_decode_grouped_heads_bf16_ragged_lengths():
    layout = (("t", 40, -1), ("v", 300, 0), ("t", 30, -1), ("v", 300, 1), ("t", 10, -1), ("v", 200, 2), ("t", 120, -1))
    for hq, hkv in ((8, 2), (6, 2), (7, 1), (8, 1), (4, 2)):      # groups of 4, 3, 7, 8, 2
        wl = variant(TINY, name=f"dec_g{hq // hkv}", n_layers=3, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, dtype="bf16",
                     layout=layout, window=32, total_budget=3 * 230, seed=2)
        _check(wl, n_new=3)


def test_decode_d64_and_fp32_d128():
    layout = (("t", 50, -1), ("v", 500, 0), ("t", 150, -1))
    _check(variant(TINY, name="dec_bf16_d64", n_layers=2, n_q_heads=4, n_kv_heads=1, head_dim=64, dtype="bf16",
                   layout=layout, window=64, total_budget=2 * 200, seed=5), n_new=2)
    _check(variant(TINY, name="dec_f32_d128", n_layers=2, n_q_heads=2, n_kv_heads=2, head_dim=128, dtype="f32",
                   layout=layout, window=32, total_budget=2 * 200, seed=4))


def test_decode_full_budget_is_attention_over_the_original_cache():
    wl = variant(TINY, name="dec_identity", total_budget=TINY.n_layers * TINY.seq_len)
    _check(wl)


def test_decode_llava7b_full_size_sampled_layers():
    wl = get_workload("llava7b_multi_image")
    _check(wl, n_new=17, layers=[0, 13, wl.n_layers - 1])


def test_decode_long_video_full_size_sampled_layers():
    # 7 query heads per kv head (padded to 8 in the kernel), 37376 positions, ragged budgets of the full-size pass
    wl = get_workload("long_video")
    _check(wl, n_new=5, layers=[0, 13, wl.n_layers - 1])


def test_decode_long_multi_image_full_size_sampled_layers():
    # 4 query heads per kv head at full size
    wl = get_workload("long_multi_image")
    _check(wl, n_new=0, layers=[1, wl.n_layers - 2])
