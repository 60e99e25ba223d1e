"""The decoding step through the entry point that allocates nothing (its chunk partials live in a device array
built into the library) against the same step through meda_decode_attention with a caller-provided workspace:
same kernels, so the outputs must be bit-identical; two calls in a row, the second on a smaller input, so that
whatever the first call left in the shared array is seen to do no harm.  Also checked against the fp64 oracle
with the tolerance of the decoding step."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import decode_oracle as D
from workloads import generate, get_workload, variant
from workloads.gen import to_float64

from parity import decode_error

pytestmark = pytest.mark.gpu


def _case(wl, n_new, seed):
    import paper_2502_17599_amd as pkg
    print(f"\n[no-alloc case] {wl.name}: L={wl.n_layers} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
          f"T={wl.seq_len} B={wl.total_budget} {wl.dtype} n_new={n_new}", flush=True)
    dev = torch.device("cuda:0")
    data = generate(wl)
    dt = data["q"].dtype
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, dt, wl.recent_num, wl.recent_den)
    cache = pkg.Compressor(params, dev)(data["q"].to(dev), data["k"].to(dev), data["v"].to(dev), data["mask"].to(dev))
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(wl.n_layers, wl.n_q_heads, wl.head_dim, generator=g).to(dt).to(dev)
    k_new = v_new = None
    if n_new:
        k_new = torch.randn(wl.n_layers, wl.n_kv_heads, n_new, wl.head_dim, generator=g).to(dt).to(dev)
        v_new = torch.randn(wl.n_layers, wl.n_kv_heads, n_new, wl.head_dim, generator=g).to(dt).to(dev)
    dparams = pkg.make_decode_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.total_budget, dt, n_new)
    assert pkg.meda_decode_workspace_bytes(dparams) <= pkg.DECODE_NOALLOC_MAX_BYTES
    want = pkg.Decoder(dparams, dev)(q, cache.k_out, cache.v_out, cache.layer_len, cache.layer_off, k_new, v_new).clone()
    got = torch.full_like(want, float("nan"))
    pkg.meda_decode_attention_noalloc(dparams, q, cache.k_out, cache.v_out, cache.layer_len, cache.layer_off, got,
                                      k_new, v_new)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), "outputs of the two entry points differ"
    # and against the oracle, layer by layer
    kc = cache.k_out.to(torch.float64).cpu().numpy(); vc = cache.v_out.to(torch.float64).cpu().numpy()
    ref = D.decode_step(to_float64(q.cpu()), kc, vc, cache.layer_len.cpu().numpy(), cache.layer_off.cpu().numpy(),
                        wl.n_kv_heads, None if k_new is None else to_float64(k_new.cpu()),
                        None if v_new is None else to_float64(v_new.cpu()))
    vmax = max(np.abs(vc).max(), 0.0 if v_new is None else float(v_new.abs().max()))
    err = decode_error(got.to(torch.float64).cpu().numpy(), ref, vmax, dt == torch.bfloat16)
    print(f"[no-alloc case] bit-identical to the workspace entry point; error against the oracle {err:.2e}", flush=True)


def test_no_alloc_decode_two_calls_second_smaller():
    big = variant(get_workload("long_multi_image"), n_layers=4,
                  layout=get_workload("llava7b_multi_image").layout, total_budget=4 * 1500)
    _case(big, n_new=300, seed=5)          # several chunks of cached rows and of appended rows
    small = variant(get_workload("tiny"), total_budget=2 * 100)
    _case(small, n_new=0, seed=6)          # one chunk, fp32, fewer layers and heads: most of the array keeps old data


def test_no_alloc_rejects_what_does_not_fit():
    import paper_2502_17599_amd as pkg
    # 128 layers x 64 heads x 64 chunks x 130 floats is above the built-in array: refused on the host, nothing launched
    dparams = pkg.make_decode_params(128, 64, 8, 128, 128 * 100000, torch.bfloat16)
    assert pkg.meda_decode_workspace_bytes(dparams) > pkg.DECODE_NOALLOC_MAX_BYTES
    dev = torch.device("cuda:0")
    dummy = torch.zeros(4096, dtype=torch.uint8, device=dev)
    out = torch.zeros(128, 64, 128, dtype=torch.bfloat16, device=dev)
    # through the library itself (the binding would first ask for a cache of 10^8 rows): the data pointers are never read
    import ctypes
    ptr = ctypes.c_void_p(dummy.data_ptr())
    st = pkg.load_library().meda_decode_attention_noalloc(ctypes.byref(dparams), ptr, ptr, ptr, ptr, ptr, None, None,
                                                          ctypes.c_void_p(out.data_ptr()), None)
    assert st == 6 and "scratch" in pkg.meda_status_string(st)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
