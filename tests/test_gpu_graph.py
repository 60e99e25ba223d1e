"""The pass and the decoding step recorded into a HIP graph: every replay must equal the eager result (the library
records only kernel launches; the replays are interleaved with eager calls and synchronisations)."""
import time

import pytest
import torch

from workloads import generate, get_workload, variant

pytestmark = pytest.mark.gpu
TINY = get_workload("tiny")


def test_graph_replays_equal_eager_results():
    import paper_2502_17599_amd as pkg
    dev = torch.device("cuda:0")
    wl = variant(TINY, name="graph")
    data = generate(wl)
    q, k, v, mask = (data[n].to(dev) for n in ("q", "k", "v", "mask"))
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, q.dtype, wl.recent_num, wl.recent_den)
    comp = pkg.Compressor(params, dev, want_merge_assign=True)
    dq = torch.randn(wl.n_layers, wl.n_q_heads, wl.head_dim, generator=torch.Generator().manual_seed(3)).to(q.dtype).to(dev)
    dec = pkg.Decoder(pkg.make_decode_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.total_budget,
                                             q.dtype), dev)
    pkg.meda_profile_enable(False)

    def step(stream=None):
        out = comp(q, k, v, mask, stream)
        att = dec(dq, out.k_out, out.v_out, out.layer_len, out.layer_off, None, None, stream)
        return out, att

    out, att = step()                       # eager reference (also loads every code object before the capture)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out.k_out, out.v_out, out.layer_len, out.layer_off, out.sel_idx, out.merge_assign, att)]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream(dev))
    for i in range(3):
        for t in (out.k_out, out.v_out, att):
            t.zero_()                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        now = (out.k_out, out.v_out, out.layer_len, out.layer_off, out.sel_idx, out.merge_assign, att)
        for a, b in zip(ref, now):
            assert torch.equal(a, b), f"replay {i}"
        step()                              # and an eager call between the replays
        torch.cuda.synchronize()

    def timed(fn, n=200):
        torch.cuda.synchronize(); t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize(); return (time.perf_counter() - t0) / n * 1e3
    print(f"\n  tiny: eager {timed(step):.4f} ms per pass + decoding step, graph replay {timed(graph.replay):.4f} ms", flush=True)
