"""Several sequences per call (meda_params.n_seqs): every sequence of a batch must come out exactly as from a
call of its own, and as the oracle computes it on its own; the decoding step runs on a sequence's slice of the
batched result.  The sequences of a batch differ in seed and in the positions of their vision segments."""
import numpy as np
import pytest
import torch

from oracle import decode_oracle, meda_oracle
from workloads import generate, generate_batch, get_workload, variant
from workloads.gen import to_float64

from parity import decode_error

pytestmark = pytest.mark.gpu


def _batch_workloads(base, layouts):
    return [variant(base, layout=lay, seed=11 + 7 * i) for i, lay in enumerate(layouts)]


def _run_batch(wls, dev, flags=0):
    import paper_2502_17599_amd as pkg
    w0 = wls[0]
    data = generate_batch(wls)
    params = pkg.make_params(w0.n_layers, w0.n_q_heads, w0.n_kv_heads, w0.head_dim, w0.seq_len, w0.window,
                             w0.total_budget, data["q"].dtype, w0.recent_num, w0.recent_den, 0.0, flags, len(wls))
    comp = pkg.Compressor(params, dev, want_merge_assign=True)
    out = comp(data["q"].to(dev), data["k"].to(dev), data["v"].to(dev), data["mask"].to(dev))
    torch.cuda.synchronize()
    return data, out


def _run_single(wl, data_n, dev, flags=0):
    import paper_2502_17599_amd as pkg
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, data_n["q"].dtype, wl.recent_num, wl.recent_den, 0.0, flags)
    comp = pkg.Compressor(params, dev, want_merge_assign=True)
    out = comp(data_n["q"].to(dev), data_n["k"].to(dev), data_n["v"].to(dev), data_n["mask"].to(dev))
    torch.cuda.synchronize()
    return out


def _check_against_single_and_oracle(wls, flags=0, oracle=True):
    dev = torch.device("cuda:0")
    data, out = _run_batch(wls, dev, flags)
    w0 = wls[0]
    N, L, Hkv, B = len(wls), w0.n_layers, w0.n_kv_heads, w0.total_budget
    assert out.layer_len.shape == (N, L) and out.layer_off.shape == (N, L + 1)
    rows_per_seq = B * Hkv
    for n, wl in enumerate(wls):
        data_n = {key: data[key][n].contiguous() for key in ("q", "k", "v", "mask")}
        single = _run_single(wl, data_n, dev, flags)
        seq = out.sequence(n)
        # absolute offsets: the sequence's block starts at n*B
        off_b = seq.layer_off.cpu().numpy()
        assert off_b[0] == n * B and off_b[-1] == (n + 1) * B
        assert np.array_equal(off_b - n * B, single.layer_off.cpu().numpy())
        assert torch.equal(seq.layer_len, single.layer_len)
        assert torch.equal(seq.entropy, single.entropy)                       # bit-identical doubles
        blk = slice(n * rows_per_seq, (n + 1) * rows_per_seq)
        assert torch.equal(out.sel_idx[blk], single.sel_idx)
        assert torch.equal(out.k_out[blk].view(torch.uint8), single.k_out.view(torch.uint8))
        assert torch.equal(out.v_out[blk].view(torch.uint8), single.v_out.view(torch.uint8))
        assert torch.equal(seq.merge_assign, single.merge_assign)
        if not oracle:
            continue
        # and the oracle on this sequence alone (budgets, entropies, index sets, merged rows)
        ref = meda_oracle.meda_compress_batch(to_float64(data["q"][n:n + 1]), to_float64(data["k"][n:n + 1]),
                                              to_float64(data["v"][n:n + 1]), data["mask"][n:n + 1].numpy(),
                                              B, wl.window, wl.dtype)[0]
        np.testing.assert_allclose(seq.entropy.cpu().numpy(), ref["entropy"], rtol=1e-3)
        if np.array_equal(seq.layer_len.cpu().numpy(), ref["S"]):
            tol = 2e-2 if wl.dtype == "bf16" else 1e-4
            for l in range(L):
                k_l, v_l, idx_l = seq.layer(l)
                for g in range(Hkv):
                    assert idx_l[g].cpu().tolist() == ref["heads"][l][g]["idx_c"].tolist(), (n, l, g)
                scale = max(1.0, float(np.abs(ref["k_out"][l]).max()))
                assert np.abs(k_l.double().cpu().numpy() - ref["k_out"][l]).max() <= tol * scale
                assert np.abs(v_l.double().cpu().numpy() - ref["v_out"][l]).max() <= tol * max(
                    1.0, float(np.abs(ref["v_out"][l]).max()))
        else:  # a budget on a rounding boundary of the entropy softmax: only the sums are fixed
            assert int(seq.layer_len.sum()) == B
    return data, out


def test_batch_of_three_tiny_f32():
    base = get_workload("tiny")                    # T = 1024 = 768 vision + 256 text
    layouts = [base.layout,
               (("t", 100, -1), ("v", 600, 0), ("t", 60, -1), ("v", 168, 1), ("t", 96, -1)),
               (("v", 300, 0), ("t", 724, -1))]
    _check_against_single_and_oracle(_batch_workloads(base, layouts))


def test_batch_uniform_budget_flag():
    base = get_workload("tiny")
    layouts = [base.layout, (("t", 512, -1), ("v", 256, 0), ("t", 256, -1))]
    # the flag's own behaviour is checked on single calls; here only that a batch reproduces them
    _check_against_single_and_oracle(_batch_workloads(base, layouts), flags=1, oracle=False)


def test_batch_grouped_heads_bf16_and_decode():
    import paper_2502_17599_amd as pkg
    base = variant(get_workload("tiny"), name="batch_gqa", n_layers=3, n_q_heads=8, n_kv_heads=2, head_dim=128,
                   dtype="bf16", window=64, total_budget=3 * 200,
                   layout=(("t", 40, -1), ("v", 700, 0), ("t", 159, -1)))       # ragged T = 899
    layouts = [base.layout, (("v", 450, 0), ("t", 100, -1), ("v", 249, 1), ("t", 100, -1)),
               (("t", 899, -1),), (("t", 10, -1), ("v", 800, 0), ("t", 89, -1))]
    wls = _batch_workloads(base, layouts)
    data, out = _check_against_single_and_oracle(wls)
    # one decoding step on the slice of sequence 2 of the batched result
    dev = out.k_out.device
    n = 2
    g = torch.Generator().manual_seed(5)
    q = torch.randn(base.n_layers, base.n_q_heads, base.head_dim, generator=g).to(torch.bfloat16)
    seq = out.sequence(n)
    dparams = pkg.make_decode_params(base.n_layers, base.n_q_heads, base.n_kv_heads, base.head_dim,
                                     len(wls) * base.total_budget, torch.bfloat16)
    att = pkg.Decoder(dparams, dev)(q.to(dev), out.k_out, out.v_out, seq.layer_len, seq.layer_off)
    torch.cuda.synchronize()
    ref = decode_oracle.decode_step(to_float64(q), out.k_out.double().cpu().numpy(), out.v_out.double().cpu().numpy(),
                                    seq.layer_len.cpu().numpy(), seq.layer_off.cpu().numpy(), base.n_kv_heads)
    decode_error(att.double().cpu().numpy(), ref, np.abs(out.v_out.double().cpu().numpy()).max(), True)


@pytest.mark.parametrize("cfg", [
    dict(n_layers=1, n_q_heads=3, n_kv_heads=3, head_dim=64, dtype="f32", window=17, T=333, B=1 * 60, n=5, flags=0),
    dict(n_layers=5, n_q_heads=8, n_kv_heads=1, head_dim=128, dtype="bf16", window=64, T=1500, B=5 * 700, n=2, flags=0),
    dict(n_layers=2, n_q_heads=6, n_kv_heads=3, head_dim=128, dtype="bf16", window=32, T=700, B=2 * 90, n=3, flags=2),
    dict(n_layers=4, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="bf16", window=40, T=2100, B=4 * 2100, n=2, flags=0),
])
def test_batch_other_shapes_match_single_calls(cfg):
    """Odd sizes, one kv head, eviction instead of merging, a budget that keeps everything: a batch still
    reproduces the single calls bit for bit (the single calls' own parity is covered elsewhere)."""
    T = cfg["T"]
    base = variant(get_workload("tiny"), name="batch_misc", n_layers=cfg["n_layers"], n_q_heads=cfg["n_q_heads"],
                   n_kv_heads=cfg["n_kv_heads"], head_dim=cfg["head_dim"], dtype=cfg["dtype"], window=cfg["window"],
                   total_budget=cfg["B"], layout=(("t", T // 5, -1), ("v", T - T // 5 - T // 7, 0), ("t", T // 7, -1)))
    layouts = [base.layout]
    for i in range(1, cfg["n"]):
        a = T // (3 + i)
        layouts.append((("v", a, 0), ("t", T - a, -1)) if i % 2 else (("t", a, -1), ("v", T - 2 * a, 0), ("t", a, -1)))
    _check_against_single_and_oracle(_batch_workloads(base, layouts), flags=cfg["flags"], oracle=False)


def test_batch_with_every_prompt_row_scoring():
    """The batch dimension and MEDA_FLAG_FULL_PROMPT together (row blocks x sequences)."""
    import paper_2502_17599_amd as pkg
    base = variant(get_workload("tiny"), name="batch_fp", n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="f32",
                   window=32, total_budget=2 * 120, layout=(("t", 60, -1), ("v", 200, 0), ("t", 40, -1)), score_rows=300)
    layouts = [base.layout, (("v", 150, 0), ("t", 150, -1)), (("t", 20, -1), ("v", 100, 0), ("t", 180, -1))]
    wls = _batch_workloads(base, layouts)
    _, out = _check_against_single_and_oracle(wls, flags=pkg.FLAG_FULL_PROMPT, oracle=False)
    # the oracle on one of the sequences (every row scores: q has T rows)
    from workloads import generate
    n = 1
    data_n = generate(wls[n])
    ref = meda_oracle.meda_compress(to_float64(data_n["q"]), to_float64(data_n["k"]), to_float64(data_n["v"]),
                                    data_n["mask"].numpy(), base.total_budget, base.window, base.dtype)
    seq = out.sequence(n)
    np.testing.assert_allclose(seq.entropy.cpu().numpy(), ref["entropy"], rtol=1e-3)
    if np.array_equal(seq.layer_len.cpu().numpy(), ref["S"]):
        for l in range(base.n_layers):
            _, _, idx_l = seq.layer(l)
            for g in range(base.n_kv_heads):
                assert idx_l[g].cpu().tolist() == ref["heads"][l][g]["idx_c"].tolist()


def test_batch_limits():
    import paper_2502_17599_amd as pkg
    # 129 sequences of 2 layers exceed the 256 layers one call handles
    p = pkg.make_params(2, 4, 4, 64, 1024, 32, 512, torch.float32, n_seqs=129)
    assert pkg.meda_workspace_bytes(p) == 0
    p = pkg.make_params(2, 4, 4, 64, 1024, 32, 512, torch.float32, n_seqs=128)
    assert pkg.meda_workspace_bytes(p) > 0
    p = pkg.make_params(2, 4, 4, 64, 1024, 32, 512, torch.float32, n_seqs=-1)
    assert pkg.meda_workspace_bytes(p) == 0
