"""Comparison of the HIP path with the fp64 oracle on the same seeded inputs (helper, not a test).

Rules (tolerances of the compression pass):
  * column scores: relative 1e-4 (they only feed the ranking)
  * entropies: relative 1e-3
  * layer budgets: bit-exact.  The budgets round B * softmax(E); two correct implementations whose
    entropies differ in the 7th digit can round a layer differently, so a mismatch is accepted only
    if the oracle's allocator, given entropies inside the entropy tolerance (the GPU's), returns
    exactly the GPU's budgets; the affected layers are then checked against the oracle run with
    those budgets.  Strict equality is reported separately.
  * conserved index sets: bit-exact, except where the oracle's N-th and (N+1)-th boosted scores differ
    by less than 1e-4 relative: then every index that differs must have a boosted score within 1e-4
    relative of the N-th score.
  * nearest-neighbour slots: equal to the oracle's, or the oracle's cosine of the GPU's choice is
    within 1e-5 of the oracle's best (near-ties inside fp32 accumulation error); such rows are counted.
  * merged K/V: |gpu - oracle| <= 2e-2 (bf16) / 1e-4 (fp32); where index set or assignment legitimately
    differ, the oracle's merge is evaluated on the validated index set / assignment.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import meda_oracle as O
from workloads.gen import to_float64

KV_TOL = {"bf16": 2e-2, "f32": 1e-4}


def run_gpu(wl, data, device="cuda:0", flags=0):
    """Run the HIP path; returns the Compressor (for workspace regions) and host copies of all outputs."""
    import paper_2502_17599_amd as pkg
    dev = torch.device(device)
    dt = data["q"].dtype
    if wl.n_score_rows == wl.seq_len and wl.seq_len != wl.window:
        flags |= pkg.FLAG_FULL_PROMPT       # the workload carries a query for every prompt position
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, dt, wl.recent_num, wl.recent_den, 0.0, flags)
    comp = pkg.Compressor(params, dev, want_merge_assign=True)
    out = comp(data["q"].to(dev), data["k"].to(dev), data["v"].to(dev), data["mask"].to(dev))
    torch.cuda.synchronize()
    L, Hkv, T = wl.n_layers, wl.n_kv_heads, wl.seq_len
    res = {
        "entropy": out.entropy.cpu().numpy(),
        "S": out.layer_len.cpu().numpy().astype(np.int64),
        "off": out.layer_off.cpu().numpy(),
        "sel_idx": out.sel_idx.cpu().numpy(),
        "merge_assign": out.merge_assign.cpu().numpy(),
        "k_out": out.k_out.to(torch.float64).cpu().numpy(),
        "v_out": out.v_out.to(torch.float64).cpu().numpy(),
        "col_scores": comp.region("col_scores", torch.float32).cpu().numpy().reshape(L, Hkv, T),
        "inv_norm": comp.region("inv_norm", torch.float32).cpu().numpy().reshape(L, Hkv, T),
        "alloc": comp.region("alloc", torch.int32).cpu().numpy().reshape(L, 4),
    }
    return comp, res


def gpu_head(wl, gpu, l, g):
    """Conserved positions and output rows of one (layer, head) from the ragged GPU output."""
    Hkv = wl.n_kv_heads
    S = int(gpu["S"][l]); off = int(gpu["off"][l])
    a = off * Hkv + g * S
    return gpu["sel_idx"][a:a + S], gpu["k_out"][a:a + S], gpu["v_out"][a:a + S]


def oracle_scores(wl, data, layers=None, threads=1):
    """Oracle column scores and entropies for the given layers (all by default).  ``threads`` > 1 runs that many
    layers side by side (numpy releases the interpreter lock inside its loops); the result does not depend on it."""
    q = data["q"]; k = data["k"]; mask = data["mask"].numpy()
    layers = list(range(wl.n_layers) if layers is None else layers)

    slow = q.shape[1] * q.shape[2] * k.shape[2] >= (1 << 26)   # a layer takes seconds: say that it is alive

    def one(l):
        r = O.layer_scores_and_entropy(to_float64(q[l]), to_float64(k[l]), mask)
        if slow:
            print(f"[oracle {wl.name}] layer {l} scored", flush=True)
        return r

    if threads > 1 and len(layers) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as pool:
            results = list(pool.map(one, layers))
    else:
        results = [one(l) for l in layers]
    a_s = {l: r[0] for l, r in zip(layers, results)}
    ent = {l: r[1] for l, r in zip(layers, results)}
    return a_s, ent


def budget_margins(wl, e_ref):
    """How far every layer's budget is from being rounded the other way.

    The integer budgets are floor(x_l) plus one for the layers with the largest fractional parts (largest
    remainder).  A layer that got the extra slot loses it when its fractional part falls below the best one that
    did not get it; a layer that did not get it gains it when its fractional part rises above the worst one that
    did.  Returns (margin in slots, relative entropy change that would move x_l by that margin) per layer; layers
    pinned at the floor or the cap have an infinite margin unless their clamp is about to release.  With x_l
    proportional to exp(E_l), dx_l = x_l dE_l (the shift of the water level by one layer's change is second order)."""
    lo, hi = min(wl.window, wl.seq_len), wl.seq_len
    x = O.allocation_reals(np.asarray(e_ref, dtype=np.float64), wl.total_budget, lo, hi)
    fl = np.floor(x)
    frac = x - fl
    S, _, _, _ = O.allocate_budgets(np.asarray(e_ref, dtype=np.float64), wl.total_budget, wl.seq_len, wl.window,
                                    wl.recent_num, wl.recent_den)
    got = (S - fl.astype(np.int64)) > 0
    free = (x > lo) & (x < hi)
    margin = np.full(len(x), np.inf)
    if got.any() and (~got & free).any():
        best_without = frac[~got & free].max()
        worst_with = frac[got].min()
        margin[got] = frac[got] - best_without
        sel = ~got & free
        margin[sel] = worst_with - frac[sel]
    margin = np.where(free, margin, np.inf)
    rel_entropy = margin / np.maximum(x, 1.0) / np.maximum(np.abs(e_ref), 1e-30)
    return margin, rel_entropy


def check_budgets(wl, gpu, ent_oracle):
    """Returns (S, M, N, off) to be used downstream and a flag telling whether equality was strict."""
    e_ref = np.array([ent_oracle[l][2] for l in range(wl.n_layers)])
    S, M, N, off = O.allocate_budgets(e_ref, wl.total_budget, wl.seq_len, wl.window, wl.recent_num, wl.recent_den)
    assert int(gpu["S"].sum()) == wl.total_budget and int(gpu["off"][-1]) == wl.total_budget
    assert np.array_equal(np.diff(gpu["off"]), gpu["S"])
    if np.array_equal(gpu["S"], S):
        strict = True
    else:
        strict = False
        S2, M, N, off = O.allocate_budgets(gpu["entropy"], wl.total_budget, wl.seq_len, wl.window,
                                           wl.recent_num, wl.recent_den)
        assert np.array_equal(gpu["S"], S2), f"budgets {gpu['S']} not explained by the entropy tolerance ({S})"
        assert np.abs(gpu["S"] - S).max() <= max(2, int(1e-3 * S.max())), (gpu["S"], S)
        S = S2
    assert np.array_equal(gpu["alloc"][:, 0], S) and np.array_equal(gpu["alloc"][:, 1], M)
    assert np.array_equal(gpu["alloc"][:, 2], N)
    return (S, M, N, off), strict


def check_head(wl, data, gpu, a_s_oracle, l, g, n_top, n_recent, stats):
    """Selection, assignment and merged rows of one (layer, head) against the oracle."""
    mask = data["mask"].numpy()
    k = to_float64(data["k"][l, g]); v = to_float64(data["v"][l, g])
    T = wl.seq_len
    idx_gpu, k_gpu, v_gpu = gpu_head(wl, gpu, l, g)
    idx_c, idx_less = O.select_tokens(a_s_oracle[g], mask, n_top, n_recent)
    if not np.array_equal(idx_gpu, idx_c):
        boosted = O.boosted_scores(a_s_oracle[g], mask)
        cand = boosted[:T - n_recent]
        kth = np.sort(cand)[::-1][n_top - 1]
        diff = np.setxor1d(idx_gpu, idx_c)
        assert len(idx_gpu) == len(idx_c) and np.all(np.diff(idx_gpu) > 0), "conserved set malformed"
        # The selection is decided in the kernel's precision, fp32: a probability below the smallest normal number
        # (2^-126) may reach the column sum as zero, so scores that differ by less than (terms summed) x 2^-126
        # cannot be told apart there, however far apart they are in the oracle's fp64 (a single window row with a
        # sharp softmax leaves most columns below 1e-40).
        floor = wl.n_score_rows * (wl.n_q_heads // wl.n_kv_heads) * 2.0 ** -126
        assert np.all(np.abs(boosted[diff] - kth) <= 1e-4 * abs(kth) + floor), \
            f"layer {l} head {g}: index sets differ outside the 1e-4 tie band at {diff[:8]}"
        stats["sets_differing_in_tie_band"] += 1
        idx_c = idx_gpu.astype(np.int64)
        keep = np.zeros(T, bool); keep[idx_c] = True
        idx_less = np.flatnonzero(~keep)
    stats["heads"] += 1
    ma = gpu["merge_assign"][l, g]
    assert np.array_equal(ma[idx_c], np.arange(len(idx_c))), "conserved positions must map to their own slot"
    if len(idx_less) == 0:
        assign = np.empty(0, np.int64)
    else:
        assign = O.nn_assign(k, idx_c, idx_less)
        slot_gpu = ma[idx_less].astype(np.int64)
        bad = np.flatnonzero(slot_gpu != assign)
        if len(bad):
            assert slot_gpu.min() >= 0 and slot_gpu.max() < len(idx_c)
            u_best = np.einsum("ij,ij->i", _unit(k[idx_less[bad]]), _unit(k[idx_c[assign[bad]]]))
            u_gpu = np.einsum("ij,ij->i", _unit(k[idx_less[bad]]), _unit(k[idx_c[slot_gpu[bad]]]))
            assert np.all(u_best - u_gpu <= 1e-5), \
                f"layer {l} head {g}: {np.sum(u_best - u_gpu > 1e-5)} rows assigned to a worse slot"
            stats["ambiguous_rows"] += len(bad)
            assign = slot_gpu
        stats["rows"] += len(idx_less)
    k_m, v_m, _ = O.average_merge(k, v, idx_c, idx_less, assign)
    k_ref = O.round_to_storage(k_m, wl.dtype); v_ref = O.round_to_storage(v_m, wl.dtype)
    tol = KV_TOL[wl.dtype]
    dk = np.abs(k_gpu - k_ref).max() if k_ref.size else 0.0
    dv = np.abs(v_gpu - v_ref).max() if v_ref.size else 0.0
    assert dk <= tol and dv <= tol, f"layer {l} head {g}: merged K/V off by {dk:.3e}/{dv:.3e}"
    stats["max_kv_err"] = max(stats["max_kv_err"], dk, dv)
    stats["kv_elems_not_bit_exact"] += int((k_gpu != k_ref).sum() + (v_gpu != v_ref).sum())


def _unit(x):
    return x / np.maximum(np.linalg.norm(x, axis=1, keepdims=True), 1e-30)


def check_all(wl, data, gpu, heads=None, score_layers=None, verbose=True, threads=1):
    """Full comparison.  ``heads``: iterable of (layer, head) to check downstream of the scores (all by default),
    or a function of the validated budgets S returning them.
    ``score_layers``: layers whose scores/entropies are compared (all by default; budgets need all)."""
    L, Hkv = wl.n_layers, wl.n_kv_heads
    stats = {"heads": 0, "rows": 0, "ambiguous_rows": 0, "sets_differing_in_tie_band": 0,
             "max_kv_err": 0.0, "kv_elems_not_bit_exact": 0, "layers_passing_only_by_entropy_floor": 0}
    a_s, ent = oracle_scores(wl, data, score_layers, threads)
    k = data["k"]
    for l in a_s:
        ref = a_s[l]
        err = np.abs(gpu["col_scores"][l] - ref) / np.maximum(np.abs(ref), 1e-6)
        assert err.max() <= 1e-4, f"layer {l}: column scores off by {err.max():.3e} relative"
        norms = np.linalg.norm(to_float64(k[l]), axis=-1)
        np.testing.assert_allclose(gpu["inv_norm"][l], 1.0 / np.maximum(norms, 1e-30), rtol=2e-6)
        e_ref = ent[l][2]
        # 1e-3 relative; the floor covers entropies of almost one-hot rows, which lie below the resolution of fp32
        # probabilities (1 - 2^-24): their absolute error of order 1e-8 moves no budget (S_l ~ exp(E))
        assert abs(gpu["entropy"][l] - e_ref) <= 1e-3 * abs(e_ref) + 1e-7, \
            f"layer {l}: entropy {gpu['entropy'][l]} vs {e_ref}"
        if abs(gpu["entropy"][l] - e_ref) > 1e-3 * abs(e_ref):
            stats["layers_passing_only_by_entropy_floor"] += 1
    stats["max_entropy_rel_err"] = max(abs(gpu["entropy"][l] - ent[l][2]) / max(abs(ent[l][2]), 1e-30) for l in ent)
    if len(ent) == L:
        (S, M, N, off), strict = check_budgets(wl, gpu, ent)
        stats["budgets_strictly_equal"] = strict
        # how close every layer is to being rounded the other way, against the entropy error actually observed
        e_vec = np.array([ent[l][2] for l in range(L)])
        margin, rel = budget_margins(wl, e_vec)
        err_rel = np.abs(gpu["entropy"] - e_vec) / np.maximum(np.abs(e_vec), 1e-30)
        stats["min_budget_margin_slots"] = float(margin.min())
        stats["min_rel_entropy_change_flipping_a_budget"] = float(rel.min())
        if verbose:
            print(f"[parity {wl.name}] budgets {S.tolist()}", flush=True)
            print(f"[parity {wl.name}] margin to the nearest rounding boundary, slots per layer: "
                  + " ".join("inf" if not np.isfinite(m) else f"{m:.3f}" for m in margin), flush=True)
            print(f"[parity {wl.name}] relative entropy change that would flip a budget: min {rel.min():.2e}; "
                  f"observed relative entropy error: max {err_rel.max():.2e}", flush=True)
    else:
        # Only some layers were scored by the oracle (very large workloads): the budgets cannot be derived
        # from oracle entropies alone.  What can be checked: the entropies of the sampled layers (above),
        # the invariants of the allocation, and that the budgets are exactly what the oracle's allocator
        # returns for the GPU's entropy vector.
        S, M, N, off = O.allocate_budgets(gpu["entropy"], wl.total_budget, wl.seq_len, wl.window,
                                          wl.recent_num, wl.recent_den)
        assert np.array_equal(gpu["S"], S) and int(gpu["S"].sum()) == wl.total_budget
        assert np.array_equal(gpu["alloc"][:, 1], M) and np.array_equal(gpu["alloc"][:, 2], N)
        assert np.array_equal(np.diff(gpu["off"]), gpu["S"])
        stats["budgets_strictly_equal"] = None
    if callable(heads):
        heads = heads(S)
    pairs = [(l, g) for l in range(L) for g in range(Hkv)] if heads is None else list(heads)
    for l, g in pairs:
        check_head(wl, data, gpu, a_s[l], l, g, int(N[l]), int(M[l]), stats)
    if verbose:
        print(f"[parity {wl.name}] " + ", ".join(f"{k}={v}" for k, v in stats.items()), flush=True)
    return stats


def decode_error(got, ref, vmax, bf16):
    """Checks one decoding step against the oracle and returns max |got - ref| / vmax.

    The kernel multiplies exactly, sums d and S_l terms in fp32 and rounds the result once to the storage type.  The
    fp32 part stays below 1e-6 of vmax (the largest |v| of the layer: the output is a convex combination of value
    rows).  The rounding to bf16 (8 significant bits, round to nearest) moves a value x by up to half an ulp,
    2^(floor(log2 |x|) - 8): a bound per element, which a single figure relative to vmax cannot replace (2^-9 vmax is
    exceeded by an output just above a power of two close to vmax, 2^-8 vmax is loose everywhere else).
    """
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    tol = np.full(ref.shape, 1e-6 * vmax)
    if bf16:
        a = np.maximum(np.abs(ref), 2.0 ** -126)
        tol = tol + 2.0 ** (np.floor(np.log2(a)) - 8)
    diff = np.abs(got - ref)
    bad = diff > tol
    assert not bad.any(), (int(bad.sum()), float((diff - tol).max()), float(diff.max() / vmax))
    return float(diff.max() / vmax)
