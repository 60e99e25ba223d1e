#!/usr/bin/env python3
"""Throughput of the whole compression pass on one MI355X.

One step = one meda_compress call: every phase of the pass over all layers and heads of one synthetic
sequence whose inputs are already resident in HBM.  Prints one JSON line with the whole-job throughput
(context tokens compressed per second), the roofline figures of the dominant kernel (HIP-event time of
that kernel measured inside the timed region) and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
# kernels a phase launches (the similarity step is one launch of each of its two kernels: a layer goes to the
# resident-set kernel when its conserved keys fit into LDS, else to the tiled one)
PHASE_KERNELS = {"score_stats": ["score_stats_kernel"], "stats_combine": ["stats_combine_kernel"],
                 "score_accum": ["score_accum_kernel"], "allocate": ["allocate_kernel"], "select": ["select_kernel"],
                 "similarity": ["similarity_argmax_kernel", "similarity_resident_kernel"],
                 "segment_sort": ["segment_sort_kernel"], "merge_write": ["merge_write_kernel"]}
PHASE_BOUND = {"score_stats": "hbm", "score_accum": "hbm", "similarity": "mfma", "merge_write": "hbm",
               "select": "hbm", "segment_sort": "hbm", "stats_combine": "hbm", "allocate": "hbm"}


def algorithmic_work(wl, budgets):
    """Per launch: bytes the method itself must move (hbm phases) or flops it must do (similarity; the
    scoring when every prompt row scores: the logits of the causal triangle once)."""
    L, Hkv, T, d = wl.n_layers, wl.n_kv_heads, wl.seq_len, wl.head_dim
    e = 2 if wl.dtype == "bf16" else 4
    k_bytes = L * Hkv * T * d * e
    out_rows = int(sum(budgets)) * Hkv
    less = [(T - s) * Hkv for s in budgets]
    full_prompt = wl.n_score_rows == T and T != wl.window
    return {
        "score_stats": (1.0 * L * wl.n_q_heads * T * (T + 1) * d) if full_prompt else k_bytes,   # flops / every key once
        "score_accum": k_bytes,                                    # every key once
        "similarity": sum(2.0 * (T - s) * s * d * Hkv for s in budgets),   # flops
        "merge_write": 2 * k_bytes + 2 * out_rows * d * e,         # every K and V row once + the output
        "select": L * Hkv * T * 4,
        "segment_sort": sum(less) * 8,
        "stats_combine": 0,
        "allocate": 0,
    }


def measured_traffic(workload, kernel):
    """HBM bytes per launch of ``kernel`` from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE and WRITE_SIZE, already scaled by the plain-copy calibration), or None."""
    path = os.path.join(ROOT, "profiles", f"hbm_counters_{workload}.md")
    if not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == kernel:
            try:
                return float(cells[1]) + float(cells[2])
            except ValueError:
                return None
    return None


def decode_step_record(pkg, torch, wl, out, q_dtype, k, v, dev, iters=50):
    """The step that follows the compression pass (Section 3.1 of the paper: one decoding query per layer and
    head attends over the cache): its time over the compressed cache of this run and over the full cache,
    with the HBM rate on the bytes it has to read (every cached key and value once)."""
    L, Hq, Hkv, d, T = wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len
    e = 2 if wl.dtype == "bf16" else 4
    g = torch.Generator().manual_seed(wl.seed + 1)
    q = torch.randn(L, Hq, d, generator=g).to(q_dtype).to(dev)

    def timed(dec, *args):
        for _ in range(3):
            dec(*args)
        torch.cuda.synchronize()
        t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(iters):
            dec(*args)
        t1.record(); torch.cuda.synchronize()
        return t0.elapsed_time(t1) / iters

    dec = pkg.Decoder(pkg.make_decode_params(L, Hq, Hkv, d, wl.total_budget, q_dtype), dev)
    ms_c = timed(dec, q, out.k_out, out.v_out, out.layer_len, out.layer_off)
    # the uncompressed cache [L][Hkv][T][d] is the same layout with S_l = T
    full_len = torch.full((L,), T, dtype=torch.int32, device=dev)
    full_off = (torch.arange(L + 1, dtype=torch.int64) * T).to(dev)
    dec_f = pkg.Decoder(pkg.make_decode_params(L, Hq, Hkv, d, L * T, q_dtype), dev)
    ms_f = timed(dec_f, q, k.view(-1, d), v.view(-1, d), full_len, full_off)
    bytes_c = 2.0 * wl.total_budget * Hkv * d * e
    bytes_f = 2.0 * L * T * Hkv * d * e
    fp8 = {}
    if q_dtype == torch.bfloat16:   # the same step over the 8-bit storage of the compressed cache
        def quantise():
            return pkg.meda_quantize_fp8(out.k_out), pkg.meda_quantize_fp8(out.v_out)
        (kc, ks), (vc, vs) = quantise()
        ms_q = timed(lambda: quantise())
        ms_8 = timed(dec.fp8, q, kc, vc, ks, vs, out.layer_len, out.layer_off)
        bytes_8 = 2.0 * wl.total_budget * Hkv * (d + 4)      # codes and one scale per row
        fp8 = {"compressed_fp8_ms": ms_8, "compressed_fp8_GBps": bytes_8 / (ms_8 * 1e-3) / 1e9,
               "quantise_ms": ms_q,
               "quantise_GBps": (bytes_c + bytes_8) / (ms_q * 1e-3) / 1e9}   # reads the bf16 rows, writes the codes
    return {**fp8, "compressed_ms": ms_c, "compressed_GBps": bytes_c / (ms_c * 1e-3) / 1e9,
            "compressed_hbm_frac": bytes_c / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "full_cache_ms": ms_f, "full_cache_GBps": bytes_f / (ms_f * 1e-3) / 1e9,
            "full_cache_hbm_frac": bytes_f / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "speedup": ms_f / ms_c, "cache_bytes_ratio": bytes_c / bytes_f}


def cpu_baseline(wl, seconds_target=20.0):
    """The fp64 oracle on a bounded sample: the first n layers of the same workload with the budget
    scaled to n layers, n chosen from a one-layer probe so the run takes roughly ``seconds_target``."""
    import numpy as np
    from oracle import meda_oracle as O
    from workloads import generate, variant
    from workloads.gen import to_float64
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1

    def run(n_layers):
        sub = variant(wl, n_layers=n_layers, total_budget=(wl.total_budget * n_layers) // wl.n_layers)
        data = generate(sub, threads=min(8, n_layers))
        q, k, v = to_float64(data["q"]), to_float64(data["k"]), to_float64(data["v"])
        t0 = time.perf_counter()
        O.meda_compress(q, k, v, data["mask"].numpy(), sub.total_budget, sub.window, sub.dtype,
                        recent_num=sub.recent_num, recent_den=sub.recent_den)
        return time.perf_counter() - t0

    t1 = run(1)
    n = int(max(1, min(wl.n_layers, seconds_target // max(t1, 1e-3))))
    t = run(n) if n > 1 else t1
    per_pass = t * wl.n_layers / n
    return {"value": wl.seq_len / per_pass, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n} of {wl.n_layers} layers (all heads, budget scaled to {n} layers), "
                      f"{t:.1f} s, scaled by {wl.n_layers}/{n}"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llava7b_multi_image")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--full-prompt", action="store_true",
                    help="score with every prompt position instead of the observation window")
    ap.add_argument("--no-decode", action="store_true", help="skip the decoding-step measurement")
    ap.add_argument("--batch", type=int, default=0, metavar="N",
                    help="compress N sequences of the workload's shape (different seeds) per call; the "
                         "value is then the tokens of all N sequences per second")
    ap.add_argument("--no-phase-events", action="store_true",
                    help="do not record per-kernel HIP events inside the timed region")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="only run a plain device copy of BYTES bytes five times (reference for the "
                         "HBM byte counters of rocprofv3) and exit")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        src = torch.empty(args.copy_calibration, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": args.copy_calibration, "copies": 5}))
        return
    if args.gpus != 1:
        print("bench.py: this build is single-GPU only (one MI355X holds all layers and heads); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2502_17599_amd as pkg
    from workloads import generate, get_workload

    wl = get_workload(args.workload)
    flags = 0
    if args.full_prompt:       # every prompt position scores the keys (the three scoring kernels are timed as one)
        from workloads import variant
        wl = variant(wl, score_rows=wl.seq_len)
        flags = pkg.FLAG_FULL_PROMPT
        PHASE_BOUND["score_stats"] = "mfma"
        PHASE_KERNELS["score_stats"] = ["score_stats_kernel", "stats_combine_kernel", "score_accum_kernel"]
    dev = torch.device("cuda:0")
    n_seqs = max(args.batch, 0)
    if n_seqs:
        from workloads import generate_batch, variant
        data = generate_batch([variant(wl, seed=wl.seed + i) for i in range(n_seqs)], threads=16)
    else:
        data = generate(wl, threads=16)
    q, k, v, mask = (data[n].to(dev) for n in ("q", "k", "v", "mask"))
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, q.dtype, wl.recent_num, wl.recent_den, 0.0, flags, n_seqs)
    comp = pkg.Compressor(params, dev, want_entropy=True, want_sel_idx=True, want_merge_assign=False)
    stream = torch.cuda.current_stream(dev)

    names = [pkg.meda_phase_name(i) for i in range(pkg.N_PHASES)]
    # warm-up with every kernel bracketed by events: gives the per-phase times and names the dominant kernel
    comp(q, k, v, mask, stream)            # first call loads the code objects: not part of any figure
    torch.cuda.synchronize()
    pkg.meda_profile_enable(True)
    pkg.meda_profile_read(reset=True)
    for _ in range(max(args.warmup, 1)):
        comp(q, k, v, mask, stream)
    torch.cuda.synchronize()
    warm_ms, warm_calls = pkg.meda_profile_read(reset=True)
    per_phase = {n: warm_ms[i] / warm_calls for i, n in enumerate(names)}
    dom = max(names, key=lambda n: per_phase[n])
    # timed region: only the dominant kernel is bracketed (two events per call), on the stream it is launched on
    events = not args.no_phase_events
    pkg.meda_profile_enable(events, names.index(dom))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = comp(q, k, v, mask, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    phase_ms, n_calls = pkg.meda_profile_read(reset=True)
    pkg.meda_profile_enable(False)
    dom_ms = phase_ms[names.index(dom)] / n_calls if n_calls else None

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    seqs = max(n_seqs, 1)
    budgets = out.layer_len.cpu().reshape(seqs, wl.n_layers).tolist()
    work = {}
    for b in budgets:          # the sequences of a batch are independent: their work adds up
        for key, val in algorithmic_work(wl, b).items():
            work[key] = work.get(key, 0) + val

    roofline = None
    if dom_ms:
        bound = PHASE_BOUND[dom]
        t_s = dom_ms * 1e-3
        if bound == "mfma":
            achieved, peak, unit = work[dom] / t_s / 1e12, MFMA_PEAK_TFLOPS[wl.dtype], "TFLOP/s"
        else:
            achieved, peak, unit = work[dom] / t_s / 1e9, HBM_PEAK_GBS, "GB/s"
        roofline = {"kernel": dom, "launches": PHASE_KERNELS[dom], "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                    "frac": achieved / peak,
                    "traffic": None if (args.full_prompt or n_seqs) else measured_traffic(wl.name, dom),
                    "kernel_ms": dom_ms, "launches_timed": n_calls}

    e = 2 if wl.dtype == "bf16" else 4
    alg_bytes = work["merge_write"]        # K and V once + the output: the traffic of the whole pass
    rec = {
        "metric": "kv_tokens_compressed_per_sec", "value": seqs * wl.seq_len / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name + ("+full_prompt_scoring" if args.full_prompt else ""), "layers": wl.n_layers, "q_heads": wl.n_q_heads, "kv_heads": wl.n_kv_heads,
                   "head_dim": wl.head_dim, "seq_len": wl.seq_len, "window": wl.window,
                   "total_budget": wl.total_budget, "seed": wl.seed, "batch": seqs},
        "kv_rows_per_sec": seqs * wl.n_layers * wl.n_kv_heads * wl.seq_len / (ms_per_step * 1e-3),
        "pass_hbm_frac": (alg_bytes / (ms_per_step * 1e-3)) / (HBM_PEAK_GBS * 1e9),
        "pass_mfma_frac": ((work["similarity"] + 2.0 * seqs * wl.n_layers * wl.n_q_heads * wl.window * wl.seq_len * wl.head_dim)
                           / (ms_per_step * 1e-3)) / (MFMA_PEAK_TFLOPS[wl.dtype] * 1e12),
        "phase_ms_warmup": per_phase,
        "roofline": roofline,
    }
    if not args.no_decode and not n_seqs:
        rec["decode_step"] = decode_step_record(pkg, torch, wl, out, q.dtype, k, v, dev)
    if not args.no_cpu_baseline and not n_seqs:
        rec["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
