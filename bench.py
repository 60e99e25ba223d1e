#!/usr/bin/env python3
"""Throughput of the whole compression pass on one MI355X.

One step = one meda_compress call: every phase of the pass over all layers and heads of one synthetic
sequence whose inputs are already resident in HBM.  Prints one JSON line with the whole-job throughput
(context tokens compressed per second) of the headline workload (the largest configuration, ``extreme``,
unless --workload names another), the roofline figures of its dominant kernel (HIP-event time of that kernel
measured inside the timed region), short runs of the other configurations (``per_workload``), the rates the
chip delivers to a plain read stream and to back-to-back matrix instructions (``measured_peak``), and the CPU
oracle timed on the host cores (``cpu_baseline``).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
HEADLINE = "extreme"
# kernels a phase launches (score_accum: one of the three, by the shape: grouped heads take the _dma form, the
# full-prompt mode the _blocks form; similarity: the packing kernel, then the tiled and the resident-set kernel)
PHASE_KERNELS = {"score_stats": ["score_stats_kernel"], "stats_combine": ["stats_combine_kernel"],
                 "score_accum": ["score_accum_kernel | score_accum_dma_kernel | score_accum_blocks_kernel"],
                 "allocate": ["allocate_kernel"], "select": ["select_kernel"],
                 "similarity": ["pack_conserved_kernel", "similarity_argmax_kernel", "similarity_resident_kernel"],
                 "segment_sort": ["segment_sort_kernel"], "merge_write": ["merge_write_kernel"]}
PHASE_BOUND = {"score_stats": "hbm", "score_accum": "hbm", "similarity": "mfma", "merge_write": "hbm",
               "select": "hbm", "segment_sort": "hbm", "stats_combine": "hbm", "allocate": "hbm"}


def algorithmic_work(wl, budgets, full_prompt=False):
    """Per launch: bytes the method itself must move (hbm phases) or flops it must do (similarity; the
    scoring when every prompt row scores: the logits of the causal triangle once)."""
    L, Hkv, T, d = wl.n_layers, wl.n_kv_heads, wl.seq_len, wl.head_dim
    e = 2 if wl.dtype == "bf16" else 4
    k_bytes = L * Hkv * T * d * e
    out_rows = int(sum(budgets)) * Hkv
    less = [(T - s) * Hkv for s in budgets]
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


def time_pass(pkg, torch, wl, dev, steps, warmup, flags=0, n_seqs=0, phase_events=True, keep=False):
    """Generates the workload, uploads it and times ``steps`` passes.  Returns the record fields of this
    workload and, with ``keep``, the device tensors and the output object (for the decoding-step measurement)."""
    from workloads import generate, generate_batch, variant
    full_prompt = bool(flags & pkg.FLAG_FULL_PROMPT)
    if n_seqs:
        data = generate_batch([variant(wl, seed=wl.seed + i) for i in range(n_seqs)], threads=16)
    else:
        data = generate(wl, threads=16)
    q, k, v, mask = (data[n].to(dev) for n in ("q", "k", "v", "mask"))
    del data
    params = pkg.make_params(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.seq_len, wl.window,
                             wl.total_budget, q.dtype, wl.recent_num, wl.recent_den, 0.0, flags, n_seqs)
    comp = pkg.Compressor(params, dev, want_entropy=True, want_sel_idx=True, want_merge_assign=False)
    stream = torch.cuda.current_stream(dev)

    names = [pkg.meda_phase_name(i) for i in range(pkg.N_PHASES)]
    phase_kernels = dict(PHASE_KERNELS)
    phase_bound = dict(PHASE_BOUND)
    if full_prompt:            # the three scoring kernels are timed as one phase
        phase_bound["score_stats"] = "mfma"
        phase_kernels["score_stats"] = ["score_stats_kernel", "stats_combine_kernel", "score_accum_kernel"]
    # warm-up with every kernel bracketed by events: gives the per-phase times and names the dominant kernel
    comp(q, k, v, mask, stream)            # first call loads the code objects: not part of any figure
    torch.cuda.synchronize()
    pkg.meda_profile_enable(True)
    pkg.meda_profile_read(reset=True)
    for _ in range(max(warmup, 1)):
        comp(q, k, v, mask, stream)
    torch.cuda.synchronize()
    warm_ms, warm_calls = pkg.meda_profile_read(reset=True)
    per_phase = {n: warm_ms[i] / warm_calls for i, n in enumerate(names)}
    dom = max(names, key=lambda n: per_phase[n])
    # timed region: only the dominant kernel is bracketed (two events per call), on the stream it is launched on;
    # one more event per step on the same stream gives the per-step times whose median is reported as well
    pkg.meda_profile_enable(phase_events, names.index(dom))
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_ev[0].record(stream)
    for i in range(steps):
        out = comp(q, k, v, mask, stream)
        step_ev[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    phase_ms, n_calls = pkg.meda_profile_read(reset=True)
    pkg.meda_profile_enable(False)
    dom_ms = phase_ms[names.index(dom)] / n_calls if n_calls else None
    step_ms = [step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(steps)]

    ms_per_step = (t1 - t0) * 1e3 / steps
    seqs = max(n_seqs, 1)
    budgets = out.layer_len.cpu().reshape(seqs, wl.n_layers).tolist()
    work = {}
    for b in budgets:          # the sequences of a batch are independent: their work adds up
        for key, val in algorithmic_work(wl, b, full_prompt).items():
            work[key] = work.get(key, 0) + val

    roofline = None
    if dom_ms:
        bound = phase_bound[dom]
        t_s = dom_ms * 1e-3
        if bound == "mfma":
            achieved, peak, unit = work[dom] / t_s / 1e12, MFMA_PEAK_TFLOPS[wl.dtype], "TFLOP/s"
        else:
            achieved, peak, unit = work[dom] / t_s / 1e9, HBM_PEAK_GBS, "GB/s"
        roofline = {"kernel": dom, "launches": phase_kernels[dom], "bound": bound, "achieved": achieved,
                    "peak": peak, "unit": unit, "frac": achieved / peak,
                    # HBM bytes per launch are not measured by this program: the counter runs are separate
                    # rocprofv3 runs; the figure is read from their committed summary (null if there is none)
                    "traffic": None if full_prompt or seqs > 1 else counted_traffic(wl.name, dom),
                    "traffic_unit": "bytes (fetch + write, scaled by the copy calibration)",
                    "traffic_source": f"profiles/hbm_counters_{wl.name}.md (rocprofv3 --pmc runs)",
                    "work_per_launch": work[dom], "work_unit": "flop" if bound == "mfma" else "bytes",
                    "kernel_ms": dom_ms, "launches_timed": n_calls}

    alg_bytes = work["merge_write"]        # K and V once + the output: the traffic of the whole pass
    score_flop = 2.0 * seqs * wl.n_layers * wl.n_q_heads * wl.window * wl.seq_len * wl.head_dim
    rec = {
        "value": seqs * wl.seq_len / (ms_per_step * 1e-3), "ms_per_step": ms_per_step,
        "ms_per_step_event_median": statistics.median(step_ms),
        "config": {"workload": wl.name + ("+full_prompt_scoring" if full_prompt else ""), "layers": wl.n_layers,
                   "q_heads": wl.n_q_heads, "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim,
                   "seq_len": wl.seq_len, "window": wl.window, "total_budget": wl.total_budget, "seed": wl.seed,
                   "batch": seqs},
        "dtype": wl.dtype,
        "kv_rows_per_sec": seqs * wl.n_layers * wl.n_kv_heads * wl.seq_len / (ms_per_step * 1e-3),
        "pass_hbm_frac": (alg_bytes / (ms_per_step * 1e-3)) / (HBM_PEAK_GBS * 1e9),
        "pass_mfma_frac": ((work["similarity"] + score_flop) / (ms_per_step * 1e-3)) / (MFMA_PEAK_TFLOPS[wl.dtype] * 1e12),
        "phase_ms_warmup": per_phase,
        # every phase against its own bound, from the warm-up times (every kernel bracketed by events, which adds a
        # little to the short ones): algorithmic bytes or flops of a launch / time / published peak
        "phase_frac_warmup": {n: {"bound": phase_bound[n], "frac": (work[n] / (per_phase[n] * 1e-3))
                                  / (MFMA_PEAK_TFLOPS[wl.dtype] * 1e12 if phase_bound[n] == "mfma" else HBM_PEAK_GBS * 1e9)}
                              for n in names if work.get(n) and per_phase[n] > 0},
        "roofline": roofline,
    }
    kept = (q, k, v, out, budgets[0]) if keep else None
    return rec, kept


def counted_traffic(workload, phase):
    """HBM bytes per launch of one phase (fetched + written) from the summary of the rocprofv3 counter runs of this
    workload under profiles/, or None if that summary or the phase's row is missing."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"hbm_counters_{workload}.md")
    try:
        with open(path) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) == 4 and cells[0] == phase:
                    return float(cells[3])
    except (OSError, ValueError):
        pass
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


def measured_peaks(pkg, torch, dev):
    """What this chip delivers to the simplest kernels: a read stream over 2 GiB and back-to-back bf16 matrix
    instructions from registers (median of 5 launches each, after one untimed launch)."""
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    buf = torch.empty(2 << 30, dtype=torch.uint8, device=dev).fill_(1)

    def median_ms(fn, n=5):
        fn()
        torch.cuda.synchronize()
        times = []
        for _ in range(n):
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        return statistics.median(times)

    ms_read = median_ms(lambda: pkg.meda_peak_stream_read(buf, sink))
    total = [0]

    def mfma(random_operands):
        def run():
            total[0] = pkg.meda_peak_mfma_bf16(1 << 17, sink, random_operands)
        return run
    ms_mfma = median_ms(mfma(False))
    ms_mfma_rnd = median_ms(mfma(True))
    del buf
    # vector work beside the matrix instructions: nanoseconds per round of 16 matrix instructions and 16 V
    # multiply-adds per wave, written between the matrix instructions or as a phase after them
    rounds = 20000
    beside = {}
    for waves in (1, 2):
        for inter in (True, False):
            for v in (0, 4, 6, 8):
                if v == 0 and not inter:
                    continue
                ms = median_ms(lambda: pkg.meda_peak_mfma_valu(rounds, v, inter, waves, sink), n=3)
                beside[f"{waves}w_{'interleaved' if inter else 'phased'}_V{v}"] = round(ms * 1e6 / rounds, 1)
    return {"hbm_read_GBps": (2 << 30) / (ms_read * 1e-3) / 1e9,
            "mfma_with_valu_ns_per_round": beside,
            "bf16_mfma_TFLOPs": total[0] * 32768.0 / (ms_mfma * 1e-3) / 1e12,
            # the same instruction stream on operands whose bits toggle: the power-limited rate real data allows
            "bf16_mfma_random_operands_TFLOPs": total[0] * 32768.0 / (ms_mfma_rnd * 1e-3) / 1e12,
            "published": {"hbm_GBps": HBM_PEAK_GBS, "bf16_mfma_TFLOPs": MFMA_PEAK_TFLOPS["bf16"]},
            "how": "meda_peak_stream_read over 2 GiB; meda_peak_mfma_bf16, 131072 32x32x16 instructions per wave, "
                   "2 waves per SIMD, nearly constant and pseudo-random operands; median of 5 launches; "
                   "meda_peak_mfma_valu, 20000 rounds of 16 matrix instructions + 16 V multiply-adds per wave, "
                   "1 or 2 waves per SIMD, median of 3 launches"}


def _cpu_info():
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    return model, int(threads)


def cpu_baseline(wl, budgets, seconds_target=20.0):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload.

    Small workloads (the whole pass fits the time box): the oracle's whole pass on the first n layers, budget
    scaled to n layers, scaled by L/n.  Large workloads: the scoring of one layer and the selection / matching /
    merging of heads of the layer with the smallest and of the layer with the largest budget (the two ends of
    the per-head cost, which grows with the similarity flops 2 (T - S) S d); the pass is extrapolated as
    L * t_score + Hkv * sum_l (a + b * flops_l) with a, b from those two measurements.  The layer budgets S_l of
    the sampled layers are this run's (timing only: no parity statement rests on this number)."""
    import numpy as np
    from oracle import meda_oracle as O
    from workloads import generate, variant
    from workloads.gen import to_float64
    model, threads = _cpu_info()
    base = {"unit": "tokens/s", "cores": threads, "host_cpus": os.cpu_count(), "cpu_model": model, "kind": "oracle"}
    L, Hkv, T, d, W = wl.n_layers, wl.n_kv_heads, wl.seq_len, wl.head_dim, wl.window

    def whole(n_layers):
        sub = variant(wl, n_layers=n_layers, total_budget=(wl.total_budget * n_layers) // L)
        data = generate(sub, threads=min(8, n_layers))
        q, k, v = to_float64(data["q"]), to_float64(data["k"]), to_float64(data["v"])
        t0 = time.perf_counter()
        O.meda_compress(q, k, v, data["mask"].numpy(), sub.total_budget, sub.window, sub.dtype,
                        recent_num=sub.recent_num, recent_den=sub.recent_den)
        return time.perf_counter() - t0

    flops = [2.0 * (T - s) * s * d for s in budgets]            # per head
    if sum(flops) * Hkv < 2e11:                                  # small: time whole layers
        t1 = whole(1)
        n = int(max(1, min(L, seconds_target // max(t1, 1e-3))))
        t = whole(n) if n > 1 else t1
        per_pass = t * L / n
        return {**base, "value": T / per_pass,
                "sample": f"first {n} of {L} layers (all heads, budget scaled to {n} layers), {t:.1f} s, "
                          f"scaled by {L}/{n}"}

    l_lo, l_hi = int(np.argmin(budgets)), int(np.argmax(budgets))
    mask = generate(variant(wl, n_layers=1), layers=[0])["mask"].numpy()

    def sample_layer(l, score, max_heads, box):
        data = generate(wl, layers=[l], threads=1)
        q, k, v = to_float64(data["q"][0]), to_float64(data["k"][0]), to_float64(data["v"][0])
        t_score = None
        t0 = time.perf_counter()
        a_s, _ = O.layer_scores_and_entropy(q, k, mask)
        if score:
            t_score = time.perf_counter() - t0
        s = int(budgets[l])
        m = max(min(W, s), (s * wl.recent_num) // wl.recent_den)
        heads, t_heads = 0, 0.0
        while heads < max_heads and (heads == 0 or t_heads * (heads + 1) / heads < box):
            t0 = time.perf_counter()
            O.compress_layer_head(k[heads], v[heads], a_s[heads], mask, s - m, m, wl.dtype)
            t_heads += time.perf_counter() - t0
            heads += 1
        return t_score, t_heads / heads, heads

    t_score, t_lo, h_lo = sample_layer(l_lo, True, Hkv, 0.25 * seconds_target)
    _, t_hi, h_hi = sample_layer(l_hi, False, Hkv, 0.5 * seconds_target)
    if flops[l_hi] > flops[l_lo]:
        b = (t_hi - t_lo) / (flops[l_hi] - flops[l_lo])
        a = t_lo - b * flops[l_lo]
    else:
        a, b = 0.0, t_hi / max(flops[l_hi], 1.0)
    per_pass = L * t_score + Hkv * sum(a + b * f for f in flops)
    return {**base, "value": T / per_pass, "extrapolated": True,
            "sample": f"scoring of layer {l_lo} ({t_score:.1f} s, all heads); selection, matching and merging of "
                      f"{h_lo} head(s) of layer {l_lo} (S={budgets[l_lo]}, {t_lo:.2f} s/head) and {h_hi} head(s) of "
                      f"layer {l_hi} (S={budgets[l_hi]}, {t_hi:.2f} s/head); pass = {L} x scoring + {Hkv} heads x "
                      f"sum over layers of a + b x 2(T-S)S d flops, a, b from the two layers: {per_pass:.0f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-workload", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--no-peaks", action="store_true", help="skip the read-stream and matrix-instruction micro-kernels")
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
    from workloads import get_workload
    from workloads.configs import ORDER

    wl = get_workload(args.workload)
    flags = 0
    if args.full_prompt:       # every prompt position scores the keys
        from workloads import variant
        wl = variant(wl, score_rows=wl.seq_len)
        flags = pkg.FLAG_FULL_PROMPT
    dev = torch.device("cuda:0")
    n_seqs = max(args.batch, 0)
    plain = not (args.full_prompt or n_seqs)

    head, kept = time_pass(pkg, torch, wl, dev, args.steps, args.warmup, flags, n_seqs,
                           phase_events=not args.no_phase_events, keep=True)
    q, k, v, out, budgets = kept
    rec = {
        "metric": "kv_tokens_compressed_per_sec", "value": head["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"],
        "data": "synthetic",
    }
    rec.update({key: val for key, val in head.items() if key not in rec})
    rec["layer_budgets"] = budgets
    if not args.no_decode and not n_seqs:
        rec["decode_step"] = decode_step_record(pkg, torch, wl, out, q.dtype, k, v, dev)
    del q, k, v, out, kept
    torch.cuda.empty_cache()
    if plain and not args.no_per_workload:
        # short runs of the other configurations (parity-test cases; context for the headline)
        others = []
        for name in ORDER:
            if name == wl.name:
                continue
            o, _ = time_pass(pkg, torch, get_workload(name), dev, steps=10, warmup=2)
            torch.cuda.empty_cache()
            others.append({"workload": name, "ms_per_step": o["ms_per_step"],
                           "ms_per_step_event_median": o["ms_per_step_event_median"], "tokens_per_s": o["value"],
                           "dtype": o["dtype"], "pass_hbm_frac": o["pass_hbm_frac"], "pass_mfma_frac": o["pass_mfma_frac"],
                           "dominant_kernel": o["roofline"]["kernel"], "dominant_bound": o["roofline"]["bound"],
                           "dominant_kernel_ms": o["roofline"]["kernel_ms"], "dominant_frac": o["roofline"]["frac"],
                           "phase_ms_warmup": o["phase_ms_warmup"],
                           "phase_frac_warmup": {n: round(v["frac"], 4) for n, v in o["phase_frac_warmup"].items()}})
        rec["per_workload"] = others
    if not args.no_peaks:
        rec["measured_peak"] = measured_peaks(pkg, torch, dev)
    if not args.no_cpu_baseline and not n_seqs:
        rec["cpu_baseline"] = cpu_baseline(wl, budgets)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
