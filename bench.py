#!/usr/bin/env python3
"""Benchmark of the EFCP / Sparse M-FAC step on one MI355X.

One "step" is one efcp_step call: error feedback, exact Top-k, ring insertion
with its Gram row, the SP pass, the m x m coefficient solve and the LCG pass,
on a gradient already resident in HBM.  The workload is the BERT-base-sized
configuration (d = 110,000,000, m = 1024, k = 1,100,000, lambda = 1e-6) with a
FULL 1024-row window: the window is filled with 1024 untimed steps first.

Prints one JSON line:
  value / ms_per_step   steps per second and milliseconds per step: wall clock over exactly --steps steps
  step_ms               median / min / max / mean of individual step times: max(--steps, 50) further steps
                        right after the timed region, one HIP event before each on the steps' stream
                        (the event itself costs a few microseconds per step, so these run slightly
                        above ms_per_step)
  kernel_ms             from 20 more steps with the library's HIP events around every kernel group
  step_bytes            algorithmic bytes of one step, 16*n*k + 24*d + 8*k (n rows filled): the method's
                        format, an int32 index and an fp32 value per window entry
  achieved_GBps, hbm_frac   step_bytes / median step time, and that over the 8 TB/s HBM peak
  stored_step_bytes, stored_GBps, hbm_frac_stored   the same with the bytes the library really keeps per
                        entry (a 16-bit in-slice index next to the value): what HBM has to deliver
  roofline              the slower of the two window passes (k_sp, k_lcg): algorithmic bytes per
                        launch / HIP-event time per launch, against the HBM peak (`achieved`, `frac`);
                        achieved_stored / frac_stored: the same with the stored entry size, i.e. the
                        bytes HBM really has to deliver; `traffic`: HBM bytes per launch that rocprofv3's
                        FETCH_SIZE / WRITE_SIZE counted in the committed profile named by
                        `traffic_source` (read from that file at run time; null when the file has no
                        figure for this kernel and configuration)
  device_copy_GBps      a plain torch device copy of d floats on the same box (bytes read + written / time):
                        what a simple streaming kernel reaches here, for context
  cpu_baseline          the CPU oracle timed on this host at the full d: one measured step from the empty
                        state, the measured cost of one more window row, the coefficient recursion alone;
                        `value` = the full-window step put together from them (`sample` says how)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch that rocprofv3 counted (FETCH_SIZE / WRITE_SIZE scaled by a torch kernel of
# known size) for the full 1024-row window of the bert_base workload are kept in this summary, on
# lines of the form "traffic_bytes_per_launch <kernel> <bytes>".
TRAFFIC_PROFILE = "profiles/k_sp_k_lcg_k_ef_hist_bert_base_hbm_counters.txt"
MIN_TIMED_STEPS = 50            # individual step times are collected over at least this many steps
METRIC = "Sparse M-FAC EFCP steps/s + achieved HBM GB/s (d=110M, m=1024, 1% density)"


def step_bytes(d, k, n, entry=8, mode="grad"):
    """Bytes of one step with n filled rows at `entry` bytes per window entry.
    Algorithmic bytes use the entry of the method's own format: 8 (int32 index +
    fp32 value; 16*n*k + 24*d + 8*k for the benchmark's step) or 6 (int32 + bf16);
    stored bytes use what the library keeps in HBM: 6 (16-bit in-slice index +
    fp32) or 4 (+ bf16).
    mode: "grad" (x = g, F^-1 g written: the benchmark's definition), "compressed"
    (x = c_t: no dense x is read), "update" / "compressed-update" (the parameters
    are read and written instead of F^-1 x being written)."""
    x_read = 0 if mode.startswith("compressed") else 4 * d
    dst = 8 * d if mode.endswith("update") else 4 * d
    by = {
        "ef": 12 * d + entry * k,              # read g, read e, write e; write the new row
        "sp": entry * n * k + x_read,          # window once + x
        "lcg": entry * n * k + x_read + dst,   # window once + x + out (or theta in and out)
    }
    by["total"] = by["ef"] + by["sp"] + by["lcg"]
    return by


def measured_traffic(kernel, path=None):
    """Bytes per launch of `kernel` ("k_sp", "k_lcg", ...) recorded in the committed counter
    summary, or None if the file or the line is not there."""
    path = path or os.path.join(ROOT, TRAFFIC_PROFILE)
    try:
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "traffic_bytes_per_launch" and w[1] == kernel:
                    return float(w[2])
    except (OSError, ValueError):
        pass
    return None


def step_time_stats(ms):
    """median / min / max / mean of a list of per-step milliseconds."""
    v = sorted(ms)
    n = len(v)
    med = v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])
    return {"median": med, "min": v[0], "max": v[-1], "mean": sum(v) / n, "n": n}


def cpu_baseline(wl, bf16=False, rows=32):
    """The oracle as it stands (one thread) on this host, every piece timed at the workload's
    full d, bounded to about half a minute:
      T1    one full step from the empty state: error feedback, the sort of d pairs, one row
      r     what one more window row costs a step: its share of the Gram row (the time of loading
            a row into a window of `rows` rows, per row) and of q and the LCG sum (apply() on
            `rows` rows minus apply() on one row, per row)
      c     the O(m^3) coefficient recursion on an m x m Gram matrix, timed alone
    The step with the full m-row window, which is what `value` stands for, is T1 + (m-1)*r + c:
    every cost of a step is linear in the number of rows except the recursion."""
    import numpy as np
    import oracle
    from paper_2306_06098_amd import synth
    oracle.build()
    rows = max(1, min(rows, wl.m))
    s = synth.GradientStream(wl.d, wl.rho, wl.seed)
    g = s.next()
    del s
    o = oracle.Oracle(wl.d, wl.m, wl.k, wl.lam, values_bf16=bf16)
    t0 = time.perf_counter()
    o.step(g)
    t_first = time.perf_counter() - t0

    def t_apply():
        best = float("inf")
        for _ in range(2):
            t0 = time.perf_counter()
            o.apply(g)
            best = min(best, time.perf_counter() - t0)
        return best
    a1 = t_apply()
    rng = np.random.default_rng(1234)
    t_load = 0.0
    for _ in range(rows - 1):
        row = synth.random_sparse_row(wl.d, wl.k, rng)
        t0 = time.perf_counter()
        o.load_row(*row)
        t_load = time.perf_counter() - t0          # the last one: Gram products with `rows` rows
    an = t_apply() if rows > 1 else a1
    o.close()
    del o, g
    gram_row = t_load / rows
    ql_row = max(an - a1, 0.0) / max(rows - 1, 1)
    B = rng.standard_normal((wl.m, 48))
    S = B @ B.T + np.eye(wl.m)
    t0 = time.perf_counter()
    oracle.coefficients(S, rng.standard_normal(wl.m), wl.m, wl.lam)
    t_coef = time.perf_counter() - t0
    t_full = t_first + (wl.m - 1) * (gram_row + ql_row) + t_coef
    return {
        "value": 1.0 / t_full, "unit": "steps/s", "cores": 1, "host_cores": os.cpu_count(), "kind": "oracle",
        "seconds_per_step_full_window": t_full,
        "seconds_per_step_first_step_measured": t_first,
        "seconds_per_window_row": gram_row + ql_row,
        "seconds_coefficient_recursion": t_coef,
        "sample": (f"all at the full d={wl.d:,}, k={wl.k:,}: one oracle step from the empty state {t_first:.2f} s "
                   f"(measured); one more window row costs {gram_row + ql_row:.4f} s (Gram row: loading a row into a "
                   f"window of {rows} rows, per row {gram_row:.4f} s; q and LCG: apply() on {rows} rows minus apply() "
                   f"on 1 row, per row {ql_row:.4f} s); the O(m^3) coefficient recursion for m={wl.m}, alone, "
                   f"{t_coef:.3f} s. value = 1 / ({t_first:.2f} + {wl.m - 1} * {gram_row + ql_row:.4f} + {t_coef:.3f}) "
                   f"= 1 / {t_full:.1f} s: the step with the full {wl.m}-row window. One thread of {os.cpu_count()} "
                   "host cores."),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="bert_base")
    ap.add_argument("--fill", type=int, default=-1, help="untimed steps before warm-up (default m)")
    ap.add_argument("--values", choices=["fp32", "bf16"], default="fp32",
                    help="window format: fp32 = the benchmark's definition (8-byte entries); "
                         "bf16 = bfloat16 values + 16-bit in-slice indices (4-byte entries)")
    ap.add_argument("--mode", choices=["grad", "compressed", "update", "compressed-update"], default="grad",
                    help="grad = the benchmark's definition (F^-1 g written); compressed: x = c_t; "
                         "update: parameters updated in place by the LCG kernel")
    ap.add_argument("--topk", choices=["global", "block"], default="global",
                    help="global = exact global Top-k (the benchmark's definition); block = Top-k applied "
                         "in blocks of 16,384 coordinates, ceil(16384*k/d) entries per block")
    ap.add_argument("--precond", choices=["mfac", "ggt"], default="mfac",
                    help="mfac = Sparse M-FAC (the benchmark's definition); ggt = Sparse GGT on the same "
                         "window with m = 100 and epsilon = 1e-3 (the paper runs it at the resnet20 size)")
    ap.add_argument("--launch", choices=["eager", "graph"], default="eager",
                    help="eager: every step is an efcp_step call (its kernel launches); graph: one step per "
                         "resident gradient buffer is captured into a HIP graph once (no kernel argument of a "
                         "step depends on the step number) and the timed steps are replays of those graphs")
    ap.add_argument("--single-stream", action="store_true",
                    help="efcp_options.single_stream: with --topk block, the eviction update on the step's own "
                         "stream, no second queue (for counter collection with rocprofv3 --pmc); the global "
                         "Top-k never uses a second stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives exist); use --gpus 1")

    import torch
    from paper_2306_06098_amd import binding, synth

    wl = synth.WORKLOADS[args.workload]
    ggt = args.precond == "ggt"
    if ggt:
        import dataclasses
        wl = dataclasses.replace(wl, m=min(wl.m, 100), lam=1e-3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bf16 = args.values == "bf16"
    if args.topk == "block":
        kb = -(-binding.TOPK_BLOCK * wl.k // wl.d)
        ctx = binding.Efcp(wl.d, wl.m, kb, wl.lam, values=binding.VALUES_BF16 if bf16 else binding.VALUES_FP32,
                           topk_block=binding.TOPK_BLOCK, ggt=ggt, single_stream=args.single_stream)
    else:
        ctx = binding.Efcp(wl.d, wl.m, wl.k, wl.lam,
                           values=binding.VALUES_BF16 if bf16 else binding.VALUES_FP32, ggt=ggt,
                           single_stream=args.single_stream)
    k_row = ctx.k
    stream = synth.TorchGradientStream(wl.d, wl.rho, wl.seed, dev)
    out = torch.empty(wl.d, dtype=torch.float32, device=dev)
    pool = [torch.empty(wl.d, dtype=torch.float32, device=dev) for _ in range(4)]

    fill = wl.m if args.fill < 0 else args.fill
    t_fill = time.perf_counter()
    xsrc = binding.X_COMPRESSED if args.mode.startswith("compressed") else binding.X_GRAD
    if args.mode.endswith("update"):
        out.normal_(0.0, 0.02)               # stands for the parameters
        # lr small enough that 50 updates of synthetic gradients keep the parameters finite
        dest = dict(param=out, lr=1e-12, weight_decay=0.01)
    else:
        dest = dict(out=out)

    for i in range(fill + args.warmup):
        g = pool[i % len(pool)]
        stream.next_into(g)
        # filling the window needs no output: skip the LCG pass until the warm-up steps
        if i >= fill:
            ctx.step_ex(g, xsrc, **dest)
        else:
            ctx.step(g, None)
        if (i + 1) % 256 == 0:
            torch.cuda.synchronize()
            print(f"[bench] filled {i + 1} steps, {time.perf_counter() - t_fill:.1f} s",
                  file=sys.stderr, flush=True)
    for g in pool:                       # timed steps cycle over resident gradients
        stream.next_into(g)
    torch.cuda.synchronize()

    def eager_step(i):
        if args.mode == "grad":
            ctx.step(pool[i % len(pool)], out)
        else:
            ctx.step_ex(pool[i % len(pool)], xsrc, **dest)

    one_step = eager_step
    if args.launch == "graph":
        # one graph per resident gradient buffer; capturing records the launches and runs nothing
        graphs = []
        cap_stream = torch.cuda.Stream()
        torch.cuda.synchronize()
        for j in range(len(pool)):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=cap_stream):
                if args.mode == "grad":
                    ctx.step(pool[j], out, stream=cap_stream)
                else:
                    ctx.step_ex(pool[j], xsrc, stream=cap_stream, **dest)
            graphs.append(gr)
        torch.cuda.synchronize()

        def one_step(i):
            graphs[i % len(graphs)].replay()
        for i in range(args.warmup):
            one_step(i)
        torch.cuda.synchronize()

    # (1) The timed region: exactly --steps steps between two synchronisations, nothing else on
    # the stream (an event record between kernels costs several microseconds of its own).
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # (2) Individual step times: max(--steps, MIN_TIMED_STEPS) further steps with one HIP event
    # before each (on torch's current stream, which is the stream the steps run on).
    n_events = max(args.steps, MIN_TIMED_STEPS)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_events + 1)]
    for i in range(n_events):
        marks[i].record()
        one_step(i)
    marks[n_events].record()
    torch.cuda.synchronize()
    per_step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(n_events)]
    stats = step_time_stats(per_step_ms)
    # (3) Time per kernel group: 20 more eager steps with the library's own events around each group.
    ctx.profile_enable(True)
    for i in range(20):
        eager_step(i)
    torch.cuda.synchronize()
    ms_groups, covered = ctx.profile_read()
    ctx.profile_enable(False)
    sm = ctx.get_small()                 # raises if the library flagged a numeric problem
    assert torch.isfinite(out).all().item()

    n = min(sm["step"], wl.m)
    by = step_bytes(wl.d, k_row, n, 6 if bf16 else 8, args.mode)          # algorithmic
    st = step_bytes(wl.d, k_row, n, 4 if bf16 else 6, args.mode)          # as stored
    ms_step = (t1 - t0) * 1e3 / args.steps
    ms_med = stats["median"]
    per_launch = {kname: ms_groups[kname] / max(covered, 1) for kname in ms_groups}
    dom = "lcg" if per_launch["lcg"] >= per_launch["sp"] else "sp"
    achieved = by[dom] / (per_launch[dom] * 1e-3) / 1e9
    achieved_stored = st[dom] / (per_launch[dom] * 1e-3) / 1e9
    headline = n == wl.m and not bf16 and args.mode == "grad" and args.topk == "global" and not ggt \
        and wl.name == "bert_base"
    traffic = measured_traffic("k_" + dom) if headline else None
    result = {
        "metric": METRIC, "value": 1e3 / ms_step, "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": None, "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: d={wl.d} m={wl.m} k={k_row} lambda={wl.lam} "
                               f"window rows filled={n}", "fill_steps": fill,
                   "window_format": ("bf16 value" if bf16 else "fp32 value") + " + 16-bit in-slice index "
                                    "(int32 indices at the interface)",
                   "mode": args.mode, "topk": args.topk,
                   "preconditioner": args.precond, "launch": args.launch,
                   "single_stream": bool(args.single_stream)},
        "step_ms": stats,
        "step_bytes": by["total"],
        "achieved_GBps": by["total"] / (ms_med * 1e-3) / 1e9,
        "hbm_frac": by["total"] / (ms_med * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "stored_step_bytes": st["total"],
        "stored_GBps": st["total"] / (ms_med * 1e-3) / 1e9,
        "hbm_frac_stored": st["total"] / (ms_med * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kernel_ms": per_launch,
        "roofline": {"bound": "hbm", "kernel": "k_" + dom, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": TRAFFIC_PROFILE if traffic is not None else None,
                     "bytes_per_launch": by[dom], "ms_per_launch": per_launch[dom],
                     "stored_bytes_per_launch": st[dom], "achieved_stored": achieved_stored,
                     "frac_stored": achieved_stored / HBM_PEAK_GBPS,
                     "note": "achieved/frac count a window entry at the 8 bytes of the method's own format "
                             "(int32 index + fp32 value), as the benchmark defines its bytes; the library keeps "
                             "6 (4 with bf16 values), so achieved_stored/frac_stored is what HBM really delivers"},
    }
    ctx.destroy()
    # practical ceiling of this machine for context: a plain device copy of d floats (read d, write d)
    src = pool[0]
    for _ in range(3):
        out.copy_(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(20):
        out.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    result["device_copy_GBps"] = 20 * 8 * wl.d / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del pool, out, stream, src
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline and not ggt:
        result["cpu_baseline"] = cpu_baseline(wl, bf16)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
