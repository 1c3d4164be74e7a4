#!/usr/bin/env python3
"""Benchmark of the LookupFFN forward pass (hash + gather) on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM: lookupffn_forward = hash kernel + gather kernel.  The default
workload is the RoBERTa-base-shaped layer the headline metric is quoted on (config 2:
16384 tokens, d = 768 padded to 1024, 3 hash rounds, k = 96 tables, tau = 8, fp32).
The learned tables are prepared once before the timed region (lookupffn_prepare_tables:
model-load work, like any weight pre-packing; --no-prepare times the row-major tables).

Prints ONE JSON line: tokens/s of the whole pass; `roofline` = the dominant (gather) kernel
against the resource that binds it (LDS reads for the staged kernel, else compulsory HBM
bytes), with HIP-event kernel times from inside the timed region (mean, min, median);
`hbm_compulsory` and `hbm_effective_x_peak` beside it; the CPU oracle's throughput on this
host (all threads and one thread); and `parity_checked`: how many tokens of the timed y
were compared with the oracle after the timed region.
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5, 6, 7, 8],
                    help="benchmark configuration (2 = the headline RoBERTa-base-shaped layer; 5 = the "
                         "8-token, 12-layer latency chain: a step is one pass through all 12 layers; 6-8 = the "
                         "paper's own layer shapes at its 32768-token batch)")
    ap.add_argument("--weighted", action="store_true",
                    help="time the weighted variant (lookupffn_forward_weighted: the hash also emits one fp32 "
                         "weight per token and table, the gather multiplies each row by it) instead of the plain sum")
    ap.add_argument("--probes", action="store_true",
                    help="time the multi-probe lookup (lookupffn_forward_probes: 1 + tau rows per token and table, "
                         "weighted by their soft-max shares)")
    ap.add_argument("--hash", choices=["sign-diagonal", "bh4"], default="sign-diagonal",
                    help="hash of the pass: the sign-diagonal x Hadamard rounds of the headline metric, or the "
                         "paper's BH4 (four block-diagonal x Hadamard factors, lookupffn_forward_bh)")
    ap.add_argument("--block", type=int, default=64, choices=[16, 32, 64], help="block size of the BH4 factors")
    ap.add_argument("--gather-path", type=int, default=0, choices=[0, 1, 2],
                    help="tuning: 1 = always the direct gather kernel, 2 = the LDS-staged one whenever the shape allows")
    ap.add_argument("--slice-lanes", type=int, default=0, choices=[0, 4, 8],
                    help="tuning: column-slice width of the staged gather in 16-byte lanes (0 = library default)")
    ap.add_argument("--token-slots", type=int, default=0, choices=[0, 4, 8, 13, 16],
                    help="tuning: most token slots per lane of the staged gather (0 = library default)")
    ap.add_argument("--zipf", type=float, default=0.0,
                    help="also time lookupffn_gather alone on codes with Zipf(s)-skewed buckets (reported beside, "
                         "never instead of, the hashed codes of the rotated Gaussian input)")
    ap.add_argument("--no-prepare", action="store_true",
                    help="pass the row-major tables / BH factors instead of their one-time prepared copies")
    ap.add_argument("--y-dtype", choices=["f32", "bf16", "f16"], default="f32",
                    help="storage type of y (the sums are fp32 either way; 16-bit y is rounded once when stored)")
    ap.add_argument("--layer-loop", action="store_true",
                    help="config 5: time the loop of per-layer lookupffn_forward calls instead of the single launch")
    ap.add_argument("--latency-passes", choices=["both", "warm", "cold"], default="both",
                    help="config 5: which passes the latency report times (one kind only: for counter runs, so that "
                         "every dispatch after the timed steps is of that kind)")
    ap.add_argument("--parity-tokens", type=int, default=1024,
                    help="tokens of the timed y compared with the oracle after the timed region (0 = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle timing")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="after the timed region, also run 3 plain device-to-device copies of this many MiB "
                         "(a kernel of known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def traffic_from_profiles(w, weighted: bool = False):
    """(HBM bytes per gather launch, file) from a committed rocprofv3 --pmc summary, if there is one: a
    figure measured in an earlier run of the same command under the profiler, not in this run."""
    f = ROOT / "profiles" / f"gather_config{w.index}{'_weighted' if weighted else ''}_pmc_hbm_traffic.txt"
    if not f.exists():
        return None, None
    for line in f.read_text().splitlines():
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":", 1)[1].split()[0]), f"profiles/{f.name}"
    return None, None


def cpu_baseline(w, x, signs, tables, budget_s: float, weighted: bool = False, bh: bool = False,
                 probes: bool = False) -> dict:
    """The CPU oracle as it stands, on the same batch: on all host threads it gets, and on one thread."""
    import oracle  # only this leg of the bench (and the parity check) touches the oracle
    threads = oracle.max_threads()
    n = x.shape[0]
    sample = min(n, 16384)
    xs = x[:sample]
    run = ((oracle.bh_forward_weighted if weighted else oracle.bh_forward) if bh else oracle.forward_probes if probes
           else oracle.forward_weighted if weighted else oracle.forward)
    run(xs[:256], signs, tables)                       # page in
    reps, t_total = 0, 0.0
    while reps < 3 or (t_total < budget_s and reps < 1000):
        t0 = time.perf_counter()
        run(xs, signs, tables)
        t_total += time.perf_counter() - t0
        reps += 1
        if t_total > 3 * budget_s:
            break
    # one thread: a smaller sample of the same batch (about a quarter of the budget)
    one = min(sample, max(64, int(sample * reps / t_total / max(threads, 1) * budget_s / 4)))
    oracle.set_threads(1)
    try:
        t0 = time.perf_counter()
        run(xs[:one], signs, tables)
        t_one = time.perf_counter() - t0
    finally:
        oracle.set_threads(threads)
    return {"value": sample * reps / t_total, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample} tokens of the batch, {reps} passes, {t_total:.1f} s, "
                      f"gcc -O2 -fopenmp, {os.cpu_count()} logical CPUs visible",
            "single_thread": {"value": one / t_one, "unit": "tokens/s", "cores": 1,
                              "sample": f"first {one} tokens, one pass, {t_one:.1f} s"}}


def parity_check(w, x, signs, tables, y_dev, n_check: int, weighted: bool, bh: bool, probes: bool) -> dict:
    """Compares tokens of the y the timed steps wrote with the oracle: an odd stride over the whole batch
    plus its first and last tokens (untimed)."""
    import oracle
    n = x.shape[0]
    step = max(1, n // max(n_check, 1)) | 1
    idx = np.unique(np.concatenate([np.arange(0, n, step), np.arange(0, min(64, n)), np.arange(max(0, n - 64), n)]))
    y16 = hasattr(y_dev, "dtype") and str(y_dev.dtype) in ("torch.bfloat16", "torch.float16")
    got = y_dev[idx].float().cpu().numpy() if hasattr(y_dev, "cpu") else y_dev[idx]
    xs = x[idx]
    if bh:
        ref = (oracle.bh_forward_weighted if weighted else oracle.bh_forward)(xs, signs, tables)
    elif probes:
        ref = oracle.forward_probes(xs, signs, tables)
    elif weighted:
        ref = oracle.forward_weighted(xs, signs, tables)
    else:
        ref = oracle.forward(xs, signs, tables, acc64=True)
    r = ref.astype(np.float64)
    err = float(np.max(np.abs(got.astype(np.float64) - r)) / np.sqrt(np.mean(r ** 2)))
    tol = 1e-2 if w.table_dtype == "bf16" else 1e-4
    out = {"tokens": int(len(idx)), "max_abs_err_over_rms": err, "tolerance": tol, "ok": bool(err <= tol)}
    if y16:
        # y stored in 16 bits: the tolerance plus one rounding to y's type per element (twice half an ulp allowed)
        rel = 2.0 ** -8 if "bfloat16" in str(y_dev.dtype) else 2.0 ** -11
        out["ok"] = bool(np.all(np.abs(got.astype(np.float64) - r) <= rel * np.abs(r) + tol * np.sqrt(np.mean(r ** 2))))
        out["tolerance"] = f"{tol} of rms + {rel} relative per element (16-bit y)"
    if not (weighted or probes):
        seq = (oracle.bh_forward if bh else oracle.forward)(xs, signs, tables, acc64=False)
        if y16:
            narrow = oracle.float_to_bf16 if "bfloat16" in str(y_dev.dtype) else oracle.float_to_half
            bits = y_dev[idx].view(__import__("torch").int16).cpu().numpy().view(np.uint16)
            out["bit_equal_to_rounded_fp32_sequential_sum"] = bool(np.array_equal(bits, narrow(seq)))
        else:
            out["bit_equal_to_fp32_sequential_sum"] = bool(np.array_equal(got, seq))
    return out


def launches_per_step_layers(w, args):
    """Layers one launch of the timed kernel covers."""
    return w.n_layers if (w.n_layers > 1 and not args.layer_loop) else 1


def latency_report(w, args, xd, loop_step, stack_step, y_last):
    """Latency of the layer chain, microseconds per pass and per layer: the single launch
    (lookupffn_forward_stack), the loop of per-layer launches, and the loop replayed from a HIP graph; each
    warm (the same batch again: the rows it touches stay in the caches) and cold (a different batch of a
    rotation of 16 and a 1 GiB overwrite before every timed pass)."""
    import torch
    from paper_2403_07221_amd import synth

    flush = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    batches = [xd] + [torch.from_numpy(synth.make_x(synth.seed_for(w.index, 0, 5) + i, w.n_tokens, w.d, w.x_dtype)).cuda()
                      for i in range(1, 16)]
    x_run = torch.empty_like(xd)     # the launches (and the graph) read this buffer

    def timed(fn, cold, reps):
        total = []
        for i in range(reps):
            x_run.copy_(batches[i % 16] if cold else batches[0])
            if cold:
                flush.zero_()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            total.append(e0.elapsed_time(e1) * 1e3)
        total.sort()
        return total[len(total) // 2]

    saved = xd.clone()
    runs = {"single_launch": lambda: stack_step(x_run)}

    def loop_on_x_run():
        xd.copy_(x_run)          # the per-layer loop reads xd
        loop_step()
    runs["layer_loop"] = loop_on_x_run
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    loop_on_x_run()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            loop_on_x_run()
    runs["layer_loop_graph"] = graph.replay
    graph1 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph1, stream=side):
            stack_step(x_run)
    runs["single_launch_graph"] = graph1.replay
    rep = {"layers": w.n_layers, "unit": "us", "cold_means": "another batch of 16 and a 1 GiB overwrite before each timed pass"}
    for name, fn in runs.items():
        if args.latency_passes != "cold":     # (a cold-only run warms nothing up)
            for _ in range(3):
                fn()
        torch.cuda.synchronize()
        rep[name] = {}
        if args.latency_passes != "cold":
            warm = timed(fn, False, 21)
            rep[name].update({"warm_per_pass": warm, "warm_per_layer": warm / w.n_layers})
        if args.latency_passes != "warm":
            cold = timed(fn, True, 16)
            rep[name].update({"cold_per_pass": cold, "cold_per_layer": cold / w.n_layers})
    xd.copy_(saved)
    return rep


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the forward pass is token-parallel with replicated tables and "
              "needs no collective, so this build reports the single-GPU rate only (run with --gpus 1).",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2403_07221_amd import binding as B
    from paper_2403_07221_amd import cost, synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    B.lib()
    B.lookupffn_set_option("slice_lanes", args.slice_lanes)
    B.lookupffn_set_option("token_slots", args.token_slots)
    B.lookupffn_set_option("gather_path", args.gather_path)
    w = synth.CONFIGS[args.config]
    bh = args.hash == "bh4"
    if args.probes and args.weighted:
        print("--probes and --weighted are different variants: pick one", file=sys.stderr)
        sys.exit(2)
    if bh and (args.probes or w.n_layers > 1):
        print("--hash bh4 is timed with the plain-sum or the weighted gather on the single-layer configurations",
              file=sys.stderr)
        sys.exit(2)
    ws_bytes = (B.lookupffn_workspace_bytes_weighted if args.weighted else B.lookupffn_workspace_bytes)(w.n_tokens, w.k)
    if args.probes:
        ws_bytes = B.lookupffn_workspace_bytes_probes(w.n_tokens, w.k, w.tau)
    if bh:
        blk = args.block if args.no_prepare else (B.PREPARED | args.block)
        ws_bytes = (B.lookupffn_workspace_bytes_bh_weighted if args.weighted else B.lookupffn_workspace_bytes_bh)(
            w.n_tokens, w.d, w.k, w.tau, blk, 4)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    B.lookupffn_init()
    forward = ((B.lookupffn_forward_bh_weighted if args.weighted else B.lookupffn_forward_bh) if bh
               else B.lookupffn_forward_probes if args.probes
               else B.lookupffn_forward_weighted if args.weighted else B.lookupffn_forward)

    y_torch = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.y_dtype]
    if args.y_dtype != "f32" and w.n_layers > 1 and args.layer_loop:
        print("--layer-loop hands y from layer to layer in fp32: use --y-dtype f32 with it", file=sys.stderr)
        sys.exit(2)

    def prepared(td):
        return td if args.no_prepare else B.lookupffn_prepare_tables(td)

    if w.n_layers == 1:
        x, signs, tables = synth.make_layer(w)
        if bh:   # the block-diagonal factors take the place of the sign diagonals
            signs = synth.make_bmats(synth.seed_for(w.seed_index or w.index, 0, 3) + args.block, w.n_proj, 4,
                                     w.d_pad, args.block)
        xd, sd = B.to_device(x), torch.from_numpy(signs).cuda()
        td_rows = B.to_device(tables)
        td = prepared(td_rows)
        if bh and not args.no_prepare:
            sd = B.lookupffn_prepare_bh(sd, w.d, w.k, w.tau)
        y = torch.empty((w.n_tokens, w.d_out), dtype=y_torch, device="cuda")

        def step():
            forward(xd, sd, td, y=y, workspace=ws)
    else:
        # stacked layers, chained: layer l+1 hashes layer l's output (d_out == d)
        layers = [synth.make_layer(w, layer=l, with_x=(l == 0)) for l in range(w.n_layers)]
        x, signs, tables = layers[0]
        xd = B.to_device(x)
        dev = [(B.to_device(s_), prepared(B.to_device(t_))) for _, s_, t_ in layers]
        ys = [torch.empty((w.n_tokens, w.d_out), dtype=torch.float32, device="cuda") for _ in range(2)]

        y_last = torch.empty((w.n_tokens, w.d_out), dtype=y_torch, device="cuda")

        def loop_step():
            h = xd
            for l in range(w.n_layers):
                h = forward(h, dev[l][0], dev[l][1], y=ys[l & 1], workspace=ws)
            return h

        def stack_step(x_in=None):
            B.lookupffn_forward_stack(xd if x_in is None else x_in, [s_ for s_, _ in dev], [t_ for _, t_ in dev], y=y_last)

        # a step is one pass through all the layers: one launch (lookupffn_forward_stack) unless --layer-loop
        step = loop_step if args.layer_loop else stack_step
    launches_per_step = 1 if (w.n_layers > 1 and not args.layer_loop) else w.n_layers

    # untimed: the hash kernel's own duration (event pairs around it), outside the timed region so
    # that the timed steps carry only the one event pair the roofline entry needs
    step()                      # first launch: code-object load, workspace checks
    torch.cuda.synchronize()
    B.lookupffn_timing_reset()
    B.lookupffn_timing_enable(1)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    hash_ms, hash_n = B.lookupffn_timing_read(0)

    # timed region: K whole steps; the gather kernel (dominant) is bracketed by HIP events
    B.lookupffn_timing_reset()
    B.lookupffn_timing_enable(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gather_ms, gather_n = B.lookupffn_timing_read(1)
    gather_each = B.lookupffn_timing_read_each(1)
    B.lookupffn_timing_enable(0)
    B.lookupffn_timing_reset()
    kernel = B.lookupffn_last_gather_kernel()
    fused = kernel == "forward_stack_kernel"          # hash and gather in one kernel: no hash launch of its own
    assert gather_n == args.steps * launches_per_step and hash_n == (0 if fused else args.warmup * launches_per_step)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.n_tokens / (ms_per_step * 1e-3)

    xb = 2 if w.x_dtype == "bf16" else 4
    tb = 2 if w.table_dtype == "bf16" else 4
    yb = 4 if args.y_dtype == "f32" else 2
    path_bytes = cost.bytes_per_token(w.d, w.k, w.d_out, xb, tb) * w.n_tokens * w.n_layers
    n_probe = (w.tau + 1) if args.probes else 1
    side_floats = w.k * n_probe if (args.weighted or args.probes) else 0      # weights / shares per token
    # the gather kernel alone: k table rows (x probes) + the y row + the k uint16 codes (+ weights) it reads, per token
    gather_bytes = (w.k * n_probe * w.d_out * tb + w.d_out * yb + w.k * 2 + side_floats * 4) * w.n_tokens
    path_bytes += (w.k * (n_probe - 1) * w.d_out * tb + 2 * side_floats * 4) * w.n_tokens * w.n_layers
    gather_avg_ms = gather_ms / gather_n
    staged = kernel in ("gather_lds_kernel", "gather_ring_kernel")
    # compulsory HBM traffic of one gather launch: every table byte once (as the kernel reads it: the prepared
    # copy is fp32), codes (+ weights) once, y once
    read_tb = 4 if (staged or not args.no_prepare) else tb
    table_bytes_read = w.k * w.rows * w.d_out * read_tb
    compulsory = table_bytes_read + (w.k * 2 + side_floats * 4 + w.d_out * yb) * w.n_tokens
    if w.n_tokens * w.k < w.k * w.rows:          # fewer lookups than rows: only the rows touched
        compulsory = (w.k * n_probe * w.d_out * read_tb + w.k * 2 + side_floats * 4 + w.d_out * yb) * w.n_tokens
    if fused:                                    # one launch: x, the sign diagonals and the rows touched, per layer
        compulsory = ((w.k * w.d_out * read_tb + w.d * xb + w.d_out * yb) * w.n_tokens
                      + w.n_proj * w.n_rounds * w.d_pad) * launches_per_step_layers(w, args)
    each = sorted(gather_each)
    times = {"avg_kernel_ms": gather_avg_ms, "min_kernel_ms": each[0] if each else None,
             "median_kernel_ms": each[len(each) // 2] if each else None, "launches_timed": len(each)}
    traffic, traffic_file = traffic_from_profiles(w, args.weighted)
    # The staged kernel serves every (token, table[, probe]) row piece from LDS, so LDS read bandwidth is the
    # resource that binds it: 256 CUs x 256 bytes per clock (16-byte reads) x 2.4 GHz.  The direct kernel is
    # priced against HBM on the bytes that must cross it.
    lds_peak = 256 * 256 * 2.4  # GB/s
    lds_bytes = w.k * w.d_out * 4 * w.n_tokens * n_probe
    if staged:
        rate = lds_bytes / (gather_avg_ms * 1e-3) / 1e9
        roofline = {"kernel": kernel, "bound": "lds", "achieved": rate, "peak": lds_peak, "unit": "GB/s",
                    "frac": rate / lds_peak, "bytes_per_launch": lds_bytes,
                    "bytes_definition": "k * d_out * 4 * n_tokens (* (1 + tau) probes): every selected row piece is read from LDS once"}
    else:
        rate = compulsory / (gather_avg_ms * 1e-3) / 1e9
        roofline = {"kernel": kernel, "bound": "hbm", "achieved": rate, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": rate / HBM_PEAK_GBS, "bytes_per_launch": compulsory,
                    "bytes_definition": "compulsory HBM bytes: tables (or the rows touched) + codes (+ weights) + y, once each"}
    roofline.update(times)
    roofline["traffic"] = traffic
    roofline["traffic_source"] = (f"{traffic_file}: rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE of an earlier profiled run of "
                                  "this command, not measured in this run") if traffic_file else None
    roofline["algorithmic_bytes_per_launch"] = gather_bytes

    out = {
        "metric": "tokens/sec and achieved GB/s vs HBM peak for LookupFFN forward at d=768",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if tb == 4 else "bf16-storage/f32-accumulate",
        "data": "synthetic",
        "config": {"workload": w.name, "n_tokens": w.n_tokens, "d": w.d, "d_pad": w.d_pad,
                   "hash_rounds": w.n_rounds, "k_tables": w.k, "tau": w.tau, "d_out": w.d_out,
                   "x_dtype": w.x_dtype, "table_dtype": w.table_dtype, "y_dtype": args.y_dtype,
                   "table_bytes": w.k * w.rows * w.d_out * tb,
                   "tables_prepared_once": not args.no_prepare,
                   "variant": "weighted" if args.weighted else "multi-probe" if args.probes else "plain-sum",
                   "hash": f"bh4-block{args.block}" if bh else "sign-diagonal"},
        "roofline": roofline,
        # the same kernel time against the bytes that must cross HBM at least once
        "hbm_compulsory": {"bytes_per_launch": compulsory, "achieved": compulsory / (gather_avg_ms * 1e-3) / 1e9,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": compulsory / (gather_avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        # algorithmic bytes (one HBM row read per token and table, as if nothing were re-used) / kernel time /
        # 8 TB/s: a ratio, not a fraction -- above 1 it measures the re-use the kernel extracts on chip
        "hbm_effective_x_peak": gather_bytes / (gather_avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernels_ms": {"hash": None if fused else hash_ms / max(hash_n, 1), "gather": gather_avg_ms},
        "whole_path": {"algorithmic_bytes_per_step": path_bytes,
                       "effective_GBps": path_bytes / (ms_per_step * 1e-3) / 1e9,
                       "compulsory_hbm_bytes_per_step": (compulsory + w.d * xb * w.n_tokens) * w.n_layers,
                       "frac_of_hbm_peak_on_compulsory_bytes":
                           (compulsory + w.d * xb * w.n_tokens) * w.n_layers / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if staged:
        # measured with a stand-alone read loop (16 waves per CU, 16-byte reads, row offsets in registers):
        # contiguous 147.7 TB/s; 8 lanes per random 128-byte row 82.8 TB/s; 4 lanes per random 64-byte row 68.5 TB/s
        wide = w.tau <= 8 if args.slice_lanes == 0 else args.slice_lanes == 8
        ceiling = 82800.0 if wide else 68500.0
        roofline["random_row_ceiling"] = ceiling
        roofline["frac_of_random_row_ceiling"] = roofline["achieved"] / ceiling
    if bh:
        # the block-diagonal products are the path's one dense contraction: priced against the fp32
        # matrix-core peak (flops of the products only; the transform and the code extraction ride along).
        # The time is the hash step's event pair: the operand re-ordering kernel plus the hash kernel.
        flops = w.n_proj * 4 * 2 * w.d_pad * args.block * w.n_tokens
        hash_s = hash_ms / max(hash_n, 1) * 1e-3
        out["hash_roofline"] = {"kernel": "bh_pack_kernel + bh_hash_kernel", "bound": "mfma", "achieved": flops / hash_s / 1e12,
                                "peak": 157.3, "unit": "TFLOP/s", "frac": flops / hash_s / 1e12 / 157.3,
                                "flops_per_launch": flops, "avg_kernel_ms": hash_s * 1e3}
    elif not fused and hash_n:
        # the sign-diagonal hash is bound by vector-ALU issue: the butterflies alone are d_pad * log2(d_pad)
        # fp32 adds per round, projection and token, against one 64-lane add per SIMD every four clocks
        # (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T adds/s: packed fp32 is not used and an add is
        # not a fused multiply-add, so this is a quarter of the 157.3 TFLOP/s vector figure).  The time is
        # the hash step's event pair, which includes a few microseconds of launch and queue time.
        adds = w.n_proj * w.n_rounds * w.d_pad * (w.d_pad.bit_length() - 1) * w.n_tokens
        hash_s = hash_ms / hash_n * 1e-3
        alu_peak = 256 * 4 * 16 * 2.4e9 / 1e12
        out["hash_roofline"] = {"kernel": B.lookupffn_last_hash_kernel(), "bound": "alu", "achieved": adds / hash_s / 1e12,
                                "peak": alu_peak, "unit": "T fp32 adds/s", "frac": adds / hash_s / 1e12 / alu_peak,
                                "adds_per_launch": adds, "avg_kernel_ms": hash_s * 1e3}
    if w.n_layers > 1:
        out["latency"] = latency_report(w, args, xd, loop_step, stack_step, y_last)
    if args.zipf > 0 and w.n_layers == 1:
        def time_gather(codes_np):
            cd = torch.from_numpy(codes_np.view(np.int16)).cuda()
            yz = torch.empty((w.n_tokens, w.d_out), dtype=torch.float32, device="cuda")
            for _ in range(5):
                B.lookupffn_gather(cd, td, y=yz, workspace=ws)
            torch.cuda.synchronize()
            B.lookupffn_timing_reset()
            B.lookupffn_timing_enable(2)
            for _ in range(args.steps):
                B.lookupffn_gather(cd, td, y=yz, workspace=ws)
            torch.cuda.synchronize()
            ms, cnt = B.lookupffn_timing_read(1)
            B.lookupffn_timing_enable(0)
            B.lookupffn_timing_reset()
            return ms / cnt
        uni = np.random.default_rng(1).integers(0, w.rows, size=(w.n_tokens, w.k), dtype=np.uint16)
        zc = synth.make_zipf_codes(synth.seed_for(w.seed_index or w.index, 0, 4), w.n_tokens, w.k, w.tau, args.zipf)
        out["skewed_gather"] = {"zipf_s": args.zipf, "kernel": None, "uniform_codes_avg_kernel_ms": time_gather(uni),
                                "zipf_codes_avg_kernel_ms": time_gather(zc)}
        out["skewed_gather"]["kernel"] = B.lookupffn_last_gather_kernel()
    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes_each_way"] = src.numel() * 4
    if args.parity_tokens > 0:
        # the y the timed steps wrote (for the chain: the first layer's, recomputed into a buffer of its own)
        if w.n_layers == 1:
            step()
            torch.cuda.synchronize()
            y_check = y
        else:
            y_check = forward(xd, dev[0][0], dev[0][1], workspace=ws)
            torch.cuda.synchronize()
        pc = parity_check(w, x, signs, tables, y_check, args.parity_tokens, args.weighted, bh, args.probes)
        if w.n_layers > 1:
            # the whole chain: the timed step's final y against the oracle's fp32 sequential chain, bit for bit
            import oracle
            step()
            torch.cuda.synchronize()
            y_end = y_last if not args.layer_loop else ys[(w.n_layers - 1) & 1]
            h = x
            for _, s_, t_ in layers:
                h = oracle.forward(h, s_, t_, acc64=False)
            if args.y_dtype == "f32":
                got = y_end.cpu().numpy()
            else:   # the last layer's output rounded once
                got = y_end.view(torch.int16).cpu().numpy().view(np.uint16)
                h = (oracle.float_to_bf16 if args.y_dtype == "bf16" else oracle.float_to_half)(h)
            pc["chain_layers"] = w.n_layers
            pc["chain_bits_equal"] = bool(np.array_equal(got, h))
            pc["ok"] = bool(pc["ok"] and pc["chain_bits_equal"])
        out["parity_checked"] = pc["tokens"]
        out["parity"] = pc
        if not pc["ok"]:
            print(json.dumps(out))
            print("bench.py: the timed output does not match the oracle", file=sys.stderr)
            sys.exit(1)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x, signs, tables, args.cpu_seconds, args.weighted, bh, args.probes)
        if w.n_layers > 1:
            out["cpu_baseline"]["sample"] += "; one layer (the first) of the chain"
    print(json.dumps(out))


if __name__ == "__main__":
    main()
