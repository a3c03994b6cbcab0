#!/usr/bin/env python3
"""Benchmark of the sparse-FFN hot path on one MI355X.

One step = one pass of the whole hot path (predict -> update_window -> load_bundles ->
sparse_ffn for every token) over the workload's token stream, starting from an empty
neuron cache.  Inputs, weights and the pinned bundle store are resident before the timed
region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--ffn-mode skip|full]
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

HBM_PEAK_GBS = 8000.0          # MI355X datasheet HBM3E bandwidth


def describe(w):
    return (f"{w.name}: d_model={w.d_model} d_ffn={w.d_ffn} rank={w.rank} k={w.window_k} "
            f"p_active={w.p_active} rho={w.rho} {w.dtype} {'gated' if w.glu else 'relu'} "
            f"batch={w.batch} tokens={w.tokens} capacity_rows={w.capacity_rows}")


def cpu_baseline(w, L, X, budget_s=20.0):
    """The oracle, as it stands, on the host cores: whole path per token."""
    import numpy as np
    from oracle import lif_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu, L.A, L.B, L.c, L.theta,
                        L.b, L.bundles)
    t0 = time.perf_counter()
    done = 0
    for t in range(len(X)):
        ora.step(X[t])
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": dt / done * 1e6, "unit": "us/token/layer", "cores": int(cores), "kind": "oracle",
            "sample": f"first {done} tokens of the same stream, whole path (predict, window, delete, insert, FFN)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--ffn-mode", default="skip", choices=["skip", "full"],
                    help="skip: down columns read only for rows with a non-zero activation; full: whole bundles")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from the host instead of a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as wl
    import paper_2312_11514_amd as lif
    from tests.harness import GpuLayer

    w = wl.WORKLOADS[args.workload]
    if w.layers != 1:
        print("bench.py: multi-layer workloads are driven by the parity tests, not by the bench line", file=sys.stderr)
        sys.exit(2)
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w) if w.batch > 1 else wl.make_inputs(w)
    T = len(X)
    mode = {"skip": lif.FFN_SKIP_DEAD, "full": lif.FFN_FULL_BUNDLE}[args.ffn_mode]
    reads_all = args.ffn_mode == "full"
    gpu = GpuLayer(w, L, ffn_mode=mode)
    lay = gpu.layer
    xd = gpu.upload_x(X)                                   # [T, (batch,) d] resident in HBM
    yd = torch.zeros_like(xd)

    def run_stream():
        lay.reset()
        for t in range(T):
            lay.step(xd[t], yd[t], w.batch)

    # eager pass: validates the chain and provides counters for the byte accounting
    run_stream()
    torch.cuda.synchronize()
    st, cnt = lay.state(), lay.counters()
    assert st["error"] == 0, st
    rows_per_tok = cnt["ffn_rows"] / cnt["ffn_calls"]
    active_per_tok = cnt["ffn_active"] / cnt["ffn_calls"]
    added_per_tok = cnt["added"] / cnt["steps"]

    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run_stream()
    step = graph.replay if graph is not None else run_stream

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    us_per_token = ms_per_step * 1e3 / T / w.layers

    # FFN alone, on the cache state the stream ends in: R back-to-back lif_sparse_ffn calls in a HIP graph,
    # timed with HIP events on the launch stream; the byte count comes from the device counters of those calls
    R = 200
    ffn = None
    if not args.no_profile:
        c0 = lay.counters()
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2):
            for _ in range(R):
                lay.sparse_ffn(xd[T - 1], yd[T - 1], w.batch)
        g2.replay()
        torch.cuda.synchronize()
        c0 = lay.counters()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 5
        e0.record()
        for _ in range(reps):
            g2.replay()
        e1.record()
        torch.cuda.synchronize()
        c1 = lay.counters()
        calls = c1["ffn_calls"] - c0["ffn_calls"]
        assert calls == R * reps
        rows = (c1["ffn_rows"] - c0["ffn_rows"]) / calls
        act = (c1["ffn_active"] - c0["ffn_active"]) / calls
        ffn = {"us": e0.elapsed_time(e1) * 1e3 / calls, "rows": rows, "active": act}

    # per-kernel durations over one more eager pass of the whole stream: HIP events recorded by the library
    # on the launch stream around every kernel (these include the event/dispatch overhead of ~2 us per launch)
    kern = {}
    if not args.no_profile:
        lay.profile_begin(7 * T + 8)
        run_stream()
        for k, (ms, n) in lay.profile_collect().items():
            if n:
                kern[k] = {"avg_us": ms / n * 1e3, "launches": n}

    E, d, G = w.elem_bytes, w.d_model, w.vectors_per_bundle
    nominal = rows_per_tok * G * d * E
    out = {
        "metric": "sparse-FFN us/token/layer (whole hot path: predict + window + load + FFN)",
        "value": us_per_token, "unit": "us/token/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": describe(w), "tokens_per_step": T, "ffn_mode": args.ffn_mode,
                   "launch": "eager" if graph is None else "hip-graph of the whole token stream",
                   "llc": "single layer: the cache working set stays warm in the 256 MB Infinity Cache"},
        "per_token": {"rows_in_cache": rows_per_tok, "rows_active": active_per_tok, "rows_added": added_per_tok,
                      "h2d_bytes": added_per_tok * w.bundle_bytes, "nominal_bundle_bytes": nominal},
    }
    if ffn:
        up_bytes = ffn["rows"] * (G - 1) * d * E
        down_bytes = (ffn["rows"] if reads_all else ffn["active"]) * d * E
        touched = up_bytes + down_bytes
        nominal_f = ffn["rows"] * G * d * E
        ach = touched / (ffn["us"] * 1e-6) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "ffn_up + ffn_down",
                           "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                           "traffic": None, "algorithmic_bytes_per_launch": touched, "avg_launch_us": ffn["us"],
                           "rows": ffn["rows"], "rows_active": ffn["active"],
                           "nominal_bundle_bytes": nominal_f,
                           "nominal_GBs": nominal_f / (ffn["us"] * 1e-6) / 1e9,
                           "nominal_frac": nominal_f / (ffn["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS}
    if kern:
        out["h2d"] = {"GBs_in_load_kernel": added_per_tok * w.bundle_bytes / (kern["load"]["avg_us"] * 1e-6) / 1e9}
        out["kernels_avg_us_event_timed"] = {k: round(v["avg_us"], 3) for k, v in kern.items()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, L, X)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
