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
    ap.add_argument("--ffn-mode", default="skip", choices=["skip", "full"])
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
    mode = lif.FFN_SKIP_DEAD if args.ffn_mode == "skip" else lif.FFN_FULL_BUNDLE
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

    # per-kernel durations: HIP events recorded by the library on the launch stream, around every
    # kernel of one more pass over the same stream
    kern = {}
    if not args.no_profile:
        lay.profile_begin(7 * T + 8)
        run_stream()
        for k, (ms, n) in lay.profile_collect().items():
            kern[k] = {"avg_us": ms / max(n, 1) * 1e3, "launches": n}

    E, d, G = w.elem_bytes, w.d_model, w.vectors_per_bundle
    bytes_up = rows_per_tok * (G - 1) * d * E               # ffn_up reads the up (and gate) vector of every cached row
    bytes_down = (active_per_tok if args.ffn_mode == "skip" else rows_per_tok) * d * E
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
    if kern:
        up_us, down_us = kern["ffn_up"]["avg_us"], kern["ffn_down"]["avg_us"]
        ach = bytes_up / (up_us * 1e-6) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "ffn_up", "achieved": ach, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None,
                           "algorithmic_bytes_per_launch": bytes_up, "avg_launch_us": up_us}
        ffn_us = up_us + down_us
        out["ffn"] = {"us_per_token": ffn_us,
                      "nominal_bundle_GBs": nominal / (ffn_us * 1e-6) / 1e9,
                      "nominal_frac_of_hbm_peak": nominal / (ffn_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                      "touched_GBs": (bytes_up + bytes_down) / (ffn_us * 1e-6) / 1e9}
        out["h2d"] = {"GBs_in_load_kernel": added_per_tok * w.bundle_bytes / (kern["load"]["avg_us"] * 1e-6) / 1e9}
        out["kernels_avg_us"] = {k: round(v["avg_us"], 3) for k, v in kern.items()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, L, X)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
