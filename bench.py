#!/usr/bin/env python3
"""Benchmark of the sparse-FFN hot path on one MI355X.

One step = one pass of the whole hot path (predict -> update_window -> load_bundles ->
sparse_ffn for every token and every layer) over the workload's token stream, starting from
empty neuron caches.  Inputs, weights and the pinned bundle store are resident before the
timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2|C3|C4|C4b8|C5|N1|N2] [--ffn-mode skip|full]
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
            f"batch={w.batch} tokens={w.tokens} layers={w.layers} capacity_rows={w.capacity_rows}")


def cpu_baseline(w, L, X, budget_s=20.0):
    """The oracle, as it stands, on the host cores: whole path per token, one layer."""
    from oracle import lif_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    gate = w.gate_resident
    ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu and not gate, L.A, L.B, L.c,
                        L.theta, L.b, L.bundles, shrink=w.shrink, w_gate=L.w_gate if gate else None)
    t0 = time.perf_counter()
    done = 0
    for t in range(len(X)):
        if w.spec_keep > 0:
            ora.step_tokens(X[t], w.spec_keep)
        else:
            ora.step(X[t])
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    out = {"value": dt / done * 1e6, "unit": "us/token/layer", "cores": int(cores), "kind": "oracle",
           "sample": f"first {done} steps of the same stream on layer 0, whole path "
                     f"(predict, window, delete, insert, FFN)"}
    # the same oracle on one core, on a shorter sample
    try:
        from threadpoolctl import threadpool_limits
        ora1 = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu and not gate, L.A, L.B, L.c,
                             L.theta, L.b, L.bundles, shrink=w.shrink, w_gate=L.w_gate if gate else None)
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            done1 = 0
            for t in range(len(X)):
                if w.spec_keep > 0:
                    ora1.step_tokens(X[t], w.spec_keep)
                else:
                    ora1.step(X[t])
                done1 += 1
                if time.perf_counter() - t0 > budget_s / 4:
                    break
            out["one_core"] = {"value": (time.perf_counter() - t0) / done1 * 1e6, "unit": "us/token/layer",
                               "sample": f"first {done1} steps"}
    except ImportError:
        pass
    # untimed: how good the synthetic predictor is on a few tokens (the oracle's mask against the sign of the
    # true pre-activation) - describes the workload, not the kernels
    import numpy as np
    xs = X[:8].reshape(-1, X.shape[-1])[:8]
    w_act = L.w_gate if L.w_gate is not None else L.w_up
    hit = pred = true = 0
    for x in xs:
        m = np.asarray(ora.predict(x)).reshape(-1)
        tm = O.true_mask(w_act, L.b, x)
        hit += int((m & tm).sum()); pred += int(m.sum()); true += int(tm.sum())
    out["predictor_recall"] = hit / max(true, 1)
    out["predictor_precision"] = hit / max(pred, 1)
    return out


def pmc_traffic(pmc_dir):
    """HBM-side bytes per lif_sparse_ffn call from two rocprofv3 --pmc runs of this script (FETCH_SIZE, WRITE_SIZE),
    each scaled by what the same counter reported for the 256 MiB device copy of --pmc-copy.  Expects
    <pmc_dir>/pmc_FETCH_SIZE/*_counter_collection.csv and <pmc_dir>/pmc_WRITE_SIZE/*_counter_collection.csv."""
    import csv
    import glob
    out = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        files = glob.glob(os.path.join(pmc_dir, f"pmc_{counter}", "*counter_collection.csv"))
        if not files:
            return None
        rows = [r for r in csv.DictReader(open(files[0])) if r["Counter_Name"] == counter]
        copies = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]]
        if not copies or max(copies) <= 0:
            return None
        scale = 262144.0 / max(copies)                       # reported KiB -> true KiB (the copy moves 256 MiB each way)
        up = [(int(r["Dispatch_Id"]), float(r["Counter_Value"])) for r in rows if "k_ffn_up" in r["Kernel_Name"]]
        if not up:
            return None
        lo, hi = min(i for i, _ in up), max(i for i, _ in up)  # the FFN-only phase (lif_step never launches k_ffn_up alone)
        ffn = [float(r["Counter_Value"]) for r in rows
               if lo <= int(r["Dispatch_Id"]) <= hi and "k_ffn_" in r["Kernel_Name"]]
        out[counter] = {"scale": scale, "bytes_per_call": sum(ffn) * scale * 1024.0 / len(up)}
    return out


def sweep_window(args):
    """Memory-latency trade-off over the window size k (the synthetic analogue of the paper's Fig. 4a / Fig. 7):
    larger windows hold more rows in the cache and load fewer bytes per token."""
    import torch
    import workloads as wl
    from workloads.device import GpuLayer
    base_w = wl.WORKLOADS[args.workload]
    L = wl.make_layer(base_w)
    X = wl.make_inputs(base_w)
    T = len(X)
    rows = []
    for k in (1, 2, 3, 4, 5, 6, 8, 12, 16):
        w = wl.scaled(base_w, window_k=k, capacity_rows=base_w.d_ffn)
        gpu = GpuLayer(w, L)
        lay = gpu.layer
        xd = gpu.upload_x(X)
        yd = torch.zeros_like(xd)

        def run():
            lay.reset()
            for t in range(T):
                lay.step(xd[t], yd[t])
        run()
        torch.cuda.synchronize()
        cnt = lay.counters()
        lay.set_expected_rows(int(0.9 * cnt["ffn_rows"] / cnt["ffn_calls"]))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run()
        for _ in range(2):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / 5 / T * 1e6
        rows.append({"k": k, "rows_in_cache": cnt["ffn_rows"] / cnt["ffn_calls"],
                     "cache_fraction_of_ffn": cnt["ffn_rows"] / cnt["ffn_calls"] / w.d_ffn,
                     "rows_added_per_token": cnt["added"] / cnt["steps"],
                     "h2d_bytes_per_token": cnt["added"] / cnt["steps"] * w.bundle_bytes,
                     "us_per_token": us})
        lay.close()
        del gpu, lay
    print(json.dumps({"sweep": "window size k", "workload": describe(base_w), "rows": rows}))


def sweep_chunk(args):
    """Host-to-device throughput of the bundle gather against the chunk size (the analogue of the paper's
    Fig. 2b and of Table 1's bundling row: one read of 2*d*E bytes per neuron instead of two reads of d*E).
    Same bytes per step (about 2.4 MB of new bundles) at every chunk size; masks are forced through the
    predictor offset so that exactly `rows` new neurons appear per step."""
    import numpy as np
    import torch
    import paper_2312_11514_amd as lif
    dev = torch.device("cuda:0")
    F, r = 16384, 32
    rng = np.random.default_rng(0)
    out = []
    for d in (256, 512, 1024, 2048, 4096, 8192):
        bundle = 2 * d * 2
        rows = max(1, int(round(2.4e6 / bundle)))
        host = torch.from_numpy(rng.standard_normal((F, 2 * d), dtype=np.float32).astype(np.float16)).pin_memory()
        A = torch.zeros((r, d), dtype=torch.float16, device=dev)
        B = torch.zeros((r, F), dtype=torch.float16, device=dev)
        c = torch.zeros(F, device=dev)
        b = torch.zeros(F, device=dev)
        x = torch.zeros(d, dtype=torch.float16, device=dev)
        y = torch.zeros(d, dtype=torch.float16, device=dev)
        lay = lif.Layer(d_model=d, d_ffn=F, rank=r, window_k=1, capacity_rows=F, dtype="f16", A=A, B=B, c=c, b=b,
                        host_bundles=host)
        ts = []
        for it in range(14):
            m = np.full(F, -1.0, np.float32)
            m[rng.choice(F, rows, replace=False)] = 1.0
            c.copy_(torch.from_numpy(m))
            torch.cuda.synchronize()
            lay.profile_begin(16)
            lay.step(x, y)
            ts.append(lay.profile_collect()["load"][0] * 1e3)
        t = float(np.median(ts[4:]))
        out.append({"d_model": d, "chunk_bytes": bundle, "unbundled_chunk_bytes": bundle // 2, "rows_per_step": rows,
                    "load_kernel_us_event_timed": t, "GBs": rows * bundle / t / 1e3})
        lay.close()
    print(json.dumps({"sweep": "chunk size (bundle bytes) at ~2.4 MB per step", "rows": out}))


def sweep_rows(args):
    """Bandwidth of one lif_sparse_ffn call against the number of cached rows n (full-bundle mode reads n bundles,
    skip mode reads the activation vector of every row and the down column of the rows that fire).  Shows where the
    two FFN kernels leave the launch/latency regime: bytes grow with n, the fixed cost does not."""
    import numpy as np
    import torch
    import workloads as wl
    import paper_2312_11514_amd as lif
    from workloads.device import GpuLayer
    w0 = wl.WORKLOADS[args.workload]
    w = wl.scaled(w0, capacity_rows=w0.d_ffn)
    L = wl.make_layer(w)
    X = wl.make_inputs(w) if w.batch == 1 else wl.make_batch_inputs(w)
    rng = np.random.default_rng(1)
    E, d, G = w.elem_bytes, w.d_model, w.vectors_per_bundle
    out = []
    for mode_name, mode in (("full", lif.FFN_FULL_BUNDLE), ("skip", lif.FFN_SKIP_DEAD)):
        gpu = GpuLayer(w, L, ffn_mode=mode)
        lay = gpu.layer
        xd = gpu.upload_x(X[0])
        n = 256
        while n <= w.d_ffn:
            ids = np.sort(rng.choice(w.d_ffn, n, replace=False))
            lay.reset()
            gpu.fill_cache(ids, L)
            lay.set_expected_rows(n)
            calls = 50
            g = torch.cuda.CUDAGraph()
            lay.sparse_ffn(xd, gpu.y, w.batch)
            torch.cuda.synchronize()
            with torch.cuda.graph(g):
                for _ in range(calls):
                    lay.sparse_ffn(xd, gpu.y, w.batch)
            g.replay()
            torch.cuda.synchronize()
            c0 = lay.counters()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(4):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            c1 = lay.counters()
            us = e0.elapsed_time(e1) * 1e3 / (4 * calls)
            active = (c1["ffn_active"] - c0["ffn_active"]) / (c1["ffn_calls"] - c0["ffn_calls"])
            req = n * (G - 1) * d * E + (n if mode_name == "full" else active) * d * E
            out.append({"mode": mode_name, "rows": n, "rows_active": active, "us_per_call": us,
                        "requested_bytes": req, "GBs": req / us / 1e3, "frac_of_8TBs": req / us / 1e3 / 8000.0})
            n *= 2
        lay.close()
        del gpu, lay
    print(json.dumps({"sweep": "cached rows per lif_sparse_ffn call", "workload": describe(w), "rows": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--ffn-mode", default="skip", choices=["skip", "full"],
                    help="skip: down columns read only for rows with a non-zero activation; full: whole bundles")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from the host instead of a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also run a plain 256 MiB device copy three times (calibration of rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--pmc-dir", default=None,
                    help="directory with the rocprofv3 --pmc outputs of this script; fills roofline.traffic")
    ap.add_argument("--no-hint", action="store_true", help="do not give the library the expected number of cached rows")
    ap.add_argument("--structured", action="store_true",
                    help="second workload: 1/j singular spectrum of the ReLU'd projection, so that the rank-r predictor "
                         "is accurate (labelled in the output; never mixed with the default)")
    ap.add_argument("--overpredict", type=float, default=1.0,
                    help="predictor calibrated to fire on overpredict * p_active of the neurons")
    ap.add_argument("--sweep", default=None, choices=["k", "chunk", "rows"],
                    help="instead of the bench line: window-size sweep or chunk-size sweep (one JSON line each)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.sweep == "k":
        return sweep_window(args)
    if args.sweep == "chunk":
        return sweep_chunk(args)
    if args.sweep == "rows":
        return sweep_rows(args)

    import torch
    import workloads as wl
    import paper_2312_11514_amd as lif
    from workloads.device import GpuLayer

    if args.pmc_copy:
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float16, device="cuda:0")      # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    w = wl.WORKLOADS[args.workload]
    NL = w.layers
    steps = args.steps if args.steps is not None else (20 if NL == 1 else 3)
    warmup = args.warmup if args.warmup is not None else (3 if NL == 1 else 1)
    mode = {"skip": lif.FFN_SKIP_DEAD, "full": lif.FFN_FULL_BUNDLE}[args.ffn_mode]
    reads_all = args.ffn_mode == "full"

    base = wl.make_layer(w, structured=args.structured, overpredict=args.overpredict)
    spec = w.spec_keep > 0
    X = wl.make_inputs(w) if (w.batch == 1 or spec) else wl.make_batch_inputs(w)
    if spec:
        # pass p verifies tokens [p * keep, p * keep + batch): the next pass starts after the accepted ones
        import numpy as np
        n_pass = (len(X) - w.batch) // w.spec_keep + 1
        X = np.stack([X[p * w.spec_keep:p * w.spec_keep + w.batch] for p in range(n_pass)])
    T = len(X)
    gpus = []
    for l in range(NL):
        Ll = wl.make_layer_variant(base, w, l)
        gpus.append(GpuLayer(w, Ll, ffn_mode=mode))      # uploads A, B, c, b; pins the bundle store
        del Ll
    layers = [g.layer for g in gpus]
    xd = gpus[0].upload_x(X)                              # [T, (batch,) d] resident in HBM
    yd = torch.zeros((NL,) + tuple(xd.shape), dtype=xd.dtype, device=xd.device)

    if NL == 1:
        # whole token stream of the layer in one HIP graph
        def run_stream(tokens=None):
            lay0 = layers[0]
            lay0.reset()
            for t in range(T if tokens is None else tokens):
                if spec:
                    lay0.step_tokens(xd[t], yd[0, t], w.batch, w.spec_keep)
                else:
                    lay0.step(xd[t], yd[0, t], w.batch)
        graph = None
        run_stream()                                      # eager pass: validates the chain, fills counters
        torch.cuda.synchronize()
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                run_stream()
        step = graph.replay if graph is not None else run_stream
        launch = "eager" if graph is None else "hip-graph of the whole token stream"
    else:
        # one HIP graph per token (all layers); x of the token is copied to a fixed staging buffer first
        x_stage = torch.zeros_like(xd[0])
        y_stage = torch.zeros((NL,) + tuple(xd[0].shape), dtype=xd.dtype, device=xd.device)

        def token_all_layers():
            for l, lay in enumerate(layers):
                lay.step(x_stage, y_stage[l], w.batch)
        for lay in layers:
            lay.reset()
        x_stage.copy_(xd[0])
        token_all_layers()
        torch.cuda.synchronize()
        graph = None
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                token_all_layers()
        tok = graph.replay if graph is not None else token_all_layers

        def step():
            for lay in layers:
                lay.reset()
            for t in range(T):
                x_stage.copy_(xd[t])
                tok()
        step()                                            # validation pass, fills counters
        torch.cuda.synchronize()
        launch = "eager" if graph is None else "one hip-graph per token (all layers), x copied to a staging buffer"

    sts = [lay.state() for lay in layers]
    assert all(s["error"] == 0 for s in sts), sts
    window_len_end = sts[0]["window_len"]
    cnts = [lay.counters() for lay in layers]
    tot = {k: sum(c[k] for c in cnts) for k in cnts[0]}
    rows_per_call = tot["ffn_rows"] / tot["ffn_calls"]
    active_per_call = tot["ffn_active"] / tot["ffn_calls"]
    added_per_call = tot["added"] / tot["steps"]

    # row-count hint for the FFN launch geometry (performance only): 90 % of the mean rows in use
    if not args.no_hint:
        for lay in layers:
            lay.set_expected_rows(int(0.9 * rows_per_call))
        if graph is not None:                             # launch geometry changed: capture again
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                (run_stream if NL == 1 else token_all_layers)()
            if NL == 1:
                step = graph.replay
            else:
                tok = graph.replay

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    us_per_token_layer = ms_per_step * 1e3 / T / NL

    # steady state (single layer, graph launches): the first 2k steps fill the cache and load far more than the
    # later ones; a second graph over just those steps is timed and subtracted
    steady = None
    Wm = 2 * w.window_k
    if NL == 1 and graph is not None and T > 2 * Wm:
        gw = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gw):
            run_stream(Wm)
        gw.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            gw.replay()
        torch.cuda.synchronize()
        warm_ms = (time.perf_counter() - t0) / steps * 1e3
        steady = {"first_steps_excluded": Wm, "us_per_step": (ms_per_step - warm_ms) * 1e3 / (T - Wm),
                  "us_per_step_in_the_first_steps": warm_ms * 1e3 / Wm}

    # host link reference on the same box: one large pinned-to-device copy by the runtime (copy engine)
    h2d_ref = None
    if not args.no_profile:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8).pin_memory()
        dst = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=xd.device)
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            dst.copy_(src, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        h2d_ref = 3 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst

    # FFN alone, on the cache state the stream ends in: R rounds of lif_sparse_ffn over all layers in a HIP graph,
    # timed with HIP events on the launch stream; the byte count comes from the device counters of those calls.
    # With one layer the rows stay warm in the 256 MB Infinity Cache; with 32 layers each call reads its rows from HBM.
    ffn = None
    if not args.no_profile:
        R = 200 if NL == 1 else 8
        x_last = xd[T - 1]
        def ffn_rounds():
            for _ in range(R):
                for l, lay in enumerate(layers):
                    lay.sparse_ffn(x_last, yd[l, T - 1], w.batch)
        if args.no_graph:
            class _Eager:
                replay = staticmethod(ffn_rounds)
            g2 = _Eager()
        else:
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                ffn_rounds()
        g2.replay()
        torch.cuda.synchronize()
        c0 = [lay.counters() for lay in layers]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 5
        e0.record()
        for _ in range(reps):
            g2.replay()
        e1.record()
        torch.cuda.synchronize()
        c1 = [lay.counters() for lay in layers]
        calls = sum(b["ffn_calls"] - a["ffn_calls"] for a, b in zip(c0, c1))
        assert calls == R * reps * NL
        rows = sum(b["ffn_rows"] - a["ffn_rows"] for a, b in zip(c0, c1)) / calls
        act = sum(b["ffn_active"] - a["ffn_active"] for a, b in zip(c0, c1)) / calls
        ffn = {"us": e0.elapsed_time(e1) * 1e3 / calls, "rows": rows, "active": act}

    # per-kernel durations over one more eager pass (layer 0 only is instrumented): HIP events recorded by the
    # library on the launch stream around every kernel (these include ~2 us of event/dispatch overhead per launch)
    kern = {}
    if not args.no_profile:
        layers[0].profile_begin(7 * T + 8)
        if NL == 1:
            run_stream()
        else:
            for lay in layers:
                lay.reset()
            for t in range(T):
                x_stage.copy_(xd[t])
                token_all_layers()
        for k, (ms, n) in layers[0].profile_collect().items():
            if n:
                kern[k] = {"avg_us": ms / n * 1e3, "launches": n}

    E, d, G = w.elem_bytes, w.d_model, w.vectors_per_bundle
    nominal = rows_per_call * G * d * E
    out = {
        "metric": "sparse-FFN us/token/layer (whole hot path: predict + window + load + FFN)",
        "value": us_per_token_layer, "unit": "us/token/layer", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": describe(w) + (" structured-spectrum" if args.structured else "") +
                               (f" overpredict={args.overpredict}" if args.overpredict != 1.0 else ""),
                   "tokens_per_step": T, "layers": NL, "ffn_mode": args.ffn_mode,
                   "launch": launch,
                   "llc": ("single layer: the cache working set stays warm in the 256 MB Infinity Cache" if NL == 1 else
                           f"{NL} layers rotate {NL * nominal / 1e6:.0f} MB of cached rows per token: FFN reads come from HBM")},
        "per_token_per_layer": {"rows_in_cache": rows_per_call, "rows_active": active_per_call,
                                "rows_added": added_per_call, "h2d_bytes": added_per_call * w.bundle_bytes,
                                "nominal_bundle_bytes": nominal},
        "window_len_at_end": window_len_end,
        "steady_state": steady,
        "speculative": ({"tokens_per_pass": w.batch, "kept_per_pass": w.spec_keep, "passes": T,
                         "us_per_accepted_token": us_per_token_layer / w.spec_keep} if spec else None),
        "end_to_end_us_per_token": us_per_token_layer * NL,
        "h2d_bytes_per_token": added_per_call * w.bundle_bytes * NL,
    }
    if ffn:
        up_bytes = ffn["rows"] * (G - 1) * d * E
        down_bytes = (ffn["rows"] if reads_all else ffn["active"]) * d * E
        touched = up_bytes + down_bytes
        nominal_f = ffn["rows"] * G * d * E
        ach = touched / (ffn["us"] * 1e-6) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "ffn_up + ffn_down (one lif_sparse_ffn call)",
                           "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                           "traffic": None, "algorithmic_bytes_per_launch": touched, "avg_launch_us": ffn["us"],
                           "rows": ffn["rows"], "rows_active": ffn["active"],
                           "nominal_bundle_bytes": nominal_f,
                           "nominal_GBs": nominal_f / (ffn["us"] * 1e-6) / 1e9,
                           "nominal_frac": nominal_f / (ffn["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS}
    if ffn and args.pmc_dir:
        tr = pmc_traffic(args.pmc_dir)
        if tr:
            out["roofline"]["traffic"] = tr["FETCH_SIZE"]["bytes_per_call"] + tr["WRITE_SIZE"]["bytes_per_call"]
            out["roofline"]["traffic_detail"] = tr
    if kern:
        out["h2d"] = {"GBs_in_load_kernel": added_per_call * w.bundle_bytes / (kern["load"]["avg_us"] * 1e-6) / 1e9,
                      "GBs_large_pinned_memcpy_same_box": h2d_ref}
        out["kernels_avg_us_event_timed"] = {k: round(v["avg_us"], 3) for k, v in kern.items()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, base, X)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
