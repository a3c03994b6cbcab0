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
           "cores_note": "threads of the BLAS pool under numpy's matrix products; the oracle itself is one Python "
                         "thread (its window, delete and insert steps are plain loops), so more threads do not help it",
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
        # one lif_sparse_ffn call = a k_ffn_up dispatch and the k_ffn_down (+ finish) dispatches right after it
        # (lif_step never launches k_ffn_up on its own, so these are exactly the FFN-only calls)
        rows.sort(key=lambda r: int(r["Dispatch_Id"]))
        calls, total, open_call = 0, 0.0, False
        for r in rows:
            name = r["Kernel_Name"]
            if "k_ffn_up" in name:
                calls, open_call = calls + 1, True
                total += float(r["Counter_Value"])
            elif open_call and "k_ffn_down" in name:
                total += float(r["Counter_Value"])
            else:
                open_call = False
        if not calls:
            return None
        out[counter] = {"scale": scale, "bytes_per_call": total * scale * 1024.0 / calls, "calls": calls}
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
    for k in range(1, 17):
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


def _forced_gather(d, F, rows, unbundled, pairs_list, rng, steps=14):
    """Event-timed load kernel of lif_step when exactly `rows` new neurons appear per step (masks forced through the
    predictor offset).  Returns {pairs: median us}."""
    import numpy as np
    import torch
    import paper_2312_11514_amd as lif
    dev = torch.device("cuda:0")
    r = 32
    store = rng.standard_normal((F, 2 * d), dtype=np.float32).astype(np.float16)
    if unbundled:
        host = torch.from_numpy(np.ascontiguousarray(store[:, :d])).pin_memory()
        host_down = torch.from_numpy(np.ascontiguousarray(store[:, d:])).pin_memory()
    else:
        host, host_down = torch.from_numpy(store).pin_memory(), None
    A = torch.zeros((r, d), dtype=torch.float16, device=dev)
    B = torch.zeros((r, F), dtype=torch.float16, device=dev)
    c = torch.zeros(F, device=dev)
    b = torch.zeros(F, device=dev)
    x = torch.zeros(d, dtype=torch.float16, device=dev)
    y = torch.zeros(d, dtype=torch.float16, device=dev)
    lay = lif.Layer(d_model=d, d_ffn=F, rank=r, window_k=1, capacity_rows=F, dtype="f16", A=A, B=B, c=c, b=b,
                    host_bundles=host, host_down=host_down)
    out = {}
    for pairs in pairs_list:
        lay.set_loader_pairs(pairs)
        ts = []
        for it in range(steps):
            m = np.full(F, -1.0, np.float32)
            m[rng.choice(F, rows, replace=False)] = 1.0
            c.copy_(torch.from_numpy(m))
            torch.cuda.synchronize()
            lay.profile_begin(16)
            lay.step(x, y)
            ts.append(lay.profile_collect()["load"][0] * 1e3)
        out[pairs] = float(np.median(ts[4:]))
    lay.close()
    return out


def sweep_chunk(args):
    """Host-to-device throughput of the bundle gather against the chunk size (the analogue of the paper's
    Fig. 2b and of Table 1's bundling row: one read of 2*d*E bytes per neuron instead of two reads of d*E from two
    arrays).  Same bytes per step (about 2.4 MB of new bundles) at every chunk size; both layouts are measured."""
    import numpy as np
    F = 16384
    rng = np.random.default_rng(0)
    out = []
    for d in (256, 512, 1024, 2048, 4096, 8192):
        bundle = 2 * d * 2
        rows = max(1, int(round(2.4e6 / bundle)))
        tb = _forced_gather(d, F, rows, False, [0], rng)[0]
        tu = _forced_gather(d, F, rows, True, [0], rng)[0]
        out.append({"d_model": d, "chunk_bytes": bundle, "unbundled_chunk_bytes": bundle // 2, "rows_per_step": rows,
                    "load_kernel_us_event_timed": tb, "GBs": rows * bundle / tb / 1e3,
                    "unbundled_load_kernel_us_event_timed": tu, "unbundled_GBs": rows * bundle / tu / 1e3})
    print(json.dumps({"sweep": "chunk size (bundle bytes) at ~2.4 MB per step, bundled and not bundled", "rows": out}))


def sweep_loaders(args):
    """Host-link throughput of lif_step's gather against the number of loader wave pairs (bundles in flight), at the
    OPT shape: 146 new bundles of 16 KiB per step.  Shows the ceiling of a shader-driven gather on this link."""
    import numpy as np
    rng = np.random.default_rng(0)
    d, F, rows = 4096, 16384, 146
    pairs = [2, 4, 6, 8, 10, 12, 16, 20, 24, 32, 48, 64]
    t = _forced_gather(d, F, rows, False, pairs, rng)
    out = [{"loader_pairs": p, "KiB_in_flight": p * 16, "load_kernel_us_event_timed": t[p],
            "GBs": rows * 4 * d / t[p] / 1e3} for p in pairs]
    print(json.dumps({"sweep": "loader wave pairs of lif_step at 146 bundles of 16 KiB per step", "rows": out}))


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


_T0 = time.perf_counter()


def progress(msg):
    print(f"[bench {time.perf_counter() - _T0:6.1f}s] {msg}", file=sys.stderr, flush=True)


def _timed_replays(graph, reps):
    """HIP events on the launch stream around `reps` replays of a captured graph; returns milliseconds."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1)


def read_floor(dev, sizes):
    """Same-box reference for the roofline: a plain streaming-read kernel (lif_profile_read) launched back to back
    inside a HIP graph, for an empty launch and for the given byte counts.  Buffers up to 64 MB are read again and
    again (warm in the 256 MB Infinity Cache, like a single layer's cache); the larger ones cycle through 2 GiB."""
    import torch
    import paper_2312_11514_amd as lif
    big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    big.zero_()
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    out = {}
    for name, nbytes in sizes:
        nbytes = int(nbytes) // 16 * 16
        warm = nbytes <= (64 << 20)
        n_launch = 200 if warm else max(4, min(64, (8 << 30) // max(nbytes, 1)))
        slots = 1 if warm else max(1, (2 << 30) // nbytes)
        g = torch.cuda.CUDAGraph()
        lif.profile_read(big, nbytes, sink)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            for i in range(n_launch):
                lif.profile_read(big[(i % slots) * nbytes:], nbytes, sink)
        g.replay()
        torch.cuda.synchronize()
        us = _timed_replays(g, 5) * 1e3 / (5 * n_launch)
        out[name] = {"bytes": nbytes, "us_per_launch": us, "GBs": nbytes / us / 1e3 if nbytes else None,
                     "source": "Infinity-Cache warm" if warm else "HBM (2 GiB cycled)"}
    del big
    # what a hand-off inside one kernel costs against a second launch: lif_profile_handoff plain, with a fence +
    # ticket tail, and with stamped words polled by one workgroup; 200 launches back to back in a graph.  Every
    # launch of the stamped form needs a fresh stamp, so its graph is replayed once only, three graphs.
    scratch = torch.zeros(lif.profile_handoff_bytes(), dtype=torch.uint8, device=dev)
    ho, stamp = {}, 1
    for mode, key in ((0, "plain_us_per_launch"), (1, "fenced_tail_us_per_launch"), (2, "stamped_words_polled_us_per_launch")):
        lif.profile_handoff(scratch, mode, stamp)
        stamp += 1
        torch.cuda.synchronize()
        times = []
        for rep in range(3):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(200):
                    lif.profile_handoff(scratch, mode, stamp)
                    stamp += 1
            torch.cuda.synchronize()
            times.append(_timed_replays(g, 1) * 1e3 / 200)
        ho[key] = min(times)
    ho["stamped_words_give_ups"] = int(scratch[256 * 16384 + 4100:256 * 16384 + 4104].view(torch.int32).item())
    ho["what"] = ("256 workgroups read 16 KiB and produce 8 bytes each (the mask kernel's shape); fenced tail: every "
                  "workgroup passes __threadfence and a ticket, the last one reads the 2 KiB back; stamped words: "
                  "relaxed device-scope atomic stores of (payload, stamp) words that workgroup 0 polls, bounded")
    out["handoff_inside_a_kernel"] = ho
    return out


def ffn_over_states(w, gpu0, L0, states, xd, mode, hint, no_graph):
    """The FFN alone over several (cache state, x) pairs of the stream.

    One more layer handle per state shares layer 0's predictor arrays and bundle store and holds that token's cache
    (same slot order).  warm: per state, a HIP graph of 50 back-to-back lif_sparse_ffn calls (the rows stay in the
    256 MB Infinity Cache).  cold: one HIP graph that calls every state's layer in turn, 8 rounds: 32 caches of
    ~20 MB are 640 MB, so every call streams its rows from HBM."""
    import torch
    from workloads.device import GpuLayer
    import numpy as np
    E, d, G = w.elem_bytes, w.d_model, w.vectors_per_bundle
    reads_all = mode != 0
    lays = []
    for t, ids in states:
        g = GpuLayer(w, L0, ffn_mode=mode, share=gpu0)
        g.fill_cache(ids, L0)
        if hint:
            g.layer.set_expected_rows(hint)
        if w.gate_resident:
            g.layer.predict(xd[t], w.batch)           # leaves the gate activations the FFN of this variant reads
        lays.append((t, g))
    torch.cuda.synchronize()

    def measure(calls_fn, n_calls, reps, which):
        if no_graph:
            class _E:
                replay = staticmethod(calls_fn)
            g = _E()
        else:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                calls_fn()
        g.replay()
        torch.cuda.synchronize()
        c0 = [l.layer.counters() for _, l in which]
        ms = _timed_replays(g, reps)
        c1 = [l.layer.counters() for _, l in which]
        calls = sum(b["ffn_calls"] - a["ffn_calls"] for a, b in zip(c0, c1))
        assert calls == n_calls * reps, (calls, n_calls, reps)
        rows = sum(b["ffn_rows"] - a["ffn_rows"] for a, b in zip(c0, c1)) / calls
        act = sum(b["ffn_active"] - a["ffn_active"] for a, b in zip(c0, c1)) / calls
        return ms * 1e3 / calls, rows, act

    def fig(us, rows, act):
        touched = rows * (G - 1) * d * E + (rows if reads_all else act) * d * E
        nominal = rows * G * d * E
        return {"avg_launch_us": us, "rows": rows, "rows_active": act, "algorithmic_bytes_per_launch": touched,
                "achieved": touched / us / 1e3, "nominal_bundle_bytes": nominal, "nominal_GBs": nominal / us / 1e3}

    per_state = []
    for t, g in lays[:16]:
        def calls(g=g, t=t):
            for _ in range(50):
                g.layer.sparse_ffn(xd[t], g.y, w.batch)
        per_state.append(fig(*measure(calls, 50, 4, [(t, g)])))

    def all_layers():
        for _ in range(8):
            for t, g in lays:
                g.layer.sparse_ffn(xd[t], g.y, w.batch)
    cold = fig(*measure(all_layers, 8 * len(lays), 5, lays))
    cold["caches"] = len(lays)
    cold["bytes_cycled"] = sum(len(ids) for _, ids in states) * G * d * E
    cold["address_span_bytes"] = len(lays) * w.capacity_rows * G * d * E
    for _, g in lays:
        g.layer.close()
    del lays
    # the same states in caches preallocated for 2048 rows only: a quarter of the address span, same bytes read -
    # separates the reach of the address translation from the latency of HBM itself
    small_cap = 2048
    if max(len(ids) for _, ids in states) <= small_cap < w.capacity_rows:
        lays = []
        for t, ids in states:
            g = GpuLayer(w, L0, ffn_mode=mode, share=gpu0, capacity=small_cap)
            g.fill_cache(ids, L0)
            if hint:
                g.layer.set_expected_rows(hint)
            if w.gate_resident:
                g.layer.predict(xd[t], w.batch)
            lays.append((t, g))
        torch.cuda.synchronize()
        c2 = fig(*measure(all_layers, 8 * len(lays), 5, lays))
        cold["compact_caches"] = {"capacity_rows": small_cap, "address_span_bytes": len(lays) * small_cap * G * d * E,
                                  "avg_launch_us": c2["avg_launch_us"], "achieved": c2["achieved"]}
        for _, g in lays:
            g.layer.close()
    return per_state, cold


def roofline_object(f, kernel, extra=None):
    out = {"bound": "hbm", "kernel": kernel, "achieved": f["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": f["achieved"] / HBM_PEAK_GBS, "traffic": None,
           "algorithmic_bytes_per_launch": f["algorithmic_bytes_per_launch"], "avg_launch_us": f["avg_launch_us"],
           "rows": f["rows"], "rows_active": f["rows_active"], "nominal_bundle_bytes": f["nominal_bundle_bytes"],
           "nominal_GBs": f["nominal_GBs"], "nominal_frac": f["nominal_GBs"] / HBM_PEAK_GBS}
    out.update(extra or {})
    return out


def bench_stacked(w, base, mode, steps, warmup, no_graph=False, hint=True, ffn_rounds=8, profile=True):
    """Stacked layers (C5): every layer has its own predictor, window, cache and pinned bundle store; one HIP graph
    per token covers all layers.  Returns the figures of the bench line that depend on the run."""
    import torch
    import workloads as wl
    from workloads.device import GpuLayer
    NL = w.layers
    X = wl.make_inputs(w)
    T = len(X)
    gpus = []
    for l in range(NL):
        Ll = wl.make_layer_variant(base, w, l)
        gpus.append(GpuLayer(w, Ll, ffn_mode=mode))      # uploads A, B, c, b; pins the bundle store
        del Ll
        if l % 8 == 7:
            progress(f"  layer {l + 1} of {NL} uploaded")
    layers = [g.layer for g in gpus]
    xd = gpus[0].upload_x(X)
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

    def capture():
        if no_graph:
            return token_all_layers
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            token_all_layers()
        return g.replay
    tok = capture()

    def step():
        for lay in layers:
            lay.reset()
        for t in range(T):
            x_stage.copy_(xd[t])
            tok()
    step()                                            # validation pass, fills counters
    torch.cuda.synchronize()
    progress("  stacked validation pass done")
    sts = [lay.state() for lay in layers]
    assert all(s["error"] == 0 for s in sts), sts
    cnts = [lay.counters() for lay in layers]
    tot = {k: sum(c[k] for c in cnts) for k in cnts[0]}
    rows_per_call = tot["ffn_rows"] / tot["ffn_calls"]
    if hint:
        for lay in layers:
            lay.set_expected_rows(int(1.15 * rows_per_call))
        tok = capture()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    res = {"T": T, "NL": NL, "ms_per_step": ms_per_step, "us_per_token_layer": ms_per_step * 1e3 / T / NL,
           "rows_per_call": rows_per_call, "active_per_call": tot["ffn_active"] / tot["ffn_calls"],
           "added_per_call": tot["added"] / tot["steps"], "window_len_end": sts[0]["window_len"],
           "launch": "eager" if no_graph else "one hip-graph per token (all layers), x copied to a staging buffer",
           "ffn": None, "kern": {}}
    if profile:
        # FFN alone on the cache states the stream ends in: every call reads another layer's rows, i.e. from HBM
        x_last = xd[T - 1]

        def rounds():
            for _ in range(ffn_rounds):
                for l, lay in enumerate(layers):
                    lay.sparse_ffn(x_last, y_stage[l], w.batch)
        if no_graph:
            class _E:
                replay = staticmethod(rounds)
            g2 = _E()
        else:
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                rounds()
        g2.replay()
        torch.cuda.synchronize()
        c0 = [lay.counters() for lay in layers]
        ms = _timed_replays(g2, 5)
        c1 = [lay.counters() for lay in layers]
        calls = sum(b["ffn_calls"] - a["ffn_calls"] for a, b in zip(c0, c1))
        res["ffn"] = {"us": ms * 1e3 / calls,
                      "rows": sum(b["ffn_rows"] - a["ffn_rows"] for a, b in zip(c0, c1)) / calls,
                      "active": sum(b["ffn_active"] - a["ffn_active"] for a, b in zip(c0, c1)) / calls}
        layers[0].profile_begin(7 * T + 8)
        for lay in layers:
            lay.reset()
        for t in range(T):
            x_stage.copy_(xd[t])
            token_all_layers()
        for k, (ms, n) in layers[0].profile_collect().items():
            if n:
                res["kern"][k] = {"avg_us": ms / n * 1e3, "launches": n}
    for lay in layers:
        lay.close()
    return res


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
    ap.add_argument("--no-c5", action="store_true",
                    help="skip the stacked-layer leg (32 layers, 512 tokens) that the default C2 line carries as `c5`")
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
    ap.add_argument("--sweep", default=None, choices=["k", "chunk", "rows", "loaders"],
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
    if args.sweep == "loaders":
        return sweep_loaders(args)

    import numpy as np
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
    E, d, G = w.elem_bytes, w.d_model, w.vectors_per_bundle

    progress(f"building workload {w.name}")
    base = wl.make_layer(w, structured=args.structured, overpredict=args.overpredict)
    spec = w.spec_keep > 0
    X = wl.make_inputs(w) if (w.batch == 1 or spec) else wl.make_batch_inputs(w)
    if spec:
        # pass p verifies tokens [p * keep, p * keep + batch): the next pass starts after the accepted ones
        n_pass = (len(X) - w.batch) // w.spec_keep + 1
        X = np.stack([X[p * w.spec_keep:p * w.spec_keep + w.batch] for p in range(n_pass)])
    T = len(X)

    steady = ffn_states = ffn_cold = floor = breakdown = None
    kern = {}
    ffn = None
    if NL > 1:
        r = bench_stacked(w, base, mode, steps, warmup, no_graph=args.no_graph, hint=not args.no_hint,
                          profile=not args.no_profile)
        ms_per_step, us_per_token_layer = r["ms_per_step"], r["us_per_token_layer"]
        rows_per_call, active_per_call, added_per_call = r["rows_per_call"], r["active_per_call"], r["added_per_call"]
        window_len_end, launch, ffn, kern = r["window_len_end"], r["launch"], r["ffn"], r["kern"]
        h2d_ref = None
    else:
        progress("uploading layer 0")
        gpu0 = GpuLayer(w, base, ffn_mode=mode)               # uploads A, B, c, b; pins the bundle store
        lay0 = gpu0.layer
        xd = gpu0.upload_x(X)                                  # [T, (batch,) d] resident in HBM
        yd = torch.zeros_like(xd)

        def one_step(t, calls=False):
            if spec:
                lay0.step_tokens(xd[t], yd[t], w.batch, w.spec_keep)
            elif calls:
                lay0.step_calls(xd[t], yd[t], w.batch)
            else:
                lay0.step(xd[t], yd[t], w.batch)

        def run_stream(tokens=None):
            lay0.reset()
            for t in range(T if tokens is None else tokens):
                one_step(t)

        # eager pass: validates the chain, fills the counters, and keeps the cache layout at 32 tokens spread over
        # the steady part of the stream (the FFN alone is timed on those states afterwards)
        snap_at = sorted(set(np.linspace(min(T - 1, 4 * w.window_k), T - 1, 32).astype(int).tolist()))
        states = []
        lay0.reset()
        for t in range(T):
            one_step(t)
            if t in snap_at and not args.no_profile:
                n = lay0.state()["num_used"]
                states.append((t, lay0.pointers[:n].cpu().numpy().astype(np.int64)))
        torch.cuda.synchronize()
        st0 = lay0.state()
        assert st0["error"] == 0, st0
        window_len_end = st0["window_len"]
        tot = lay0.counters()
        rows_per_call = tot["ffn_rows"] / tot["ffn_calls"]
        active_per_call = tot["ffn_active"] / tot["ffn_calls"]
        added_per_call = tot["added"] / tot["steps"]
        hint = 0 if args.no_hint else int(1.15 * rows_per_call)  # launch geometry only: a wave for every row of nearly every step
        lay0.set_expected_rows(hint)

        progress("validation pass done; capturing and timing the token stream")
        graph = None
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()                     # whole token stream of the layer in one HIP graph
            with torch.cuda.graph(graph):
                run_stream()
        step = graph.replay if graph is not None else run_stream
        launch = "eager" if graph is None else "hip-graph of the whole token stream"
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) / steps * 1e3
        us_per_token_layer = ms_per_step * 1e3 / T

        # steady state: the first 2k steps fill the cache and load far more than the later ones; a second graph over
        # just those steps is timed and subtracted
        Wm = 2 * w.window_k
        if graph is not None and T > 2 * Wm:
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

        h2d_ref = None
        if not args.no_profile:
            # host link reference on the same box: one large pinned-to-device copy by the runtime (copy engine)
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

            progress("timed; FFN alone over the kept cache states")
            # FFN alone over the (cache state, x) pairs kept above: warm (one state per graph) and HBM-cold
            ffn_states, ffn_cold = ffn_over_states(w, gpu0, base, states, xd, mode, hint, args.no_graph)
            mean_bytes = float(np.mean([f["algorithmic_bytes_per_launch"] for f in ffn_states]))
            mean_nominal = float(np.mean([f["nominal_bundle_bytes"] for f in ffn_states]))
            progress("read floor of the box")
            floor = read_floor(xd.device, [("empty_launch", 0), ("ffn_algorithmic_bytes", mean_bytes),
                                           ("ffn_nominal_bundle_bytes", mean_nominal), ("256MiB", 256 << 20),
                                           ("1GiB", 1 << 30)])

            # per-kernel durations over two more eager passes: HIP events recorded by the library on the launch
            # stream around every kernel (these include ~2 us of event/dispatch overhead per launch); first the
            # lif_step path that `value` times, then the four separate calls for the paper's three cost columns
            progress("event-timed passes")
            for calls in (False, True):
                lay0.profile_begin(7 * T + 8)
                lay0.reset()
                for t in range(T):
                    one_step(t, calls=calls)
                got = {k: {"avg_us": ms / n * 1e3, "launches": n}
                       for k, (ms, n) in lay0.profile_collect().items() if n}
                if not calls:
                    kern = got
                elif not spec:
                    per_tok = {k: v["avg_us"] * v["launches"] / T for k, v in got.items()}
                    breakdown = {"io": per_tok.get("load", 0.0), "mem": per_tok.get("window", 0.0),
                                 "compute": sum(per_tok.get(k, 0.0) for k in ("predict_xa", "predict_mask", "ffn_up",
                                                                              "ffn_down")),
                                 "path": "four separate calls, event-timed per kernel (about 2 us of event overhead "
                                         "in each figure), microseconds per token",
                                 "definition": "io = bundle gather from pinned host memory (the row moves of the "
                                               "deletion ride in the same kernel, hidden behind the host reads); "
                                               "mem = window update and deletion plan; compute = predictor + FFN"}

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
    kernel_name = "ffn_up + ffn_down (one lif_sparse_ffn call)"
    if ffn_states:
        us = [f["avg_launch_us"] for f in ffn_states]
        tot_b = sum(f["algorithmic_bytes_per_launch"] for f in ffn_states)
        tot_n = sum(f["nominal_bundle_bytes"] for f in ffn_states)
        mean = {"avg_launch_us": float(np.mean(us)), "rows": float(np.mean([f["rows"] for f in ffn_states])),
                "rows_active": float(np.mean([f["rows_active"] for f in ffn_states])),
                "algorithmic_bytes_per_launch": tot_b / len(us), "achieved": tot_b / sum(us) / 1e3,
                "nominal_bundle_bytes": tot_n / len(us), "nominal_GBs": tot_n / sum(us) / 1e3}
        out["roofline"] = roofline_object(mean, kernel_name, {
            "memory": "warm: one cache state per graph of 50 calls, the rows stay in the 256 MB Infinity Cache",
            "states": {"count": len(us), "tokens": [t for t, _ in states[:16]],
                       "us_min": min(us), "us_max": max(us),
                       "rows_active_min": min(f["rows_active"] for f in ffn_states),
                       "rows_active_max": max(f["rows_active"] for f in ffn_states),
                       "frac_min": min(f["achieved"] for f in ffn_states) / HBM_PEAK_GBS,
                       "frac_max": max(f["achieved"] for f in ffn_states) / HBM_PEAK_GBS},
            "floor": floor})
        out["roofline_cold"] = roofline_object(ffn_cold, kernel_name, {
            "memory": f"HBM: {ffn_cold['caches']} caches of this layer ({ffn_cold['bytes_cycled'] / 1e6:.0f} MB of "
                      "bundles) called in turn, so no call finds its rows in the Infinity Cache",
            "address_span_bytes": ffn_cold["address_span_bytes"],
            "compact_caches": ffn_cold.get("compact_caches")})
    elif ffn:
        up_bytes = ffn["rows"] * (G - 1) * d * E
        down_bytes = (ffn["rows"] if reads_all else ffn["active"]) * d * E
        nominal_f = ffn["rows"] * G * d * E
        f = {"avg_launch_us": ffn["us"], "rows": ffn["rows"], "rows_active": ffn["active"],
             "algorithmic_bytes_per_launch": up_bytes + down_bytes,
             "achieved": (up_bytes + down_bytes) / ffn["us"] / 1e3,
             "nominal_bundle_bytes": nominal_f, "nominal_GBs": nominal_f / ffn["us"] / 1e3}
        out["roofline"] = roofline_object(f, kernel_name, {"memory": "HBM: every call reads another layer's rows"})
    if "roofline" in out and args.pmc_dir:
        tr = pmc_traffic(args.pmc_dir)
        if tr:
            out["roofline"]["traffic"] = tr["FETCH_SIZE"]["bytes_per_call"] + tr["WRITE_SIZE"]["bytes_per_call"]
            out["roofline"]["traffic_detail"] = tr
    if kern:
        out["h2d"] = {"GBs_in_load_kernel": added_per_call * w.bundle_bytes / (kern["load"]["avg_us"] * 1e-6) / 1e9,
                      "GBs_large_pinned_memcpy_same_box": h2d_ref}
        out["kernels_avg_us_event_timed"] = {k: round(v["avg_us"], 3) for k, v in kern.items()}
    if breakdown:
        out["breakdown_us"] = breakdown
    if NL == 1:
        del gpu0, lay0
    if args.workload == "C2" and not args.no_c5 and not args.structured and args.overpredict == 1.0:
        # configuration 5 (32 stacked layers of this shape, 512 tokens, own pinned store per layer): one timed pass
        w5 = wl.WORKLOADS["C5"]
        progress("stacked-layer leg (C5)")
        r5 = bench_stacked(w5, base, mode, 1, 0, no_graph=args.no_graph, hint=not args.no_hint, profile=False)
        out["c5"] = {"workload": describe(w5), "launch": r5["launch"], "timed_passes": 1,
                     "end_to_end_us_per_token": r5["us_per_token_layer"] * r5["NL"],
                     "us_per_token_per_layer": r5["us_per_token_layer"],
                     "h2d_bytes_per_token": r5["added_per_call"] * w5.bundle_bytes * r5["NL"],
                     "rows_in_cache_per_layer": r5["rows_per_call"]}
    if not args.no_cpu_baseline:
        progress("oracle on the host cores")
        out["cpu_baseline"] = cpu_baseline(w, base, X, budget_s=15.0)
    progress("done")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
