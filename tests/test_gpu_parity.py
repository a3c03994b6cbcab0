"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.

Bars: masks, step masks, added/removed ids, num_used, pointers, bias and cache rows bit-exact;
FFN output within 1e-3 relative L2 of the fp64 oracle (fp16 storage, fp32 accumulation).
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import lif_oracle as O

pytestmark = pytest.mark.gpu


def make_oracle(w, L, capacity=None, k=None):
    gate = w.gate_resident
    return O.OracleLayer(w.d_model, w.d_ffn, k or w.window_k, capacity or w.capacity_rows, w.glu and not gate,
                         L.A, L.B, L.c, L.theta, L.b, L.bundles, w_gate=L.w_gate if gate else None)


def run_stream(w, L, X, ffn_mode=0, check_every=1, api="calls", **gpu_args):
    from tests.harness import GpuLayer, compare_step
    gpu = GpuLayer(w, L, ffn_mode=ffn_mode, **gpu_args)
    ora = make_oracle(w, L)
    stats = []
    for t in range(len(X)):
        print(f"[{w.name}] token {t}", flush=True) if t % 32 == 0 else None
        stats.append(compare_step(gpu, ora, X[t], w, t, check_cache=(t % check_every == 0 or t == len(X) - 1), api=api))
    cnt = gpu.layer.counters()
    assert cnt["h2d_bytes"] == ora.bytes_loaded
    assert cnt["rows_moved"] == ora.rows_moved
    assert cnt["steps"] == len(X)
    assert ora.min_margin > 1e-9
    return stats


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("ffn_mode", [0, 1])
def test_c1_tiny_fp32_whole_path(ffn_mode, api):
    w = wl.WORKLOADS["C1"]
    stats = run_stream(w, wl.make_layer(w), wl.make_inputs(w), ffn_mode, api=api)
    assert max(s["err"] for s in stats) < 1e-5          # fp32 storage: far below the fp16 bar
    assert any(s["moved"] > 0 for s in stats) and any(s["removed"] > 0 for s in stats)


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("ffn_mode", [0, 1])
@pytest.mark.parametrize("glu", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_ragged_shapes_whole_path(glu, dtype, ffn_mode, api):
    """Shapes that end in a partial tile everywhere: d = 71 x 8 (like 4544 = 71 x 64), F not a
    multiple of 128, rank not a power of two, capacity not a multiple of 1024."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="ragged", d_model=568, d_ffn=1096, rank=40, window_k=3,
                  p_active=0.08, dtype=dtype, glu=glu, tokens=24, capacity_rows=700)
    run_stream(w, wl.make_layer(w), wl.make_inputs(w), ffn_mode, api=api)


def test_c2_opt_shape_fp16_whole_path():
    """OPT-6.7B FFN shape at full size, the launch configuration bench.py times, the whole stream of 256 tokens."""
    w = wl.WORKLOADS["C2"]
    L = wl.cached_layer("C2")
    X = wl.make_inputs(w)
    stats = run_stream(w, L, X, ffn_mode=0, check_every=8, api="step")
    assert np.mean([s["n"] for s in stats[10:]]) > 800         # window union of ~3 % active masks
    print("C2 max rel-L2 %.2e" % max(s["err"] for s in stats))


@pytest.mark.parametrize("ffn_mode", [1])
def test_c2_other_ffn_modes_match_oracle(ffn_mode):
    w = wl.WORKLOADS["C2"]
    L = wl.cached_layer("C2")
    X = wl.make_inputs(w, tokens=24)
    run_stream(w, L, X, ffn_mode=ffn_mode, check_every=8)


def test_c3_falcon_shape_fp16_whole_path():
    """Falcon-7B FFN shape: d = 4544 = 71 x 64 (ragged 16-byte tail), F = 18176 = 284 x 64."""
    w = wl.WORKLOADS["C3"]
    L = wl.cached_layer("C3")
    X = wl.make_inputs(w, tokens=96)
    stats = run_stream(w, L, X, check_every=8, api="step")
    print("C3 max rel-L2 %.2e, rows %.0f" % (max(s["err"] for s in stats), np.mean([s["n"] for s in stats[10:]])))


def test_c4_llama_shape_gated_batch1():
    w = wl.WORKLOADS["C4"]
    L = wl.cached_layer("C4")
    X = wl.make_inputs(w, tokens=64)
    stats = run_stream(w, L, X, check_every=8, api="step")
    print("C4 max rel-L2 %.2e, rows %.0f" % (max(s["err"] for s in stats), np.mean([s["n"] for s in stats[10:]])))


def test_c4_llama_shape_gated_batch8():
    """Eight independent streams share one cache: step mask = OR of the eight masks."""
    w = wl.WORKLOADS["C4b8"]
    L = wl.cached_layer("C4")            # same layer as the batch-1 run
    X = wl.make_batch_inputs(w, tokens=20)
    stats = run_stream(w, L, X, check_every=5)
    run_stream(w, L, X, check_every=5, api="step")
    print("C4b8 max rel-L2 %.2e, rows %.0f" % (max(s["err"] for s in stats), np.mean([s["n"] for s in stats[4:]])))


@pytest.mark.parametrize("k", [1, 3, 12, 64])
def test_window_sizes_including_longer_than_the_stream(k):
    """k = 1: cache = current mask; k = 12: more masks than a lane keeps in registers; k >= T: nothing is removed."""
    w = wl.scaled(wl.WORKLOADS["C1"], window_k=k, tokens=40)
    stats = run_stream(w, wl.make_layer(w), wl.make_inputs(w))
    if k >= 40:
        assert all(s["removed"] == 0 for s in stats)


def test_threshold_extremes_full_and_empty_cache():
    """theta = -inf caches every neuron (num_used = capacity = F: the sparse FFN is the dense FFN);
    theta = +inf caches nothing (y = 0)."""
    from tests.harness import GpuLayer, compare_step, rel_l2
    w = wl.scaled(wl.WORKLOADS["C1"], d_model=128, d_ffn=1096, rank=16, capacity_rows=1096, tokens=3, dtype="f16")
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    for theta in (-np.inf, np.inf):
        L.theta = theta
        gpu = GpuLayer(w, L)
        ora = make_oracle(w, L)
        for t in range(3):
            r = compare_step(gpu, ora, X[t], w, t)
            assert r["n"] == (w.d_ffn if theta < 0 else 0)
        if theta < 0:
            yd = O.dense_ffn(L.w_up, L.w_down, L.b, X[2])
            assert rel_l2(gpu.y[0].cpu().numpy(), yd) <= 1e-3
        else:
            assert not gpu.y.cpu().numpy().any()


@pytest.mark.parametrize("ffn_mode", [0, 1])
@pytest.mark.parametrize("d_model,glu,batch", [(256, False, 5), (264, True, 8), (96, False, 2)])
def test_batched_ffn_over_a_cache_of_many_rows(d_model, glu, batch, ffn_mode):
    """Several tokens over 40000 cached rows (theta = -inf caches every neuron): the chunks of the batched down
    projection are 1536 rows here (three compaction passes each) and 27 of them are in use; d = 264 has a ragged last
    column slice and takes the streaming activation stage (d is no multiple of 32), d = 256 the matrix-core one.
    Checked against the dense FFN per token."""
    from tests.harness import GpuLayer, rel_l2
    F = 40000
    w = wl.scaled(wl.WORKLOADS["C1"], name="many-rows", d_model=d_model, d_ffn=F, rank=8, window_k=2, dtype="f16", glu=glu,
                  tokens=2, batch=batch, capacity_rows=F)
    L = _random_predictor_layer(w, seed=11)
    L.theta = -np.inf
    X = wl.make_batch_inputs(w)
    gpu = GpuLayer(w, L, ffn_mode=ffn_mode)
    lay = gpu.layer
    for t in range(2):
        xd = gpu.upload_x(X[t])
        lay.step(xd, gpu.y, batch=batch)
        st = lay.state()
        assert st["error"] == 0 and st["num_used"] == F
        y = gpu.y.cpu().numpy().astype(np.float64)
        for i in range(batch):
            yd = O.dense_ffn(L.w_up, L.w_down, L.b, X[t][i], w_gate=L.w_gate if glu else None)
            assert rel_l2(y[i], yd) <= 1e-3, (t, i)


def test_maximum_sizes_long_hole_list():
    """F = capacity = 65536 (the largest the window kernel takes), half the neurons flipping per step:
    tens of thousands of holes, so the hole list spills from LDS to the global scratch list."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="max", d_model=32, d_ffn=65536, rank=8, window_k=1, p_active=0.5,
                  rho=0.0, dtype="f16", tokens=4, capacity_rows=65536)
    stats = run_stream(w, wl.make_layer(w), wl.make_inputs(w))
    assert max(s["moved"] for s in stats) > 4096


def _random_predictor_layer(w, seed):
    """A layer with a random (not SVD-derived) predictor: the decomposition of a d = 8192 projection takes half
    a minute on the host and the kernels do not care where A and B come from."""
    rng = np.random.default_rng(seed)
    d, F, r, dt = w.d_model, w.d_ffn, w.rank, w.np_dtype
    g = lambda *shape: rng.standard_normal(shape, dtype=np.float32)
    w_up, w_down = (g(F, d) / np.sqrt(d)).astype(dt), (g(F, d) / np.sqrt(d)).astype(dt)
    w_gate = (g(F, d) / np.sqrt(d)).astype(dt) if w.glu else None
    w_act = w_gate if w.glu else w_up
    b = (-1.4 * np.linalg.norm(w_act.astype(np.float64), axis=1)).astype(np.float32)
    A, B = (g(d, r) / np.sqrt(d)).astype(dt), g(r, F).astype(dt)
    c = np.full(F, -1.4 * np.sqrt(r), np.float32)            # about 8 % of the logits are positive
    parts = ([w_gate] if w.glu else []) + [w_up, w_down]
    return wl.LayerData(w_up, w_down, w_gate, b, A, B, c, 0.0, np.ascontiguousarray(np.concatenate(parts, axis=1)))


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("glu,batch", [(False, 1), (True, 1), (True, 4)])
def test_widest_rows(glu, batch, api):
    """d_model = 8192 in fp16: the largest row the kernels take (16 loads of 16 bytes per lane and vector),
    32 KiB and 48 KiB bundles; batch 4 runs the MFMA activation stage at this width."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="wide", d_model=8192, d_ffn=512, rank=16, window_k=3, p_active=0.08,
                  dtype="f16", glu=glu, tokens=8, batch=batch, capacity_rows=300)
    L = _random_predictor_layer(w, seed=5)
    X = wl.make_inputs(w) if batch == 1 else wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api=api)
    assert np.mean([s["n"] for s in stats]) > 30


def test_capacity_overflow_sets_sticky_error_and_leaves_state():
    from tests.harness import GpuLayer
    import paper_2312_11514_amd as lif
    w = wl.scaled(wl.WORKLOADS["C1"], capacity_rows=96, tokens=40)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    gpu = GpuLayer(w, L)
    lay = gpu.layer
    ora = make_oracle(w, L)
    overflow_at = None
    for t in range(w.tokens):
        xd = gpu.upload_x(X[t])
        before = lay.state()
        try:
            ora.step(X[t])
            ok = True
        except OverflowError:
            ok = False
        lay.step(xd, gpu.y)
        st = lay.state()
        if ok:
            assert st["error"] == 0 and st["num_used"] == ora.cache.num_used and st["step"] == t + 1
        else:
            overflow_at = t
            assert st["error"] == lif.LIF_CAPACITY
            assert st["num_used"] == before["num_used"] and st["step"] == before["step"]
            assert int(lay.n_added.item()) == 0 and int(lay.n_removed.item()) == 0
            break
    assert overflow_at is not None and overflow_at > 0, "workload never overflowed: make capacity smaller"
    # sticky: further calls change nothing; reset clears
    ptr_before = lay.pointers.clone()
    y_before = gpu.y.clone()
    lay.step(gpu.upload_x(X[overflow_at]), gpu.y)
    st2 = lay.state()
    assert st2["error"] == lif.LIF_CAPACITY and st2["step"] == st["step"] and st2["num_used"] == st["num_used"]
    assert torch.equal(ptr_before, lay.pointers) and torch.equal(y_before, gpu.y)
    lay.reset()
    st3 = lay.state()
    assert st3 == dict(num_used=0, step=0, error=0, last_added=0, last_removed=0, last_moved=0, window_len=0)


def test_call_order_and_argument_errors():
    from tests.harness import GpuLayer
    import paper_2312_11514_amd as lif
    w = wl.scaled(wl.WORKLOADS["C1"], tokens=2)
    L = wl.make_layer(w)
    gpu = GpuLayer(w, L)
    lay = gpu.layer
    xd = gpu.upload_x(wl.make_inputs(w)[0])
    with pytest.raises(lif.LifError) as e:
        lay.load_bundles()
    assert e.value.status == lif.LIF_BAD_STATE
    lay.predict(xd)
    lay.update_window()
    with pytest.raises(lif.LifError) as e:
        lay.update_window()
    assert e.value.status == lif.LIF_BAD_STATE
    lay.load_bundles()
    with pytest.raises(lif.LifError) as e:
        lay.sparse_ffn(xd, gpu.y, batch=2)          # max_batch is 1
    assert e.value.status == lif.LIF_INVALID_ARG
    with pytest.raises(lif.LifError) as e:
        lay.predict(None)
    assert e.value.status == lif.LIF_INVALID_ARG
    lay.sparse_ffn(xd, gpu.y)
    assert lay.state()["error"] == 0


def test_reset_reproduces_the_run_bit_for_bit():
    """Two passes over the same stream from an empty cache give identical bytes (fixed summation order)."""
    from tests.harness import GpuLayer
    w = wl.WORKLOADS["C1"]
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    gpu = GpuLayer(w, L)
    xd = gpu.upload_x(X)
    outs = []
    for rep in range(2):
        gpu.layer.reset()
        ys = torch.zeros_like(xd)
        for t in range(w.tokens):
            gpu.layer.step(xd[t], ys[t])
        outs.append((ys.cpu().numpy().tobytes(), gpu.layer.pointers.cpu().numpy().tobytes(), gpu.layer.counters()))
    assert outs[0][0] == outs[1][0] and outs[0][1] == outs[1][1]
    assert outs[0][2]["h2d_bytes"] == outs[1][2]["h2d_bytes"]


@pytest.mark.parametrize("kind", ["single", "batch8-shared-launch", "passes"])
def test_hip_graph_replay_matches_eager(kind):
    """The whole token stream captured once and replayed: every replay equals the eager result (single tokens; batches
    of 8 through the shared load + MFMA launch; speculative passes of 4 tokens with 3 kept)."""
    from tests.harness import GpuLayer
    if kind == "single":
        w = wl.WORKLOADS["C1"]
        X = wl.make_inputs(w)
    elif kind == "batch8-shared-launch":
        w = wl.scaled(wl.WORKLOADS["C1"], name="g8", d_model=608, d_ffn=2200, rank=40, window_k=3, p_active=0.06,
                      dtype="f16", glu=True, tokens=12, batch=8, capacity_rows=2100)
        X = wl.make_batch_inputs(w)
    else:
        w = wl.scaled(wl.WORKLOADS["C1"], name="gp", d_model=256, dtype="f16", tokens=48, batch=4, window_k=5)
        X = wl.make_inputs(w).reshape(12, 4, -1)
    L = wl.make_layer(w)
    gpu = GpuLayer(w, L)
    lay = gpu.layer
    xd = gpu.upload_x(X)
    ys = torch.zeros_like(xd)

    def run():
        lay.reset()
        for t in range(len(X)):
            if kind == "passes":
                lay.step_tokens(xd[t], ys[t], 4, 3)
            else:
                lay.step(xd[t], ys[t], w.batch)
    run()
    torch.cuda.synchronize()
    y_eager, ptr_eager = ys.clone(), lay.pointers.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(3):
        ys.zero_()
        lay.pointers.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        n = lay.state()["num_used"]
        assert torch.equal(ys, y_eager), f"replay {rep}"
        assert torch.equal(lay.pointers[:n], ptr_eager[:n])


def test_c5_stacked_layers_share_the_stream_not_the_state():
    """Stacked OPT-shaped layers (five of the 32, spread over the stack), token-major order as bench.py runs them:
    every layer has its own predictor, window and cache; bytes loaded per token = sum over layers of |added| x
    bundle.  24 tokens: the window is full from the fifth on, so most steps delete, move and append."""
    from tests.harness import GpuLayer, compare_step
    w = wl.WORKLOADS["C5"]
    base = wl.cached_layer("C2")                      # C5 layers have the C2 shape; layer 0 is the C2 layer
    ids = (0, 1, 7, 16, 31)
    Ls = [wl.make_layer_variant(base, w, l) for l in ids]
    assert not np.array_equal(Ls[0].bundles[:64], Ls[1].bundles[:64])
    X = wl.make_inputs(w, tokens=24)
    gpus = [GpuLayer(w, L) for L in Ls]
    oras = [make_oracle(w, L) for L in Ls]
    per_token = []
    for t in range(len(X)):
        print(f"[C5] token {t}", flush=True) if t % 8 == 0 else None
        loaded = 0
        for gpu, ora in zip(gpus, oras):
            before = ora.bytes_loaded
            r = compare_step(gpu, ora, X[t], w, t, check_cache=(t % 4 == 3), api="step")
            loaded += ora.bytes_loaded - before
            assert r["n"] <= w.capacity_rows // 2          # the cache stays far below its cap (half of the FFN rows)
        per_token.append(loaded)
    for gpu, ora in zip(gpus, oras):
        cnt = gpu.layer.counters()
        assert cnt["h2d_bytes"] == ora.bytes_loaded and cnt["rows_moved"] == ora.rows_moved and ora.rows_moved > 0
    assert sum(per_token) == sum(o.bytes_loaded for o in oras)
    assert np.mean(per_token[10:]) < 0.25 * per_token[0]   # steady state loads a small part of what the first token did
    m = [g.layer.step_mask.cpu().numpy() for g in gpus]
    assert all(not np.array_equal(m[i], m[j]) for i in range(len(m)) for j in range(i))


def test_c5_all_32_layers_token_major():
    """All 32 stacked layers (32 handles, 32 pinned stores, 8.6 GB) for the first tokens of the stream, token-major as
    bench.py runs configuration 5, every layer against its own oracle; host-to-device bytes per token = sum over the
    layers of |added| x bundle bytes."""
    from tests.harness import GpuLayer, compare_step
    w = wl.WORKLOADS["C5"]
    base = wl.cached_layer("C2")
    gpus, oras = [], []
    for l in range(w.layers):
        Ll = wl.make_layer_variant(base, w, l)
        gpus.append(GpuLayer(w, Ll))
        oras.append(make_oracle(w, Ll))
        print(f"[C5 x32] layer {l} uploaded", flush=True) if l % 8 == 7 else None
    X = wl.make_inputs(w, tokens=7)
    for t in range(len(X)):
        print(f"[C5 x32] token {t}", flush=True)
        for gpu, ora in zip(gpus, oras):
            compare_step(gpu, ora, X[t], w, t, check_cache=(t == len(X) - 1), api="step")
    h2d = sum(g.layer.counters()["h2d_bytes"] for g in gpus)
    assert h2d == sum(o.bytes_loaded for o in oras) == sum(g.layer.counters()["added"] for g in gpus) * w.bundle_bytes
    assert sum(o.rows_moved for o in oras) == sum(g.layer.counters()["rows_moved"] for g in gpus) > 0
    sizes = [g.layer.state()["num_used"] for g in gpus]
    assert len(set(sizes)) > 8 and max(sizes) <= w.capacity_rows // 2       # every layer its own set, far below the cap


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_row_count_hint_never_changes_results_above_2048_rows(dtype):
    """About 3000 rows in use, one token: a hint above 2048 rows selects compaction passes of 4096 slots (one pass), a
    smaller one or none passes of 2048 (two passes over the single chunk); the output bytes are the same, for both ways
    of driving the layer."""
    from tests.harness import GpuLayer
    w = wl.scaled(wl.WORKLOADS["C1"], name="hint-3000", d_model=256, d_ffn=8192, rank=32, window_k=4, p_active=0.25,
                  dtype=dtype, tokens=10, capacity_rows=8192)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    outs, rows = set(), []
    for hint in (0, 700, 2000, 3300, 9000):
        for api in ("step", "calls"):
            gpu = GpuLayer(w, L)
            if hint:
                gpu.layer.set_expected_rows(hint)
            xd = gpu.upload_x(X)
            y = torch.zeros_like(xd)
            for t in range(len(X)):
                (gpu.layer.step if api == "step" else gpu.layer.step_calls)(xd[t], y[t])
            assert gpu.layer.state()["error"] == 0
            rows.append(gpu.layer.state()["num_used"])
            outs.add(y.cpu().numpy().tobytes())
    assert 2048 < min(rows) and max(rows) <= 4096          # the last step; most of the ten steps are in that range
    assert len(outs) == 1


@pytest.mark.parametrize("glu", [False, True])
def test_row_count_hint_never_changes_results_batched(glu):
    """Eight tokens per step, fp16: the grids of both matrix-core stages are sized from the hint (a smaller grid strides
    over the tiles and chunks, a hint of 2048 rows or more moves lif_step to the shared load + activation launch);
    the output bytes are the same for every hint and for both ways of driving the layer."""
    from tests.harness import GpuLayer
    w = wl.scaled(wl.WORKLOADS["C1"], name="hint-b8", d_model=512, d_ffn=4096, rank=32, window_k=3, p_active=0.1,
                  dtype="f16", glu=glu, tokens=6, batch=8, capacity_rows=4096)
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w)
    outs = set()
    for hint in (0, 16, 900, 5000):
        for api in ("step", "calls"):
            gpu = GpuLayer(w, L)
            if hint:
                gpu.layer.set_expected_rows(hint)
            ys = []
            for t in range(len(X)):
                xd = gpu.upload_x(X[t])
                if api == "step":
                    gpu.layer.step(xd, gpu.y, batch=8)
                else:
                    gpu.layer.step_calls(xd, gpu.y, batch=8)
                ys.append(gpu.y.cpu().numpy().tobytes())
            assert gpu.layer.state()["error"] == 0 and gpu.layer.state()["num_used"] > 600
            outs.add(b"".join(ys))
    assert len(outs) == 1


@pytest.mark.parametrize("hint", [16, 900, 5000])
def test_row_count_hint_never_changes_results(hint):
    """The speculative first pass of the FFN (hint below, near and above the rows in use) gives the same bytes."""
    from tests.harness import GpuLayer
    w = wl.WORKLOADS["C2"]
    L = wl.cached_layer("C2")
    X = wl.make_inputs(w, tokens=12)
    ys = []
    for use_hint in (False, True):
        gpu = GpuLayer(w, L)
        if use_hint:
            gpu.layer.set_expected_rows(hint)
        xd = gpu.upload_x(X)
        y = torch.zeros_like(xd)
        for t in range(len(X)):
            gpu.layer.step(xd[t], y[t])
        ys.append(y.cpu().numpy().tobytes())
        assert gpu.layer.state()["error"] == 0
    assert ys[0] == ys[1]


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("batch", [2, 5, 8])
@pytest.mark.parametrize("glu", [False, True])
@pytest.mark.parametrize("d_model,dtype", [(608, "f16"), (128, "f16"), (568, "f16"), (256, "f32")])
def test_batched_tokens_small_shapes(d_model, dtype, glu, batch, api):
    """Batches of 2..8 tokens sharing one cache.  fp16 with d % 32 == 0 runs the MFMA activation kernel
    (d = 608 = 19 x 32: a k-step count that does not divide by the four waves; capacity and row counts
    not multiples of the 16-row tile); d = 568 and fp32 run the streaming kernel.  api = "step": for the MFMA
    shapes the bundle load runs next to the activation stage of the surviving rows and the rows it wrote
    are computed in a second pass."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="batched", d_model=d_model, d_ffn=1096, rank=40, window_k=3,
                  p_active=0.06, dtype=dtype, glu=glu, tokens=10, batch=batch, capacity_rows=1003)
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api=api)
    assert np.mean([s["n"] for s in stats]) > 100
    if api == "step" and dtype == "f16" and d_model % 32 == 0:
        # the same stream with a row-count hint large enough for the shared load + activation launch
        from tests.harness import GpuLayer, compare_step
        gpu = GpuLayer(w, L)
        gpu.layer.set_expected_rows(4096)
        ora = make_oracle(w, L)
        for t in range(len(X)):
            compare_step(gpu, ora, X[t], w, t, api="step")


def test_fused_step_equals_four_calls_bit_for_bit():
    """lif_step (cache update and activations in one launch) and the four separate calls give identical
    bytes everywhere: y, masks, pointers, bias, cache rows (the loaders sum in the activation kernel's order)."""
    from tests.harness import GpuLayer
    for name, tokens in (("C2", 40), ("C4", 16)):
        w = wl.WORKLOADS[name]
        L = wl.cached_layer(name)
        X = wl.make_inputs(w, tokens=tokens)
        res = []
        for api in ("calls", "step"):
            gpu = GpuLayer(w, L)
            lay = gpu.layer
            xd = gpu.upload_x(X)
            y = torch.zeros_like(xd)
            for t in range(tokens):
                (lay.step if api == "step" else lay.step_calls)(xd[t], y[t])
            n = lay.state()["num_used"]
            res.append((y.cpu().numpy().astype(np.float64), lay.pointers[:n].cpu().numpy().tobytes(),
                        lay.bias[:n].cpu().numpy().tobytes(), lay.matrix[:n].cpu().numpy().tobytes(),
                        lay.masks.cpu().numpy().tobytes(), lay.counters()))
        for a, b in zip(res[0][1:5], res[1][1:5]):
            assert a == b, name
        assert res[0][0].tobytes() == res[1][0].tobytes(), name
        ca, cb = res[0][5], res[1][5]
        assert ca["h2d_bytes"] == cb["h2d_bytes"] and ca["rows_moved"] == cb["rows_moved"]


def test_fused_step_equals_four_calls_bit_for_bit_batched():
    """Batch of 8 tokens (MFMA activation stage): lif_step overlaps the bundle load with the activations of the
    surviving rows and recomputes the slots the load wrote; every output byte equals the four separate calls."""
    from tests.harness import GpuLayer
    w = wl.scaled(wl.WORKLOADS["C1"], name="batched", d_model=608, d_ffn=2200, rank=40, window_k=3, p_active=0.06,
                  dtype="f16", glu=True, tokens=14, batch=8, capacity_rows=2100)   # >= 2048 rows: the shared launch is used
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w)
    res = []
    for api in ("calls", "step"):
        gpu = GpuLayer(w, L)
        lay = gpu.layer
        xd = gpu.upload_x(X)
        y = torch.zeros_like(xd)
        for t in range(w.tokens):
            (lay.step if api == "step" else lay.step_calls)(xd[t], y[t], w.batch)
        n = lay.state()["num_used"]
        res.append((y.cpu().numpy().tobytes(), lay.pointers[:n].cpu().numpy().tobytes(),
                    lay.matrix[:n].cpu().numpy().tobytes(), lay.masks.cpu().numpy().tobytes()))
        assert n > 300 and lay.counters()["rows_moved"] > 0
    assert res[0] == res[1]


@pytest.mark.parametrize("api", ["calls", "step"])
def test_dynamic_window_shrinks_instead_of_overflowing(api):
    """shrink_window = 1 with a capacity the fixed window overflows: the oldest masks leave the window,
    ids / cache layout / outputs still match the oracle step by step, and the window length is reported."""
    from tests.harness import GpuLayer, compare_step
    w = wl.scaled(wl.WORKLOADS["C1"], capacity_rows=96, tokens=48, window_k=6)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    gpu = GpuLayer(w, L, shrink=True)
    ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu, L.A, L.B, L.c, L.theta, L.b,
                        L.bundles, shrink=True)
    lens = []
    for t in range(w.tokens):
        compare_step(gpu, ora, X[t], w, t, api=api)
        st = gpu.layer.state()
        assert st["window_len"] == len(ora.window.masks)
        assert st["num_used"] <= w.capacity_rows
        lens.append(st["window_len"])
    assert min(lens[6:]) < w.window_k, "capacity never bound: the test does not exercise the shrink"
    assert gpu.layer.counters()["h2d_bytes"] == ora.bytes_loaded


def test_dynamic_window_single_mask_above_capacity_is_an_error():
    from tests.harness import GpuLayer
    import paper_2312_11514_amd as lif
    w = wl.scaled(wl.WORKLOADS["C1"], capacity_rows=8, tokens=4)
    L = wl.make_layer(w)
    gpu = GpuLayer(w, L, shrink=True)
    gpu.layer.step(gpu.upload_x(wl.make_inputs(w)[0]), gpu.y)      # ~50 predicted neurons > 8 rows
    st = gpu.layer.state()
    assert st["error"] == lif.LIF_CAPACITY and st["num_used"] == 0 and st["step"] == 0


def test_n1_dynamic_window_at_opt_shape():
    """The dynamic-window workload bench.py can run (OPT shape, 10 % activity, k = 8, cache = 25 % of the rows)."""
    from tests.harness import GpuLayer, compare_step
    w = wl.WORKLOADS["N1"]
    L = wl.make_layer(w)
    X = wl.make_inputs(w, tokens=48)
    gpu = GpuLayer(w, L)
    ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu, L.A, L.B, L.c, L.theta, L.b,
                        L.bundles, shrink=True)
    lens = []
    for t in range(len(X)):
        compare_step(gpu, ora, X[t], w, t, check_cache=(t % 4 == 3), api="step")
        lens.append(gpu.layer.state()["window_len"])
        assert lens[-1] == len(ora.window.masks)
    assert min(lens[8:]) < w.window_k


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("glu,dtype,d_model", [(False, "f16", 256), (True, "f16", 608), (False, "f32", 256)])
def test_speculative_verify_passes_token_granular_window(glu, dtype, d_model, api):
    """Passes of lambda + 1 = 5 consecutive tokens with a varying number of kept tokens (Section 4.3): per-token
    masks, window entries per token, transient masks leaving with the next pass, FFN for all five tokens."""
    from tests.harness import GpuLayer, rel_l2, REL_L2_TOL
    w = wl.scaled(wl.WORKLOADS["C1"], name="spec", d_model=d_model, d_ffn=1024, rank=32, window_k=4, dtype=dtype,
                  glu=glu, tokens=60, batch=5, capacity_rows=1024)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)                                           # one stream; a pass takes 5 consecutive tokens
    gpu = GpuLayer(w, L, max_batch=5)
    lay = gpu.layer
    ora = make_oracle(w, L)
    keeps = [5, 3, 0, 1, 5, 2, 4, 5, 0, 0, 3, 5]
    for p, keep in enumerate(keeps):
        xb = X[5 * p:5 * p + 5]
        ref = ora.step_tokens(xb, keep)
        xd = gpu.upload_x(xb)
        if api == "step":
            lay.step_tokens(xd, gpu.y, 5, keep)                     # the whole pass in one call
        else:
            lay.predict(xd, 5)
            lay.update_window_tokens(5, keep)
            lay.load_bundles()
            lay.sparse_ffn(xd, gpu.y, 5)
        na, nr = int(lay.n_added.item()), int(lay.n_removed.item())
        assert lay.added[:na].cpu().numpy().tolist() == ref["added"].tolist(), f"pass {p}"
        assert lay.removed[:nr].cpu().numpy().tolist() == ref["removed"].tolist(), f"pass {p}"
        st = lay.state()
        n = ref["num_used"]
        assert st["error"] == 0 and st["num_used"] == n and st["window_len"] == len(ora.window.masks)
        assert (lay.masks[:5].cpu().numpy() == O.pack_mask(ref["masks"])).all()
        assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all()
        assert lay.matrix[:n].cpu().numpy().tobytes() == ora.cache.matrix[:n].tobytes()
        assert rel_l2(gpu.y[:5].cpu().numpy(), ref["y"]) <= REL_L2_TOL
    assert lay.counters()["h2d_bytes"] == ora.bytes_loaded
    # passes of a single token, kept or not (the one-token form of the same call)
    for i, keep in enumerate([0, 1, 0]):
        xb = X[50 + i:51 + i]
        ref = ora.step_tokens(xb, keep)
        xd = gpu.upload_x(xb)
        if api == "step":
            lay.step_tokens(xd, gpu.y, 1, keep)
        else:
            lay.predict(xd, 1)
            lay.update_window_tokens(1, keep)
            lay.load_bundles()
            lay.sparse_ffn(xd, gpu.y, 1)
        n = ref["num_used"]
        assert lay.state()["num_used"] == n and lay.state()["window_len"] == len(ora.window.masks)
        assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all()
        assert rel_l2(gpu.y[:1].cpu().numpy(), ref["y"]) <= REL_L2_TOL
    # mixing with ordinary single-token steps on the same layer
    from tests.harness import compare_step
    w1 = wl.scaled(w, batch=1)
    for t in range(4):
        x = X[55 + t]
        ref = ora.step(x)
        xd = gpu.upload_x(x)
        lay.step(xd, gpu.y, 1)
        assert lay.state()["num_used"] == ref["num_used"]
        assert rel_l2(gpu.y[0].cpu().numpy(), ref["y"]) <= REL_L2_TOL


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("k,dtype,d_model,glu,cap", [(4, "f16", 256, False, 145), (6, "f16", 608, True, 135),
                                                     (12, "f32", 132, False, 230)])
def test_dynamic_window_with_speculative_passes(k, dtype, d_model, glu, cap, api):
    """Passes of several tokens with shrink_window = 1 and a capacity that the fixed window overflows: the oldest
    window masks leave until the masks of the pass and the rest fit; a pass whose own masks do not fit sets the
    error on both sides and leaves everything unchanged."""
    from tests.harness import GpuLayer, rel_l2, REL_L2_TOL
    import paper_2312_11514_amd as lif
    w = wl.scaled(wl.WORKLOADS["C1"], name="specshrink", d_model=d_model, d_ffn=1024, rank=32, window_k=k,
                  dtype=dtype, glu=glu, tokens=80, batch=5, capacity_rows=cap, p_active=0.05)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    gpu = GpuLayer(w, L, max_batch=5, shrink=True)
    lay = gpu.layer
    ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu, L.A, L.B, L.c, L.theta, L.b,
                        L.bundles, shrink=True)
    keeps = [5, 4, 5, 3, 0, 1, 5, 5, 2, 4, 5, 0, 5, 5, 3, 5]
    lens, pos = [], 0
    for p, keep in enumerate(keeps):
        ntok = 5 if p % 4 != 3 else 2                            # passes of different lengths
        keep = min(keep, ntok)
        xb = X[pos:pos + ntok]
        pos += ntok
        ref = ora.step_tokens(xb, keep)
        xd = gpu.upload_x(xb)
        if api == "step":
            lay.step_tokens(xd, gpu.y, ntok, keep)
        else:
            lay.predict(xd, ntok)
            lay.update_window_tokens(ntok, keep)
            lay.load_bundles()
            lay.sparse_ffn(xd, gpu.y, ntok)
        na, nr = int(lay.n_added.item()), int(lay.n_removed.item())
        assert lay.added[:na].cpu().numpy().tolist() == ref["added"].tolist(), f"pass {p}"
        assert lay.removed[:nr].cpu().numpy().tolist() == ref["removed"].tolist(), f"pass {p}"
        n = ref["num_used"]
        st = lay.state()
        assert st["error"] == 0 and st["num_used"] == n <= w.capacity_rows
        assert st["window_len"] == len(ora.window.masks), f"pass {p}"
        assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all()
        assert lay.matrix[:n].cpu().numpy().tobytes() == ora.cache.matrix[:n].tobytes()
        assert rel_l2(gpu.y[:ntok].cpu().numpy(), ref["y"]) <= REL_L2_TOL
        lens.append((st["window_len"], min(k, sum(min(q, 5) for q in keeps[:p + 1]))))
    assert any(a < b for a, b in lens[3:]), "capacity never bound: the test does not exercise the shrink"
    assert lay.counters()["h2d_bytes"] == ora.bytes_loaded and ora.min_margin > 1e-9
    # a pass whose own masks exceed the capacity: error, nothing changes (theta = -inf is not available per call, so
    # a second layer with a tiny capacity takes the same pass)
    w2 = wl.scaled(w, capacity_rows=40)
    gpu2 = GpuLayer(w2, L, max_batch=5, shrink=True)
    ora2 = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, 40, w.glu, L.A, L.B, L.c, L.theta, L.b, L.bundles, shrink=True)
    with pytest.raises(OverflowError):
        ora2.step_tokens(X[:5], 5)
    xd = gpu2.upload_x(X[:5])
    if api == "step":
        gpu2.layer.step_tokens(xd, gpu2.y, 5, 5)
    else:
        gpu2.layer.predict(xd, 5)
        gpu2.layer.update_window_tokens(5, 5)
    st = gpu2.layer.state()
    assert st["error"] == lif.LIF_CAPACITY and st["num_used"] == 0 and st["step"] == 0 and st["window_len"] == 0


def test_n2_speculative_passes_at_opt_shape():
    """The speculative workload bench.py can run (OPT shape; passes of 5 consecutive tokens, 4 kept, the next pass starts
    after the kept ones), in its launch configuration (lif_step_tokens)."""
    from tests.harness import GpuLayer, rel_l2, max_abs_excess, REL_L2_TOL, MAX_ABS_TOL
    w = wl.WORKLOADS["N2"]
    L = wl.cached_layer("C2")                               # N2 runs on the C2 layer
    X = wl.make_inputs(w, tokens=4 * 16 + 5)
    gpu = GpuLayer(w, L)
    lay = gpu.layer
    ora = make_oracle(w, L)
    for p in range(16):
        xb = X[p * w.spec_keep:p * w.spec_keep + w.batch]
        ref = ora.step_tokens(xb, w.spec_keep)
        lay.step_tokens(gpu.upload_x(xb), gpu.y, w.batch, w.spec_keep)
        na, nr = int(lay.n_added.item()), int(lay.n_removed.item())
        assert lay.added[:na].cpu().numpy().tolist() == ref["added"].tolist(), f"pass {p}"
        assert lay.removed[:nr].cpu().numpy().tolist() == ref["removed"].tolist(), f"pass {p}"
        n = ref["num_used"]
        st = lay.state()
        assert st["error"] == 0 and st["num_used"] == n and st["window_len"] == len(ora.window.masks)
        assert (lay.masks[:w.batch].cpu().numpy() == O.pack_mask(ref["masks"])).all()
        if p % 4 == 3:
            assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all()
            assert lay.matrix[:n].cpu().numpy().tobytes() == ora.cache.matrix[:n].tobytes()
        y = gpu.y[:w.batch].cpu().numpy()
        assert rel_l2(y, ref["y"]) <= REL_L2_TOL and max_abs_excess(y, ref["y"])[0] <= MAX_ABS_TOL
    assert lay.counters()["h2d_bytes"] == ora.bytes_loaded and ora.min_margin > 1e-9 and n > 1000


# ----------------------------------------------------------------------------- resident gate as predictor
@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("ffn_mode", [0, 1])
@pytest.mark.parametrize("dtype,d_model", [("f16", 568), ("f16", 256), ("f32", 256)])
def test_gate_predictor_small_shapes(dtype, d_model, ffn_mode, api):
    """Gate projection resident in HBM as the predictor; bundles = up | down (two vectors)."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="gate", d_model=d_model, d_ffn=1096, rank=8, window_k=3,
                  p_active=0.08, dtype=dtype, glu=True, gate_resident=True, tokens=24, capacity_rows=700)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    stats = run_stream(w, L, X, ffn_mode, api=api)
    assert any(s["moved"] > 0 for s in stats) and any(s["removed"] > 0 for s in stats)
    # exact predictor: the sparse output is the dense gated FFN
    from tests.harness import GpuLayer, rel_l2
    gpu = GpuLayer(w, L, ffn_mode=ffn_mode)
    for x in X[:6]:
        gpu.layer.step(gpu.upload_x(x), gpu.y, 1)
        dense = O.dense_ffn(L.w_up, L.w_down, L.b, x, w_gate=L.w_gate)
        assert rel_l2(gpu.y[0].cpu().numpy(), dense) <= 1e-3


def test_n4_llama_shape_gate_predictor():
    """Llama-2-7B FFN shape with the gate resident, the launch configuration bench.py times for N4."""
    w = wl.WORKLOADS["N4"]
    L = wl.cached_layer("N4")
    X = wl.make_inputs(w, tokens=64)
    stats = run_stream(w, L, X, check_every=8, api="step")
    print("N4 max rel-L2 %.2e, rows %.0f" % (max(s["err"] for s in stats), np.mean([s["n"] for s in stats[10:]])))


def test_gate_predictor_rejects_gated_bundles():
    from tests.harness import GpuLayer
    w = wl.scaled(wl.WORKLOADS["C1"], name="gate", glu=True, gate_resident=True, tokens=2)
    L = wl.make_layer(w)
    import paper_2312_11514_amd as lif
    with pytest.raises(lif.LifError):
        lif.Layer(d_model=w.d_model, d_ffn=w.d_ffn, rank=8, window_k=2, capacity_rows=64, glu=True, dtype="f32",
                  predictor=lif.PRED_GATE, A=torch.zeros(8, device="cuda"), B=None, c=None,
                  b=torch.zeros(8, device="cuda"), host_bundles=torch.zeros(8).pin_memory())
    gpu = GpuLayer(w, L)
    x2 = gpu.upload_x(np.stack([wl.make_inputs(w)[0]] * 2))
    with pytest.raises(lif.LifError):
        gpu.layer.predict(x2, 2)                      # max_batch is 1


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("batch", [2, 5, 8])
@pytest.mark.parametrize("dtype,d_model", [("f16", 608), ("f16", 568), ("f32", 256)])
def test_gate_predictor_batched_tokens(dtype, d_model, batch, api):
    """The resident gate as predictor for batches of tokens: per-token masks and gate activations, step mask = OR,
    one row of y per token over the shared cache (fp16, d % 32 == 0: MFMA activation stage; otherwise the streaming
    kernel).  Exact predictor: every row of y is also the dense gated FFN of its token."""
    from tests.harness import GpuLayer, compare_step, rel_l2
    w = wl.scaled(wl.WORKLOADS["C1"], name="gateb", d_model=d_model, d_ffn=1096, rank=8, window_k=3, p_active=0.05,
                  dtype=dtype, glu=True, gate_resident=True, tokens=10, batch=batch, capacity_rows=1003)
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api=api)
    assert np.mean([s["n"] for s in stats]) > 80 and any(s["moved"] > 0 for s in stats)
    gpu = GpuLayer(w, L)
    gpu.layer.set_expected_rows(4096)                 # fp16, d % 32 == 0: the shared load + activation launch of lif_step
    ora = make_oracle(w, L)
    for t in range(4):
        compare_step(gpu, ora, X[t], w, t, api=api)
        for bt in range(batch):
            dense = O.dense_ffn(L.w_up, L.w_down, L.b, X[t][bt], w_gate=L.w_gate)
            assert rel_l2(gpu.y[bt].cpu().numpy(), dense) <= 1e-3


@pytest.mark.parametrize("api", ["calls", "step"])
def test_gate_predictor_speculative_passes(api):
    """Passes of five consecutive tokens with the resident gate as predictor (Section 4.3 with the Appendix's
    alternative predictor): token-granular window, transient masks, FFN rows for all five tokens."""
    from tests.harness import GpuLayer, rel_l2, REL_L2_TOL
    w = wl.scaled(wl.WORKLOADS["C1"], name="gatespec", d_model=608, d_ffn=1024, rank=8, window_k=4, dtype="f16",
                  glu=True, gate_resident=True, tokens=45, batch=5, capacity_rows=1024, p_active=0.05)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    gpu = GpuLayer(w, L, max_batch=5)
    lay = gpu.layer
    ora = make_oracle(w, L)
    for p, keep in enumerate([5, 3, 0, 1, 5, 2, 4, 0, 5]):
        xb = X[5 * p:5 * p + 5]
        ref = ora.step_tokens(xb, keep)
        xd = gpu.upload_x(xb)
        if api == "step":
            lay.step_tokens(xd, gpu.y, 5, keep)
        else:
            lay.predict(xd, 5)
            lay.update_window_tokens(5, keep)
            lay.load_bundles()
            lay.sparse_ffn(xd, gpu.y, 5)
        na, nr = int(lay.n_added.item()), int(lay.n_removed.item())
        assert lay.added[:na].cpu().numpy().tolist() == ref["added"].tolist(), f"pass {p}"
        assert lay.removed[:nr].cpu().numpy().tolist() == ref["removed"].tolist(), f"pass {p}"
        n = ref["num_used"]
        st = lay.state()
        assert st["error"] == 0 and st["num_used"] == n and st["window_len"] == len(ora.window.masks)
        assert (lay.masks[:5].cpu().numpy() == O.pack_mask(ref["masks"])).all()
        assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all()
        assert rel_l2(gpu.y[:5].cpu().numpy(), ref["y"]) <= REL_L2_TOL
    assert ora.min_margin > 1e-9 and lay.counters()["h2d_bytes"] == ora.bytes_loaded


# ----------------------------------------------------------------------------- seeded random configurations
def _random_config(i):
    rng = np.random.default_rng(9000 + i)
    dtype = ["f16", "f32"][int(rng.integers(2))]
    ve = 8 if dtype == "f16" else 4
    d = int(rng.integers(2, 90)) * ve                      # ragged vector counts, below and above one wave of 16-byte loads
    F = int(rng.integers(8, 400)) * 8
    batch = int([1, 1, 1, 2, 3, 8][int(rng.integers(6))])
    glu = bool(rng.integers(2))
    k = int(rng.integers(1, 10))
    p = float(rng.uniform(0.02, 0.2))
    shrink = bool(rng.integers(2)) and batch == 1
    cap = F if not shrink else max(int(F * p * 2.5), 16)
    r = int(rng.integers(1, 6)) * ve
    return wl.scaled(wl.WORKLOADS["C1"], name=f"rand{i}", d_model=d, d_ffn=F, rank=min(r, d), window_k=k, p_active=p,
                     rho=float(rng.uniform(0.0, 0.95)), dtype=dtype, glu=glu, tokens=14, batch=batch,
                     capacity_rows=cap, shrink=shrink)


@pytest.mark.parametrize("i", range(60))
def test_seeded_random_configurations(i):
    """Shapes, window sizes, activity levels, batch sizes, dtypes and the dynamic window drawn from a seeded
    generator: every step of both APIs against the oracle (a single mask above the capacity ends the stream
    with the same error on both sides)."""
    from tests.harness import GpuLayer, compare_step
    w = _random_config(i)
    L = wl.make_layer(w)
    X = wl.make_inputs(w) if w.batch == 1 else wl.make_batch_inputs(w)
    for api in ("calls", "step"):
        gpu = GpuLayer(w, L, ffn_mode=i % 2)
        ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu, L.A, L.B, L.c, L.theta, L.b,
                            L.bundles, shrink=w.shrink)
        for t in range(len(X)):
            try:
                compare_step(gpu, ora, X[t], w, t, api=api)
            except OverflowError:
                # the oracle refused the step (its mask alone is above the capacity): the device reports the same
                xd = gpu.upload_x(X[t])
                (gpu.layer.step if api == "step" else gpu.layer.step_calls)(xd, gpu.y, w.batch)
                assert gpu.layer.state()["error"] == 3
                break
        assert ora.min_margin > 1e-9


@pytest.mark.parametrize("i", range(16))
def test_seeded_random_speculative_passes(i):
    """Token-granular window updates on seeded random shapes, pass lengths and keep counts (both APIs)."""
    from tests.harness import GpuLayer, rel_l2, REL_L2_TOL
    rng = np.random.default_rng(7000 + i)
    dtype = ["f16", "f32"][int(rng.integers(2))]
    ve = 8 if dtype == "f16" else 4
    ntok = int(rng.integers(2, 9))
    w = wl.scaled(wl.WORKLOADS["C1"], name=f"spec{i}", d_model=int(rng.integers(2, 80)) * ve,
                  d_ffn=int(rng.integers(2, 40)) * 64, rank=2 * ve, window_k=int(rng.integers(1, 8)),
                  p_active=float(rng.uniform(0.02, 0.12)), dtype=dtype, glu=bool(rng.integers(2)),
                  tokens=ntok * 10, batch=ntok)
    shrink = i % 2 == 1                                  # odd cases: dynamic window with a capacity that binds
    w = wl.scaled(w, capacity_rows=max(16, int(w.d_ffn * w.p_active * (ntok + 1.5))) if shrink else w.d_ffn)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    keeps = [int(rng.integers(0, ntok + 1)) for _ in range(10)]
    for api in ("calls", "step"):
        gpu = GpuLayer(w, L, max_batch=ntok, shrink=shrink)
        lay = gpu.layer
        ora = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu, L.A, L.B, L.c, L.theta, L.b,
                            L.bundles, shrink=shrink)
        for p, keep in enumerate(keeps):
            xb = X[ntok * p:ntok * (p + 1)]
            xd = gpu.upload_x(xb)
            try:
                ref = ora.step_tokens(xb, keep)
            except OverflowError:
                # the masks of the pass alone exceed the capacity: the device reports the same and stops
                lay.step_tokens(xd, gpu.y, ntok, keep)
                assert lay.state()["error"] == 3
                break
            if api == "step":
                lay.step_tokens(xd, gpu.y, ntok, keep)
            else:
                lay.predict(xd, ntok)
                lay.update_window_tokens(ntok, keep)
                lay.load_bundles()
                lay.sparse_ffn(xd, gpu.y, ntok)
            na, nr = int(lay.n_added.item()), int(lay.n_removed.item())
            assert lay.added[:na].cpu().numpy().tolist() == ref["added"].tolist(), f"pass {p}"
            assert lay.removed[:nr].cpu().numpy().tolist() == ref["removed"].tolist(), f"pass {p}"
            n = ref["num_used"]
            st = lay.state()
            assert st["error"] == 0 and st["num_used"] == n and st["window_len"] == len(ora.window.masks)
            assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all()
            assert lay.matrix[:n].cpu().numpy().tobytes() == ora.cache.matrix[:n].tobytes()
            assert rel_l2(gpu.y[:ntok].cpu().numpy(), ref["y"]) <= REL_L2_TOL
        assert ora.min_margin > 1e-9


# ----------------------------------------------------------------------------- advertised paths: ranks, offsets, thresholds, widths
LOGIT_07, LOGIT_04 = float(np.log(0.7 / 0.3)), float(np.log(0.4 / 0.6))     # sigmoid thresholds 0.7 and 0.4 as logits


@pytest.mark.parametrize("batch", [1, 4, 8])
@pytest.mark.parametrize("rank,dtype", [(512, "f16"), (768, "f16"), (1024, "f16"), (1152, "f16"), (2048, "f16"),
                                        (1024, "f32"), (2048, "f32")])
def test_predictor_ranks_of_the_papers_last_layers(rank, dtype, batch):
    """Predictor ranks above 256 (Appendix: 1024 for the last four OPT layers, 1152 for Falcon and Persimmon):
    the mask kernel's loop over further rank groups, and the token tiles the host picks from the LDS limit
    (rank 768 at batch 8 asks for the most LDS)."""
    w = wl.scaled(wl.WORKLOADS["C1"], name=f"rank{rank}", d_model=256, d_ffn=1096, rank=rank, window_k=3,
                  p_active=0.08, dtype=dtype, tokens=6, batch=batch, capacity_rows=1096)
    L = _random_predictor_layer(w, seed=rank + batch)
    X = wl.make_inputs(w) if batch == 1 else wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api="calls" if rank % 1024 else "step")
    assert np.mean([s["n"] for s in stats]) > 40


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("batch", [1, 3])
def test_predictor_without_offset(batch, api):
    """c = NULL: logits are (x A) B alone (about half the neurons are predicted)."""
    from tests.harness import GpuLayer, compare_step
    w = wl.scaled(wl.WORKLOADS["C1"], name="noc", d_model=128, d_ffn=520, rank=24, window_k=2, dtype="f16",
                  tokens=8, batch=batch, capacity_rows=520)
    L = wl.make_layer(w)
    L.c = None
    X = wl.make_inputs(w) if batch == 1 else wl.make_batch_inputs(w)
    gpu = GpuLayer(w, L, use_c=False)
    ora = make_oracle(w, L)
    for t in range(len(X)):
        r = compare_step(gpu, ora, X[t], w, t, api=api)
    assert 150 < r["n"] <= 520 and ora.min_margin > 1e-9


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("theta", [LOGIT_07, LOGIT_04])
@pytest.mark.parametrize("kind", ["lowrank-f16", "lowrank-f32-batch4", "gate-f16", "gate-f32"])
def test_finite_nonzero_thresholds(kind, theta, api):
    """theta = logit(0.7) and logit(0.4) (Appendix: sigmoid thresholds of the trained predictors), carried as
    fp32 through the ABI, for the low-rank and the gate predictor."""
    gate = kind.startswith("gate")
    dtype = "f32" if "f32" in kind else "f16"
    batch = 4 if "batch4" in kind else 1
    w = wl.scaled(wl.WORKLOADS["C1"], name=kind, d_model=264 if dtype == "f16" else 132, d_ffn=1096, rank=40,
                  window_k=3, p_active=0.1, dtype=dtype, glu=gate, gate_resident=gate, tokens=12, batch=batch,
                  capacity_rows=1096)
    L = wl.make_layer(w)
    L.theta = theta
    if not gate:
        L.c = (L.c * 0.5).astype(np.float32)         # logits of both signs around the threshold
    X = wl.make_inputs(w) if batch == 1 else wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api=api)
    assert np.mean([s["n"] for s in stats]) > 20


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("variant", ["plain", "gated", "gate-predictor", "batch4"])
@pytest.mark.parametrize("d_model,dtype", [(2048, "f16"), (2560, "f16"), (5120, "f16"), (1024, "f32"), (1288, "f32")])
def test_row_widths_between_the_benchmark_shapes(d_model, dtype, variant, api):
    """d_model 2048, 2560 (Phi-2) and 5120 in fp16, 1024 and 1288 in fp32: 4, 5/6 and 10/12 loads of 16 bytes per
    lane and vector, the kernel instantiations that the benchmark shapes (1, 2, 8, 9, 16 loads) do not use."""
    gate = variant == "gate-predictor"
    batch = 4 if variant == "batch4" else 1
    w = wl.scaled(wl.WORKLOADS["C1"], name=f"w{d_model}", d_model=d_model, d_ffn=512, rank=16, window_k=3,
                  p_active=0.08, dtype=dtype, glu=(variant != "plain" and variant != "batch4"), gate_resident=gate,
                  tokens=6, batch=batch, capacity_rows=300)
    L = _random_predictor_layer(wl.scaled(w, gate_resident=False), seed=d_model)
    if gate:                                             # bundles without the gate row; the gate stays resident
        L.bundles = np.ascontiguousarray(np.concatenate([L.w_up, L.w_down], axis=1))
    X = wl.make_inputs(w) if batch == 1 else wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api=api)
    assert np.mean([s["n"] for s in stats]) > 20


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("batch", [6, 7])
@pytest.mark.parametrize("d_model,dtype,glu", [(608, "f16", True), (568, "f16", False), (256, "f32", False)])
def test_batches_of_six_and_seven_tokens(d_model, dtype, glu, batch, api):
    w = wl.scaled(wl.WORKLOADS["C1"], name="batched", d_model=d_model, d_ffn=1096, rank=40, window_k=3,
                  p_active=0.06, dtype=dtype, glu=glu, tokens=8, batch=batch, capacity_rows=1003)
    run_stream(w, wl.make_layer(w), wl.make_batch_inputs(w), api=api)


def test_rejected_step_leaves_device_buffers_untouched():
    """lif_step checks every argument and the call order before its first launch: a rejected call changes neither
    the masks nor the state."""
    from tests.harness import GpuLayer
    import paper_2312_11514_amd as lif
    import ctypes as C
    w = wl.scaled(wl.WORKLOADS["C1"], tokens=3)
    L = wl.make_layer(w)
    gpu = GpuLayer(w, L)
    lay = gpu.layer
    X = gpu.upload_x(wl.make_inputs(w))
    lay.step(X[0], gpu.y)
    torch.cuda.synchronize()
    snap = lambda: (lay.masks.clone(), lay.step_mask.clone(), lay.added.clone(), lay.state(), lay.counters())
    before = snap()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: C.c_void_p(t.data_ptr())
    args = lambda y: (lay.handle, p(X[1]), 1, y, p(lay.masks), p(lay.step_mask), p(lay.added), p(lay.n_added),
                      p(lay.removed), p(lay.n_removed), st)
    assert lay.lib.lif_step(*args(C.c_void_p(0))) == lif.LIF_INVALID_ARG                   # y is null
    assert lay.lib.lif_step(*args(C.c_void_p(gpu.y.data_ptr() + 2))) == lif.LIF_INVALID_ARG   # y misaligned
    lay.predict(X[1])
    lay.update_window()                                                                   # a window update is pending
    mid = snap()
    assert lay.lib.lif_step(*args(p(gpu.y))) == lif.LIF_BAD_STATE
    assert lay.lib.lif_step_tokens(lay.handle, p(X[1]), 1, 2, p(gpu.y), p(lay.masks), p(lay.step_mask), p(lay.added),
                                   p(lay.n_added), p(lay.removed), p(lay.n_removed), st) == lif.LIF_INVALID_ARG
    torch.cuda.synchronize()
    after = snap()
    for a, b in zip(mid, after):
        assert (torch.equal(a, b) if isinstance(a, torch.Tensor) else a == b)
    assert before[3]["step"] + 1 == after[3]["step"]
    lay.load_bundles()
    lay.sparse_ffn(X[1], gpu.y)
    assert lay.state()["error"] == 0


@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("glu,dtype,d_model,batch", [(False, "f16", 568, 1), (True, "f16", 568, 1), (False, "f32", 264, 1),
                                                     (False, "f16", 4096, 1), (True, "f16", 608, 5), (True, "f32", 132, 3)])
def test_store_that_is_not_bundled_gives_the_same_cache(glu, dtype, d_model, batch, api):
    """host_down set: up (and gate) rows and down columns sit in two separate pinned arrays and every new neuron
    costs two reads (the layout Section 3.2 replaces).  Cache rows, ids and outputs are those of the bundled store."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="unbundled", d_model=d_model, d_ffn=1096 if d_model < 4096 else 512, rank=40,
                  window_k=3, p_active=0.08, dtype=dtype, glu=glu, tokens=10, batch=batch, capacity_rows=700)
    L = wl.make_layer(w) if d_model < 4096 else _random_predictor_layer(w, seed=3)
    X = wl.make_inputs(w) if batch == 1 else wl.make_batch_inputs(w)
    stats = run_stream(w, L, X, api=api, unbundled=True)
    assert any(s["moved"] > 0 for s in stats)


@pytest.mark.parametrize("pairs", [1, 7, 64])
def test_loader_pairs_never_change_results(pairs):
    from tests.harness import GpuLayer
    w = wl.WORKLOADS["C2"]
    L = wl.cached_layer("C2")
    X = wl.make_inputs(w, tokens=10)
    out = []
    for p in (0, pairs):
        gpu = GpuLayer(w, L)
        gpu.layer.set_loader_pairs(p)
        xd = gpu.upload_x(X)
        y = torch.zeros_like(xd)
        for t in range(len(X)):
            gpu.layer.step(xd[t], y[t])
        n = gpu.layer.state()["num_used"]
        out.append((y.cpu().numpy().tobytes(), gpu.layer.matrix[:n].cpu().numpy().tobytes(),
                    gpu.layer.pointers[:n].cpu().numpy().tobytes()))
    assert out[0] == out[1]
    with pytest.raises(Exception):
        gpu.layer.set_loader_pairs(65)


# ----------------------------------------------------------------------------- degenerate sizes and inputs
@pytest.mark.parametrize("api", ["calls", "step"])
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_smallest_shapes(dtype, api):
    """The smallest layer the ABI takes: one 16-byte vector per row, eight neurons, a predictor of one vector, a cache
    of a single row (the predictor offset lets exactly one neuron fire), window 1."""
    from tests.harness import GpuLayer, compare_step
    ve = 8 if dtype == "f16" else 4
    w = wl.scaled(wl.WORKLOADS["C1"], name="min", d_model=ve, d_ffn=8, rank=ve, window_k=1, dtype=dtype, tokens=6,
                  capacity_rows=1)
    L = _random_predictor_layer(w, seed=2)
    X = wl.make_inputs(w)
    L.c = np.full(8, -1e6, np.float32)
    gpu = GpuLayer(w, L)
    ora = make_oracle(w, L)
    for t in range(w.tokens):
        L.c[:] = -1e6
        L.c[t % 8] = 1e6                               # neuron t fires, whatever x is: one row in, one row out per step
        gpu.layer.c.copy_(torch.from_numpy(L.c))
        r = compare_step(gpu, ora, X[t], w, t, api=api)
        assert r["n"] == 1 and r["added"] == 1 and r["removed"] == (1 if t else 0)


def test_longest_window_and_largest_batch():
    """window_k = 256 (the largest the ABI takes) on a short stream: nothing ever leaves; max_batch = 8 with steps of
    every batch size from 1 to 8 on the same layer."""
    from tests.harness import GpuLayer, compare_step
    w = wl.scaled(wl.WORKLOADS["C1"], name="k256", d_model=264, d_ffn=1096, rank=24, window_k=256, dtype="f16",
                  tokens=40, batch=8, p_active=0.01, capacity_rows=1096)
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w)
    gpu = GpuLayer(w, L)
    ora = make_oracle(w, L)
    for t in range(16):
        b = 1 + t % 8
        r = compare_step(gpu, ora, X[t][0] if b == 1 else X[t][:b], w, t, api="step" if t % 2 else "calls")
        assert r["removed"] == 0
    assert gpu.layer.state()["window_len"] == 16


def test_non_finite_input_predicts_nothing():
    """A NaN in x makes every logit NaN, and NaN > theta is false: no neuron is predicted, the window only ages.
    (The FFN over rows cached earlier would propagate the NaN; with an empty cache y is zero.)"""
    from tests.harness import GpuLayer
    w = wl.scaled(wl.WORKLOADS["C1"], tokens=4, window_k=1)
    L = wl.make_layer(w)
    X = wl.make_inputs(w).copy()
    X[1, 5] = np.nan
    gpu = GpuLayer(w, L)
    ora = make_oracle(w, L)
    lay = gpu.layer
    for t in range(2):
        ref = ora.step(X[t])
        lay.step(gpu.upload_x(X[t]), gpu.y)
        assert (lay.masks[:1].cpu().numpy() == O.pack_mask(np.atleast_2d(ref["masks"]))).all()
        assert lay.state()["num_used"] == ref["num_used"] and lay.state()["error"] == 0
    assert ref["num_used"] == 0 and not ref["masks"].any() and not gpu.y.cpu().numpy().any()
