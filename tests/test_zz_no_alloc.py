"""lif_sparse_ffn_static (scratch in the library's static device array, nothing allocated) against lif_sparse_ffn."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def _layer(w, seed):
    rng = np.random.default_rng(seed)
    d, F, dt = w.d_model, w.d_ffn, w.np_dtype
    g = lambda *shape: rng.standard_normal(shape, dtype=np.float32)
    up, down = (g(F, d) / np.sqrt(d)).astype(dt), (g(F, d) / np.sqrt(d)).astype(dt)
    gate = (g(F, d) / np.sqrt(d)).astype(dt) if w.glu else None
    act = gate if w.glu else up
    b = (-1.0 * np.linalg.norm(act.astype(np.float64), axis=1)).astype(np.float32)
    A, B = (g(d, w.rank) / np.sqrt(d)).astype(dt), g(w.rank, F).astype(dt)
    parts = ([gate] if w.glu else []) + [up, down]
    return wl.LayerData(up, down, gate, b, A, B, np.zeros(F, np.float32), 0.0,
                        np.ascontiguousarray(np.concatenate(parts, axis=1)))


@pytest.mark.parametrize("dtype,glu,d_model,rows,ffn_mode", [
    ("f16", False, 4096, (5000, 1227), 0),     # OPT row width; several row chunks, then a single chunk
    ("f16", True, 608, (2300, 700), 1),        # gated, MFMA activation stage for the batched calls
    ("f32", False, 264, (1500, 33), 0),
])
def test_static_scratch_ffn_equals_workspace_ffn(dtype, glu, d_model, rows, ffn_mode):
    """Two calls in a row through the C ABI, the second on a smaller input (fewer cached rows and a smaller
    batch): every output byte equals lif_sparse_ffn's, which the parity tests hold to the oracle."""
    from oracle import lif_oracle as O
    from tests.harness import GpuLayer, rel_l2, REL_L2_TOL
    F = 8192
    w = wl.scaled(wl.WORKLOADS["C1"], name="static", d_model=d_model, d_ffn=F, rank=8, dtype=dtype, glu=glu,
                  batch=5, capacity_rows=F)
    L = _layer(w, seed=d_model)
    gpu = GpuLayer(w, L, ffn_mode=ffn_mode)
    lay = gpu.layer
    rng = np.random.default_rng(3)
    X = rng.standard_normal((5, d_model)).astype(w.np_dtype)
    xd = gpu.upload_x(X)
    for n, batch in zip(rows, (5, 2)):
        ids = np.sort(rng.choice(F, n, replace=False))
        lay.reset()
        gpu.fill_cache(ids, L)
        y_ws = torch.full((5, d_model), 7.0, dtype=gpu.tdtype, device=gpu.dev)
        y_st = torch.full((5, d_model), -7.0, dtype=gpu.tdtype, device=gpu.dev)
        print(f"static ffn: dtype={dtype} glu={glu} d={d_model} rows={n} batch={batch}", flush=True)
        lay.sparse_ffn(xd, y_ws, batch)
        lay.sparse_ffn_static(xd, y_st, batch)
        torch.cuda.synchronize()
        assert lay.state()["error"] == 0
        assert torch.equal(y_ws[:batch], y_st[:batch])
        assert (y_st[batch:] == -7.0).all()                      # rows past the batch are not written
        # and against the oracle directly, to the FFN bar
        cache = O.NeuronCache(n, L.bundles.shape[1], L.bundles.dtype)
        cache.matrix[:] = L.bundles[ids]
        cache.bias[:] = L.b[ids]
        cache.num_used = n
        ref = O.sparse_ffn(cache, X[:batch], d_model, glu)
        assert rel_l2(y_st[:batch].cpu().numpy(), ref) <= (1e-5 if dtype == "f32" else REL_L2_TOL)


def test_static_scratch_ffn_under_graph_capture():
    """The callers the entry point is for: captured once in a HIP graph (no allocation may happen there), replayed
    three times with eager work in between, every replay equal to the eager workspace call."""
    from tests.harness import GpuLayer
    F, d = 4096, 1024
    w = wl.scaled(wl.WORKLOADS["C1"], name="static", d_model=d, d_ffn=F, rank=8, dtype="f16", glu=False, batch=4,
                  capacity_rows=F)
    L = _layer(w, seed=9)
    gpu = GpuLayer(w, L)
    lay = gpu.layer
    rng = np.random.default_rng(4)
    ids = np.sort(rng.choice(F, 3000, replace=False))
    gpu.fill_cache(ids, L)
    xd = gpu.upload_x(rng.standard_normal((4, d)).astype(np.float16))
    y_ref = torch.zeros((4, d), dtype=torch.float16, device=gpu.dev)
    y = torch.zeros_like(y_ref)
    lay.sparse_ffn(xd, y_ref, 4)
    lay.sparse_ffn_static(xd, y, 4)                    # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        lay.sparse_ffn_static(xd, y, 4)
    for rep in range(3):
        y.fill_(9.0)
        lay.sparse_ffn(xd, gpu.y, 4)                   # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"replay {rep}"


def test_static_scratch_limit_is_an_error():
    import paper_2312_11514_amd as lif
    from tests.harness import GpuLayer
    assert lif.load_library().lif_static_scratch_bytes() == 5 << 20
    # batch 8: 4 * 8 * 65536 = 2 MiB of activations + 4 * 32 * 8 * 4096 = 4 MiB of partials > 5 MiB
    w = wl.scaled(wl.WORKLOADS["C1"], name="big", d_model=4096, d_ffn=512, rank=8, dtype="f16", batch=8,
                  capacity_rows=65536)
    L = _layer(w, seed=1)
    gpu = GpuLayer(w, L)
    x = torch.zeros((8, 4096), dtype=torch.float16, device=gpu.dev)
    y = torch.full((8, 4096), 3.0, dtype=torch.float16, device=gpu.dev)
    with pytest.raises(lif.LifError) as e:
        gpu.layer.sparse_ffn_static(x, y, 8)
    assert e.value.status == lif.LIF_INVALID_ARG and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (y == 3.0).all()
    gpu.layer.sparse_ffn_static(x, y, 4)                         # batch 4 fits: 1 MiB + 2 MiB
    torch.cuda.synchronize()
    assert not y[:4].any() and (y[4:] == 3.0).all()              # empty cache: zeros
