"""Test-side glue: uploads a workload, drives the C ABI, and compares each step with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2312_11514_amd as lif
from oracle import lif_oracle as O

REL_L2_TOL = 1e-3      # FFN output, fp16 storage + fp32 accumulation vs the fp64 oracle


def require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("a GPU test was collected on a machine without a GPU")
    lif.load_library()


class GpuLayer:
    def __init__(self, w, L, ffn_mode=lif.FFN_SKIP_DEAD, capacity=None, max_batch=None, use_c=True, shrink=False):
        require_gpu()
        dev = torch.device("cuda:0")
        self.w, self.dev = w, dev
        self.tdtype = torch.float32 if w.dtype == "f32" else torch.float16
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.host = torch.from_numpy(L.bundles).pin_memory()
        gate = w.gate_resident
        self.layer = lif.Layer(
            d_model=w.d_model, d_ffn=w.d_ffn, rank=w.rank, window_k=w.window_k,
            capacity_rows=capacity or w.capacity_rows, max_batch=max_batch or w.batch,
            glu=(w.glu and not gate), dtype=w.dtype, ffn_mode=ffn_mode, shrink_window=(shrink or w.shrink),
            predictor=lif.PRED_GATE if gate else lif.PRED_LOWRANK, threshold=L.theta,
            A=up(L.w_gate if gate else L.A.T),       # the ABI takes the contraction dimension contiguous: [rank, d_model]
            B=None if gate else up(L.B),
            c=up(L.c) if (use_c and not gate) else None, b=up(L.b), host_bundles=self.host)
        self.y = torch.zeros((max_batch or w.batch, w.d_model), dtype=self.tdtype, device=dev)

    def upload_x(self, x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(self.dev)

    def fill_cache(self, ids, L):
        """Bypass predict/window: place the bundles of `ids` directly in the cache (FFN-only tests)."""
        lay = self.layer
        n = len(ids)
        idt = torch.from_numpy(np.asarray(ids, dtype=np.int64))
        lay.matrix[:n] = self.host[idt].to(self.dev)
        lay.pointers[:n] = idt.to(torch.int32).to(self.dev)
        lay.bias[:n] = torch.from_numpy(L.b[np.asarray(ids)]).to(self.dev)
        # state block starts the workspace; first int32 is num_used
        lay.workspace[:4] = torch.from_numpy(np.array([n], dtype=np.int32).view(np.uint8)).to(self.dev)


def rel_l2(y, ref):
    y, ref = np.asarray(y, np.float64), np.asarray(ref, np.float64)
    nr = np.linalg.norm(ref, axis=-1)
    ne = np.linalg.norm(y - ref, axis=-1)
    if np.ndim(nr) == 0:
        return float(ne / nr) if nr > 0 else (0.0 if ne == 0 else np.inf)
    out = np.where(nr > 0, ne / np.where(nr > 0, nr, 1), np.where(ne == 0, 0.0, np.inf))
    return float(out.max())


def compare_step(gpu: GpuLayer, ora: O.OracleLayer, x, w, t, check_cache=True, api="calls"):
    """One token (x [d]) or one batch (x [batch, d]) through both paths; asserts parity of every output.
    api = "calls": the four C-ABI calls in sequence; "step": the single fused lif_step call."""
    lay = gpu.layer
    batch = 1 if x.ndim == 1 else x.shape[0]
    xd = gpu.upload_x(x)
    F = w.d_ffn

    ref = ora.step(x)

    if api == "step":
        lay.step(xd, gpu.y, batch)
    else:
        lay.predict(xd, batch)
        lay.update_window()
        lay.load_bundles()
        lay.sparse_ffn(xd, gpu.y, batch)
    na, nr = int(lay.n_added.item()), int(lay.n_removed.item())
    added = lay.added[:na].cpu().numpy()
    removed = lay.removed[:nr].cpu().numpy()
    st = lay.state()

    masks = lay.masks[:batch].cpu().numpy()
    ref_masks = np.atleast_2d(ref["masks"])
    tag = f"token {t}"
    assert (masks == O.pack_mask(ref_masks)).all(), f"{tag}: predictor mask differs"
    assert (lay.step_mask.cpu().numpy() == O.pack_mask(O.step_mask(ref_masks))).all(), f"{tag}: step mask"
    assert st["error"] == 0, f"{tag}: device error {st['error']}"
    assert added.tolist() == ref["added"].tolist(), f"{tag}: added ids differ"
    assert removed.tolist() == ref["removed"].tolist(), f"{tag}: removed ids differ"
    n = ref["num_used"]
    assert st["num_used"] == n, f"{tag}: num_used {st['num_used']} != {n}"
    assert st["step"] == t + 1
    if check_cache:
        assert (lay.pointers[:n].cpu().numpy() == ora.cache.pointers[:n]).all(), f"{tag}: cache layout differs"
        assert (lay.bias[:n].cpu().numpy() == ora.cache.bias[:n]).all(), f"{tag}: cache bias differs"
        gm = lay.matrix[:n].cpu().numpy()
        assert gm.tobytes() == ora.cache.matrix[:n].tobytes(), f"{tag}: cache rows differ"
    y = gpu.y[:batch].cpu().numpy().astype(np.float64)
    yref = np.atleast_2d(ref["y"])
    err = rel_l2(y, yref)
    assert err <= REL_L2_TOL, f"{tag}: FFN rel-L2 {err:.3e}"
    return dict(err=err, n=n, added=len(added), removed=len(removed), moved=st["last_moved"])
