"""Test-side glue: uploads a workload, drives the C ABI, and compares each step with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2312_11514_amd as lif
from oracle import lif_oracle as O

REL_L2_TOL = 1e-3      # FFN output, fp16 storage + fp32 accumulation vs the fp64 oracle
MAX_ABS_TOL = 1e-3     # and element by element: |y - y_ref| <= 1e-3 * max|y_ref| per token row (one fp16 rounding of
                       # the largest element is 4.9e-4 of it; fp32 accumulation adds ~1e-6), which names the column


from workloads.device import GpuLayer, require_gpu  # noqa: E402,F401  (re-exported for the tests)


def rel_l2(y, ref):
    y, ref = np.asarray(y, np.float64), np.asarray(ref, np.float64)
    nr = np.linalg.norm(ref, axis=-1)
    ne = np.linalg.norm(y - ref, axis=-1)
    if np.ndim(nr) == 0:
        return float(ne / nr) if nr > 0 else (0.0 if ne == 0 else np.inf)
    out = np.where(nr > 0, ne / np.where(nr > 0, nr, 1), np.where(ne == 0, 0.0, np.inf))
    return float(out.max())


def max_abs_excess(y, ref):
    """Largest |y - ref| / max|ref| over the token rows, and where it sits (row, column)."""
    y, ref = np.atleast_2d(np.asarray(y, np.float64)), np.atleast_2d(np.asarray(ref, np.float64))
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    err = np.abs(y - ref) / np.where(scale > 0, scale, 1.0)
    err = np.where(scale > 0, err, np.where(y == 0, 0.0, np.inf))
    i = np.unravel_index(np.argmax(err), err.shape)
    return float(err[i]), i


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
    worst, where = max_abs_excess(y, yref)
    assert worst <= MAX_ABS_TOL, f"{tag}: FFN element {where} off by {worst:.3e} of the row's largest value"
    return dict(err=err, n=n, added=len(added), removed=len(removed), moved=st["last_moved"])
