"""Uploads a synthetic workload into a layer of the HIP library (device tensors, pinned bundle store).

Shared by the GPU tests, bench.py and the smoke check.  Holds no arithmetic of the method and does
not know the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2312_11514_amd as lif


def require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("a GPU test was collected on a machine without a GPU")
    lif.load_library()


class GpuLayer:
    def __init__(self, w, L, ffn_mode=lif.FFN_SKIP_DEAD, capacity=None, max_batch=None, use_c=True, shrink=False,
                 share=None, unbundled=False):
        """share: another GpuLayer of the same workload and layer data whose predictor arrays and pinned bundle
        store this one reuses (its own cache, window state and workspace): several caches of one layer.
        unbundled: the pinned store is kept in two parts (activation vectors | down columns), two reads per neuron."""
        require_gpu()
        dev = torch.device("cuda:0")
        self.w, self.dev = w, dev
        self.tdtype = torch.float32 if w.dtype == "f32" else torch.float16
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        gate = w.gate_resident
        self.host_down = None
        if share is not None:
            sl = share.layer
            self.host, self.host_down, A, B, c, b = share.host, share.host_down, sl.A, sl.B, sl.c, sl.b
        else:
            if unbundled:
                cut = L.bundles.shape[1] - w.d_model
                self.host = torch.from_numpy(np.ascontiguousarray(L.bundles[:, :cut])).pin_memory()
                self.host_down = torch.from_numpy(np.ascontiguousarray(L.bundles[:, cut:])).pin_memory()
            else:
                self.host = torch.from_numpy(L.bundles).pin_memory()
            A = up(L.w_gate if gate else L.A.T)      # the ABI takes the contraction dimension contiguous: [rank, d_model]
            B = None if gate else up(L.B)
            c = up(L.c) if (use_c and not gate) else None
            b = up(L.b)
        self.layer = lif.Layer(
            d_model=w.d_model, d_ffn=w.d_ffn, rank=w.rank, window_k=w.window_k,
            capacity_rows=capacity or w.capacity_rows, max_batch=max_batch or w.batch,
            glu=(w.glu and not gate), dtype=w.dtype, ffn_mode=ffn_mode, shrink_window=(shrink or w.shrink),
            predictor=lif.PRED_GATE if gate else lif.PRED_LOWRANK, threshold=L.theta,
            A=A, B=B, c=c, b=b, host_bundles=self.host, host_down=self.host_down)
        self.y = torch.zeros((max_batch or w.batch, w.d_model), dtype=self.tdtype, device=dev)

    def upload_x(self, x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(self.dev)

    def fill_cache(self, ids, L):
        """Bypass predict/window: place the bundles of `ids` directly in the cache (FFN-only tests)."""
        lay = self.layer
        n = len(ids)
        idt = torch.from_numpy(np.asarray(ids, dtype=np.int64))
        rows = self.host[idt] if self.host_down is None else torch.cat([self.host[idt], self.host_down[idt]], dim=1)
        lay.matrix[:n] = rows.to(self.dev)
        lay.pointers[:n] = idt.to(torch.int32).to(self.dev)
        lay.bias[:n] = torch.from_numpy(L.b[np.asarray(ids)]).to(self.dev)
        # state block starts the workspace; first int32 is num_used
        lay.workspace[:4] = torch.from_numpy(np.array([n], dtype=np.int32).view(np.uint8)).to(self.dev)
