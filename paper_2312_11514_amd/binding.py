"""ctypes binding of include/lif.h: argument marshalling only.

Every step of the hot path runs inside liblif.so.  torch is used here for device
memory, pinned host memory and the stream handle - never for arithmetic.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblif.so")

LIF_OK, LIF_INVALID_ARG, LIF_BAD_STATE, LIF_CAPACITY, LIF_HIP_ERROR = 0, 1, 2, 3, 4
LIF_F32, LIF_F16 = 0, 1
FFN_SKIP_DEAD, FFN_FULL_BUNDLE = 0, 1
PRED_LOWRANK, PRED_GATE = 0, 1
KERNEL_NAMES = ("predict_xa", "predict_mask", "window", "load", "ffn_up", "ffn_down")
STATUS_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "BAD_STATE", 3: "CAPACITY", 4: "HIP_ERROR"}


class LifConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d_model", "d_ffn", "rank", "window_k", "capacity_rows",
                                         "max_batch", "glu", "dtype", "ffn_mode", "shrink_window",
                                         "predictor")] + \
        [("threshold", C.c_float)]


class LifBuffers(C.Structure):
    _fields_ = [("A", C.c_void_p), ("B", C.c_void_p), ("c", C.c_void_p), ("b", C.c_void_p),
                ("host_bundles", C.c_void_p), ("matrix", C.c_void_p), ("pointers", C.c_void_p),
                ("bias", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("host_down", C.c_void_p)]


class LifState(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("num_used", "step", "error", "last_added", "last_removed", "last_moved",
                                         "window_len")]


class LifCounters(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("steps", "added", "removed", "rows_moved", "h2d_bytes",
                                          "ffn_calls", "ffn_rows", "ffn_active")]


EXPORTS = {
    "lif_version": (C.c_int, []),
    "lif_last_error_string": (C.c_char_p, []),
    "lif_workspace_bytes": (C.c_size_t, [C.POINTER(LifConfig)]),
    "lif_create": (C.c_int, [C.POINTER(LifConfig), C.POINTER(LifBuffers), C.POINTER(C.c_void_p)]),
    "lif_destroy": (C.c_int, [C.c_void_p]),
    "lif_reset": (C.c_int, [C.c_void_p, C.c_void_p]),
    "lif_predict": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "lif_update_window": (C.c_int, [C.c_void_p] + [C.c_void_p] * 5 + [C.c_void_p]),
    "lif_update_window_tokens": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 4 + [C.c_void_p]),
    "lif_load_bundles": (C.c_int, [C.c_void_p] + [C.c_void_p] * 4 + [C.c_void_p]),
    "lif_sparse_ffn": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]),
    "lif_sparse_ffn_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]),
    "lif_static_scratch_bytes": (C.c_size_t, []),
    "lif_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p] + [C.c_void_p] * 6 + [C.c_void_p]),
    "lif_step_tokens": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p] + [C.c_void_p] * 6 +
                        [C.c_void_p]),
    "lif_set_expected_rows": (C.c_int, [C.c_void_p, C.c_int32]),
    "lif_set_loader_pairs": (C.c_int, [C.c_void_p, C.c_int32]),
    "lif_get_state": (C.c_int, [C.c_void_p, C.POINTER(LifState), C.c_void_p]),
    "lif_get_counters": (C.c_int, [C.c_void_p, C.POINTER(LifCounters), C.c_void_p]),
    "lif_profile_read": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "lif_profile_handoff": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint32, C.c_void_p]),
    "lif_profile_handoff_bytes": (C.c_size_t, []),
    "lif_profile_begin": (C.c_int, [C.c_void_p, C.c_int32]),
    "lif_profile_collect": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_void_p]),
}

_lib = None


class LifError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lif status {STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def load_library(path: str = LIB_PATH):
    """dlopen liblif.so and declare every prototype.  No fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is not built; run `python -m paper_2312_11514_amd.build` (needs hipcc)")
    lib = C.CDLL(path)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(rc: int):
    if rc != LIF_OK:
        raise LifError(rc, load_library().lif_last_error_string().decode(errors="replace"))


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def profile_read(src, nbytes, sink):
    """lif_profile_read: one plain streaming read of the first nbytes bytes of the device tensor src."""
    _check(load_library().lif_profile_read(_ptr(src), int(nbytes), _ptr(sink), _stream()))


def profile_handoff(scratch, mode, stamp=0):
    """lif_profile_handoff: one launch of the hand-off cost probe over a zero-initialised device byte tensor."""
    _check(load_library().lif_profile_handoff(_ptr(scratch), int(mode), int(stamp), _stream()))


def profile_handoff_bytes():
    return load_library().lif_profile_handoff_bytes()


class Layer:
    """One FFN layer behind the C ABI.  Owns (through torch) every array the library uses.

    A [rank, d_model] (or the gate projection [d_ffn, d_model]), B [rank, d_ffn], c, b: device tensors;
    host_bundles: pinned CPU tensor [F, G*d].  The four hot
    calls enqueue on torch's current stream and return immediately.
    """

    def __init__(self, *, d_model, d_ffn, rank, window_k, capacity_rows, max_batch=1, glu=False,
                 dtype="f16", ffn_mode=FFN_SKIP_DEAD, shrink_window=False, predictor=PRED_LOWRANK, threshold=0.0, A, B, c, b,
                 host_bundles, host_down=None):
        import torch
        self.lib = load_library()
        self.torch = torch
        self.cfg = LifConfig(d_model, d_ffn, rank, window_k, capacity_rows, max_batch, int(glu),
                             LIF_F32 if dtype == "f32" else LIF_F16, ffn_mode, int(shrink_window), predictor,
                             threshold)
        self.tdtype = torch.float32 if dtype == "f32" else torch.float16
        dev = A.device
        G = 3 if glu else 2
        ws_bytes = self.lib.lif_workspace_bytes(C.byref(self.cfg))
        if ws_bytes == 0:
            raise LifError(LIF_INVALID_ARG, "configuration rejected by lif_workspace_bytes")
        if not host_bundles.is_pinned() or (host_down is not None and not host_down.is_pinned()):
            raise LifError(LIF_INVALID_ARG, "host_bundles (and host_down) must be pinned host memory")
        self.A, self.B, self.c, self.b, self.host_bundles, self.host_down = A, B, c, b, host_bundles, host_down
        self.matrix = torch.empty((capacity_rows, G * d_model), dtype=self.tdtype, device=dev)
        self.pointers = torch.empty(capacity_rows, dtype=torch.int32, device=dev)
        self.bias = torch.empty(capacity_rows, dtype=torch.float32, device=dev)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.masks = torch.empty((max_batch, d_ffn // 8), dtype=torch.uint8, device=dev)
        self.step_mask = torch.empty(d_ffn // 8, dtype=torch.uint8, device=dev)
        self.added = torch.empty(d_ffn, dtype=torch.int32, device=dev)
        self.removed = torch.empty(d_ffn, dtype=torch.int32, device=dev)
        self.n_added = torch.empty(1, dtype=torch.int32, device=dev)
        self.n_removed = torch.empty(1, dtype=torch.int32, device=dev)
        self.buf = LifBuffers(A.data_ptr(), B.data_ptr() if B is not None else None,
                              c.data_ptr() if c is not None else None,
                              b.data_ptr(), host_bundles.data_ptr(), self.matrix.data_ptr(),
                              self.pointers.data_ptr(), self.bias.data_ptr(),
                              self.workspace.data_ptr(), ws_bytes,
                              host_down.data_ptr() if host_down is not None else None)
        h = C.c_void_p()
        _check(self.lib.lif_create(C.byref(self.cfg), C.byref(self.buf), C.byref(h)))
        self.handle = h
        self.reset()

    def close(self):
        if getattr(self, "handle", None):
            self.lib.lif_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the C-ABI calls, same names -------------------------------------------------
    def reset(self):
        _check(self.lib.lif_reset(self.handle, _stream()))

    def predict(self, x, batch=1, masks=None, step_mask=None):
        masks = self.masks if masks is None else masks
        step_mask = (masks if batch == 1 and step_mask is None and masks is not self.masks else
                     self.step_mask if step_mask is None else step_mask)
        _check(self.lib.lif_predict(self.handle, _ptr(x), batch, _ptr(masks), _ptr(step_mask), _stream()))
        return masks, step_mask

    def update_window(self, step_mask=None):
        step_mask = self.step_mask if step_mask is None else step_mask
        _check(self.lib.lif_update_window(self.handle, _ptr(step_mask), _ptr(self.added), _ptr(self.n_added),
                                          _ptr(self.removed), _ptr(self.n_removed), _stream()))

    def update_window_tokens(self, n_tokens, keep, masks=None):
        masks = self.masks if masks is None else masks
        _check(self.lib.lif_update_window_tokens(self.handle, _ptr(masks), n_tokens, keep, _ptr(self.added),
                                                 _ptr(self.n_added), _ptr(self.removed), _ptr(self.n_removed),
                                                 _stream()))

    def load_bundles(self):
        _check(self.lib.lif_load_bundles(self.handle, _ptr(self.added), _ptr(self.n_added),
                                         _ptr(self.removed), _ptr(self.n_removed), _stream()))

    def sparse_ffn(self, x, y, batch=1):
        _check(self.lib.lif_sparse_ffn(self.handle, _ptr(x), batch, _ptr(y), _stream()))

    def sparse_ffn_static(self, x, y, batch=1):
        """lif_sparse_ffn_static: the same call with its scratch in the library's static device array."""
        _check(self.lib.lif_sparse_ffn_static(self.handle, _ptr(x), batch, _ptr(y), _stream()))

    def step(self, x, y, batch=1):
        """lif_step: the whole step in one call (fused cache update + activations for batch 1)."""
        _check(self.lib.lif_step(self.handle, _ptr(x), batch, _ptr(y), _ptr(self.masks), _ptr(self.step_mask),
                                 _ptr(self.added), _ptr(self.n_added), _ptr(self.removed), _ptr(self.n_removed),
                                 _stream()))

    def step_tokens(self, x, y, n_tokens, keep_tokens):
        """lif_step_tokens: one speculative verification pass in one call."""
        _check(self.lib.lif_step_tokens(self.handle, _ptr(x), n_tokens, keep_tokens, _ptr(y), _ptr(self.masks),
                                        _ptr(self.step_mask), _ptr(self.added), _ptr(self.n_added),
                                        _ptr(self.removed), _ptr(self.n_removed), _stream()))

    def step_calls(self, x, y, batch=1):
        """The same step as four separate calls: predict -> update_window -> load_bundles -> sparse_ffn."""
        self.predict(x, batch)
        self.update_window()
        self.load_bundles()
        self.sparse_ffn(x, y, batch)

    def set_expected_rows(self, rows: int):
        _check(self.lib.lif_set_expected_rows(self.handle, int(rows)))

    def set_loader_pairs(self, pairs: int):
        _check(self.lib.lif_set_loader_pairs(self.handle, int(pairs)))

    # ---- introspection ---------------------------------------------------------------
    def state(self) -> dict:
        s = LifState()
        _check(self.lib.lif_get_state(self.handle, C.byref(s), _stream()))
        return {n: getattr(s, n) for n, _ in LifState._fields_}

    def counters(self) -> dict:
        s = LifCounters()
        _check(self.lib.lif_get_counters(self.handle, C.byref(s), _stream()))
        return {n: getattr(s, n) for n, _ in LifCounters._fields_}

    def profile_begin(self, max_launches: int):
        _check(self.lib.lif_profile_begin(self.handle, max_launches))

    def profile_collect(self) -> dict:
        ms = (C.c_double * len(KERNEL_NAMES))()
        cnt = (C.c_int64 * len(KERNEL_NAMES))()
        _check(self.lib.lif_profile_collect(self.handle, ms, cnt, _stream()))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_NAMES)}
