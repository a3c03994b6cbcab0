"""Seeded synthetic workloads for the sparse-FFN hot path.

This module only *generates inputs*: FFN weights, biases, low-rank predictor
factors, AR(1) token streams and the row-column bundle store.  It holds none of
the method's arithmetic (no predictor evaluation, no windowing, no cache
management, no FFN) and is the single piece shared by the CPU oracle and the
HIP path: both consume the byte-identical arrays made here.

The workloads stand in for the paper's prompted generations on OPT-6.7B,
relufied Falcon-7B and sparsified Llama-2-7B (Section 4, "Experimental Setup"):
they take the FFN shapes, the activation-sparsity levels (Section 3.1: 97 %,
95 %, 90 %) and a token-to-token correlation, nothing else.
"""
from __future__ import annotations

import dataclasses
import functools

import numpy as np
from scipy.linalg import eigh
from scipy.stats import norm

BASE_SEED = 231211514


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    d_model: int
    d_ffn: int
    rank: int
    window_k: int
    p_active: float      # target fraction of neurons that fire per token
    rho: float           # AR(1) coefficient of the token stream
    dtype: str           # "f32" | "f16": storage type of weights and activations
    glu: bool            # gated FFN: bundle = gate row | up row | down column
    tokens: int
    batch: int
    capacity_rows: int   # rows preallocated in the HBM neuron cache
    layers: int = 1
    shrink: bool = False # dynamic window: drop the oldest masks instead of overflowing
    spec_keep: int = 0   # > 0: speculative verification passes of `batch` consecutive tokens, the first spec_keep kept
    gate_resident: bool = False  # gated FFN whose gate projection stays in HBM and serves as the predictor;
                                 # bundle = up row | down column

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def vectors_per_bundle(self) -> int:
        return 3 if (self.glu and not self.gate_resident) else 2

    @property
    def bundle_elems(self) -> int:
        return self.vectors_per_bundle * self.d_model

    @property
    def bundle_bytes(self) -> int:
        return self.bundle_elems * self.elem_bytes


WORKLOADS = {
    # tiny fp32 case the oracle finishes in seconds
    "C1": Workload("C1", 256, 1024, 32, 4, 0.05, 0.9, "f32", False, 64, 1, 1024),
    # OPT-6.7B-shaped ReLU FFN layer
    "C2": Workload("C2", 4096, 16384, 128, 5, 0.03, 0.9, "f16", False, 256, 1, 8192),
    # Falcon-7B-shaped relufied FFN layer
    "C3": Workload("C3", 4544, 18176, 128, 5, 0.07, 0.85, "f16", False, 256, 1, 9088),
    # Llama-2-7B-shaped gated FFN layer, batch 1 and batch 8
    "C4": Workload("C4", 4096, 11008, 256, 4, 0.10, 0.9, "f16", True, 256, 1, 11008),
    "C4b8": Workload("C4b8", 4096, 11008, 256, 4, 0.10, 0.9, "f16", True, 256, 8, 11008),
    # 32 stacked OPT-6.7B-shaped layers, cache capped at half the FFN rows
    "C5": Workload("C5", 4096, 16384, 128, 5, 0.03, 0.9, "f16", False, 512, 1, 8192, layers=32),
    # dynamic-window case: OPT shape at 10 % activity, k = 8, cache capped at 25 % of the FFN rows
    # (the appendix's Persimmon setting: window reduced whenever the cache would pass 25 % of the FFN)
    "N1": Workload("N1", 4096, 16384, 128, 8, 0.10, 0.9, "f16", False, 256, 1, 4096, shrink=True),
    # speculative verification (Section 4.3): passes of lambda + 1 = 5 consecutive tokens of one stream, 4 of
    # them accepted (acceptance ratio 0.8), window of the last 5 kept tokens; the next pass starts after them
    # Llama-2-7B-shaped gated layer with the gate projection resident as the (exact) predictor (appendix on
    # Llama 2, alternative approaches): only up | down bundles move
    "N4": Workload("N4", 4096, 11008, 256, 4, 0.10, 0.9, "f16", True, 256, 1, 11008, gate_resident=True),
    "N2": Workload("N2", 4096, 16384, 128, 5, 0.03, 0.9, "f16", False, 256, 5, 8192, spec_keep=4),
}


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (ragged or tiny test shapes)."""
    return dataclasses.replace(w, **changes)


def _rng(offset: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + offset))


def _top_right_singular_pairs(w64: np.ndarray, r: int):
    """Top-r right singular vectors V_r of W [F x d] through the Gram matrix.

    W = U S V^T  =>  W^T W = V S^2 V^T.  Only V_r is needed: the other factor of
    the truncated decomposition is S_r U_r^T = V_r^T W^T.
    """
    d = w64.shape[1]
    gram = w64.T @ w64
    _, vecs = eigh(gram, subset_by_index=[d - r, d - 1])
    return vecs[:, ::-1].copy()           # descending singular value


@dataclasses.dataclass
class LayerData:
    """All arrays of one FFN layer, in the storage dtype of the workload."""
    w_up: np.ndarray        # [F, d]   row i feeds neuron i
    w_down: np.ndarray      # [F, d]   row i is what neuron i writes
    w_gate: np.ndarray      # [F, d] or None
    b: np.ndarray           # [F] fp32 bias of the ReLU'd projection
    A: np.ndarray           # [d, r]
    B: np.ndarray           # [r, F]
    c: np.ndarray           # [F] fp32 predictor offset
    theta: float
    bundles: np.ndarray     # [F, G*d] row i = (gate_i |) up_i | down_i


def make_layer(w: Workload, layer: int = 0, structured: bool = False,
               overpredict: float = 1.0) -> LayerData:
    """Weights N(0, 1/d) cast once to the storage dtype; predictor = rank-r
    truncated SVD of the ReLU'd projection; biases calibrated in closed form so
    that, for a stationary N(0, I) input, a fraction p of neurons fire and a
    fraction p*overpredict are predicted.

    structured=True gives the ReLU'd projection a 1/j singular spectrum so that
    a rank-r predictor is accurate (labelled separately wherever it is used).
    """
    d, F, r = w.d_model, w.d_ffn, w.rank
    rng = _rng(layer)
    dt = w.np_dtype
    scale = np.float32(1.0 / np.sqrt(d))

    def gaussian():
        return rng.standard_normal((F, d), dtype=np.float32) * scale

    if structured:
        q1, _ = np.linalg.qr(rng.standard_normal((F, d)))
        q2, _ = np.linalg.qr(rng.standard_normal((d, d)))
        s = 1.0 / np.arange(1, d + 1)
        s *= np.sqrt(F / np.sum(s * s))          # rows keep unit mean square norm
        w_act32 = ((q1 * s) @ q2.T).astype(np.float32)
    else:
        w_act32 = gaussian()
    w_other32 = gaussian() if w.glu else None
    w_down32 = gaussian()

    w_act = w_act32.astype(dt)                   # the ReLU'd projection (gate if GLU, else up)
    w_down = w_down32.astype(dt)
    if w.glu:
        w_gate, w_up = w_act, w_other32.astype(dt)
    else:
        w_gate, w_up = None, w_act

    zq = norm.ppf(1.0 - w.p_active)
    w_act64 = w_act.astype(np.float64)
    b = (-zq * np.sqrt(np.sum(w_act64 * w_act64, axis=1))).astype(np.float32)

    v_r = _top_right_singular_pairs(w_act64, r)  # [d, r]
    A = v_r.astype(dt)
    B = (v_r.T @ w_act64.T).astype(dt)           # [r, F] = S_r U_r^T
    A64, B64 = A.astype(np.float64), B.astype(np.float64)
    colnorm = np.sqrt(np.maximum(np.sum(B64 * ((A64.T @ A64) @ B64), axis=0), 0.0))
    zq_pred = norm.ppf(1.0 - min(w.p_active * overpredict, 0.999))
    c = (-zq_pred * colnorm).astype(np.float32)

    parts = ([w_gate] if (w.glu and not w.gate_resident) else []) + [w_up, w_down]
    bundles = np.ascontiguousarray(np.concatenate(parts, axis=1))
    return LayerData(w_up, w_down, w_gate, b, A, B, c, 0.0, bundles)


def make_layer_variant(base: LayerData, w: Workload, layer: int) -> LayerData:
    """Layer `layer` of a stacked workload, derived from a base layer without a new decomposition.

    Neurons are permuted by pi and the input dimensions sign-flipped by s (both seeded by the layer
    index): up_i' = s * up_pi(i), down_i' = down_pi(i), gate likewise.  The truncated SVD is
    equivariant under both operations, so A' = diag(s) A, B'[:, i] = B[:, pi(i)], c' = c[pi],
    b' = b[pi] are exactly the arrays a fresh decomposition and cast would give (up to the
    sign convention of singular vectors).  Every layer has its own bytes and, for the same token
    stream, its own masks.  layer 0 is the base itself.
    """
    if layer == 0:
        return base
    rng = _rng(1000 + layer)
    pi = rng.permutation(w.d_ffn)
    sgn = np.where(rng.random(w.d_model) < 0.5, -1, 1).astype(base.w_up.dtype)
    w_up = base.w_up[pi] * sgn
    w_down = np.ascontiguousarray(base.w_down[pi])
    w_gate = None if base.w_gate is None else base.w_gate[pi] * sgn
    A = base.A * sgn[:, None]
    B = np.ascontiguousarray(base.B[:, pi])
    parts = ([w_gate] if (w.glu and not w.gate_resident) else []) + [w_up, w_down]
    bundles = np.ascontiguousarray(np.concatenate(parts, axis=1))
    return LayerData(w_up, w_down, w_gate, base.b[pi].copy(), A, B, base.c[pi].copy(), base.theta, bundles)


def make_inputs(w: Workload, stream: int = 0, tokens: int | None = None) -> np.ndarray:
    """AR(1) token stream x_t = rho x_{t-1} + sqrt(1-rho^2) N(0, I), x_0 ~ N(0, I),
    generated in fp64 and cast per token to the storage dtype.  Shape [T, d]."""
    T = w.tokens if tokens is None else tokens
    rng = _rng(100 + stream)
    x = np.empty((T, w.d_model), dtype=np.float64)
    x[0] = rng.standard_normal(w.d_model)
    s = np.sqrt(1.0 - w.rho * w.rho)
    for t in range(1, T):
        x[t] = w.rho * x[t - 1] + s * rng.standard_normal(w.d_model)
    return x.astype(w.np_dtype)


def make_batch_inputs(w: Workload, tokens: int | None = None) -> np.ndarray:
    """Batch of independent AR(1) streams, shape [T, batch, d]."""
    return np.stack([make_inputs(w, s, tokens) for s in range(w.batch)], axis=1)


@functools.lru_cache(maxsize=4)
def cached_layer(name: str, layer: int = 0) -> LayerData:
    return make_layer(WORKLOADS[name], layer)
