"""CPU oracle for the sparse-FFN hot path of "LLM in a flash" (arXiv 2312.11514).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
statement of what the hot path computes.  It may be imported by tests, by the
smoke check and by the benchmark's CPU-baseline leg, never by the product path,
and it shares no code with the HIP implementation.

Every function restates one passage of the paper:

  predictor_logits / predict_mask   Section 3.1 "Anticipating ReLU Sparsity", Fig. 3b;
                                    "active neuron" = positive predictor output (Section 3.1,
                                    "The Sliding Window Technique")
  SlidingWindow                     Section 3.1 "The Sliding Window Technique", Fig. 4b;
                                    push_tokens: Section 4.3 "Speculative Decoding"
  bundle_bytes                      Section 3.2 "Bundling Columns and Rows", Fig. 5
  delete_neurons / insert_neurons   Section 3.3 items 1 and 2, Fig. 6
  sparse_ffn                        Section 3.3 item 3
  dense_ffn / true_mask             the FFN the method approximates (Section 3.1)

Floating point is fp64 throughout (inputs stored as fp16/fp32 are upcast
exactly).  Steps that have a plain definition are that definition written out:
the window is the brute-force union of the stored masks, deletion is the
sequential swap-with-last loop, the FFN is a sum over cached rows.

Readings of the paper taken here (the paper is silent or ambiguous):
  * the window of size k counts the current token: S_t = M_{t-k+1} | ... | M_t;
  * a neuron is active iff its logit is strictly greater than the threshold;
  * the predictor may carry a per-neuron offset c (null = 0);
  * deletion pairs the lowest dead slot with the highest live slot, repeatedly
    (Section 3.3: a deleted row is overwritten by a row taken from the end);
    insertion appends in ascending neuron id;
  * the FFN sums over every cached row (the window union), not only over the
    current token's mask;
  * a batch of tokens shares one cache: its step mask is the OR of the
    per-token masks and the window counts steps;
  * dynamic window (optional; Appendix, Persimmon, window configuration: the
    window gets smaller whenever the cache would outgrow its memory share) is
    read as dropping the oldest masks, for good, until the union of the
    remaining ones fits the cache;
  * the threshold is the fp32 value the C ABI carries (theta rounded to fp32
    once, then compared in fp64), for both predictors.
Pins: tests/test_oracle_*.py.  Nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- predictor
def predictor_logits(x, A, B, c=None):
    """z = (x A) B + c in fp64.  x [d] or [batch, d]; A [d, r]; B [r, F]; c [F] or None."""
    t = np.asarray(x, dtype=np.float64) @ np.asarray(A, dtype=np.float64)
    z = t @ np.asarray(B, dtype=np.float64)
    if c is not None:
        z = z + np.asarray(c, dtype=np.float64)
    return z


def predict_mask(x, A, B, c, theta):
    """Boolean mask(s) of predicted-active neurons and the decision margin min |z - theta|."""
    z = predictor_logits(x, A, B, c)
    th = np.float64(np.float32(theta))
    mask = z > th
    finite = np.isfinite(th)
    margin = float(np.min(np.abs(z - th))) if finite and z.size else float("inf")
    return mask, margin


def step_mask(masks):
    """OR over the tokens of a batch; a single mask is returned unchanged."""
    masks = np.asarray(masks, dtype=bool)
    return masks if masks.ndim == 1 else np.logical_or.reduce(masks, axis=0)


def pack_mask(mask):
    """Bit i of the mask is bit (i mod 8) of byte i // 8."""
    return np.packbits(np.asarray(mask, dtype=bool), axis=-1, bitorder="little")


def unpack_mask(packed, n):
    return np.unpackbits(np.asarray(packed, dtype=np.uint8), axis=-1, count=n,
                         bitorder="little").astype(bool)


# --------------------------------------------------------------------------- window
class SlidingWindow:
    """Keeps the last k step masks; the active set is their union, by brute force."""

    def __init__(self, d_ffn: int, k: int):
        assert k >= 1
        self.F, self.k = d_ffn, k
        self.masks: list[np.ndarray] = []
        self.transient = np.zeros(d_ffn, dtype=bool)     # masks needed by the last step only (push_tokens)

    def active_set(self) -> np.ndarray:
        s = self.transient.copy()
        for m in self.masks:
            s |= m
        return s

    def push_tokens(self, masks, keep, capacity=None, shrink=False):
        """One verification pass of speculative decoding (Section 4.3): `masks` [n_tokens, F] are the
        per-token masks of the pass; the first `keep` tokens enter the window one by one; every
        mask of the pass is held for this pass (all its tokens are computed), those that are not
        in the window afterwards leave with the next update.  Returns (added, removed) against what was held before.

        If what has to be held would exceed `capacity` rows: with shrink=False the state is left unchanged and
        OverflowError is raised; with shrink=True (dynamic window, Appendix, Persimmon / Phi-2 window
        configuration, applied to a pass of tokens) the oldest window masks leave for good, one at a time, until
        the masks of the pass together with the remaining window fit; only a pass whose own masks do not fit raises."""
        masks = np.asarray(masks, dtype=bool)
        before = self.active_set()
        new_masks = list(self.masks)
        for i in range(keep):
            new_masks.append(masks[i].copy())
            new_masks = new_masks[-self.k:]
        transient = np.zeros(self.F, dtype=bool)       # every token of the pass is computed in this pass,
        for i in range(len(masks)):                    # also one that enters and leaves the window at once
            transient |= masks[i]

        def held(ms):
            u = transient.copy()
            for m in ms:
                u |= m
            return u

        after = held(new_masks)
        if capacity is not None and int(after.sum()) > capacity:
            if not shrink:
                raise OverflowError("active set exceeds the neuron cache capacity")
            while new_masks and int(held(new_masks).sum()) > capacity:
                new_masks.pop(0)
            after = held(new_masks)
            if int(after.sum()) > capacity:
                raise OverflowError("the masks of the pass alone exceed the neuron cache capacity")
        self.masks, self.transient = new_masks, transient
        added = np.flatnonzero(after & ~before).astype(np.int32)
        removed = np.flatnonzero(before & ~after).astype(np.int32)
        return added, removed

    def push(self, mask, capacity=None, shrink=False):
        """Slide by one step.  Returns (added ids, removed ids), ascending int32.

        If the new active set would exceed `capacity` rows: with shrink=False the window is left
        unchanged and OverflowError is raised; with shrink=True (dynamic window, Appendix:
        Persimmon and Phi-2 reduce the window whenever the memory limit would be passed) the
        oldest masks leave the window for good, one at a time, until the union fits; only a
        mask that does not fit alone raises.
        """
        before = self.active_set()
        kept = self.masks[-(self.k - 1):] if self.k > 1 else []
        new_masks = kept + [np.array(mask, dtype=bool, copy=True)]

        def union(ms):
            u = np.zeros(self.F, dtype=bool)
            for m in ms:
                u |= m
            return u

        after = union(new_masks)
        if capacity is not None and int(after.sum()) > capacity:
            if not shrink:
                raise OverflowError("active set exceeds the neuron cache capacity")
            while len(new_masks) > 1 and int(union(new_masks).sum()) > capacity:
                new_masks.pop(0)
            after = union(new_masks)
            if int(after.sum()) > capacity:
                raise OverflowError("the step mask alone exceeds the neuron cache capacity")
        self.masks = new_masks
        self.transient = np.zeros(self.F, dtype=bool)
        added = np.flatnonzero(after & ~before).astype(np.int32)
        removed = np.flatnonzero(before & ~after).astype(np.int32)
        return added, removed


# --------------------------------------------------------------------------- cache
def bundle_bytes(d_model: int, num_bytes: int, glu: bool = False) -> int:
    """Chunk read per neuron: up row + down column (+ gate row), each d_model elements."""
    return (3 if glu else 2) * d_model * num_bytes


class NeuronCache:
    """The preallocated structure of Section 3.3: matrix, pointers, bias, num_used."""

    def __init__(self, capacity_rows: int, row_elems: int, dtype):
        self.matrix = np.zeros((capacity_rows, row_elems), dtype=dtype)
        self.pointers = np.full(capacity_rows, -1, dtype=np.int32)
        self.bias = np.zeros(capacity_rows, dtype=np.float32)
        self.num_used = 0
        self.capacity = capacity_rows


def delete_neurons(cache: NeuronCache, removed) -> int:
    """Swap-with-last deletion as a two-pointer pass.  Returns the number of rows moved."""
    n = cache.num_used
    gone = set(int(i) for i in removed)
    dead = [int(cache.pointers[s]) in gone for s in range(n)]
    c = sum(dead)
    assert c == len(gone), "a removed neuron is not cached"
    lo, hi, moved = 0, n - 1, 0
    while True:
        while hi >= 0 and dead[hi]:
            hi -= 1
        while lo < hi and not dead[lo]:
            lo += 1
        if lo >= hi:
            break
        cache.matrix[lo] = cache.matrix[hi]
        cache.pointers[lo] = cache.pointers[hi]
        cache.bias[lo] = cache.bias[hi]
        dead[lo], dead[hi] = False, True
        moved += 1
        lo += 1
        hi -= 1
    cache.num_used = n - c
    return moved


def insert_neurons(cache: NeuronCache, added, host_bundles, b) -> int:
    """Append the bundles of `added` (ascending id) after the used rows.  Returns bytes loaded."""
    n = cache.num_used
    a = len(added)
    if n + a > cache.capacity:
        raise OverflowError("neuron cache capacity exceeded")
    for j, i in enumerate(added):
        cache.matrix[n + j] = host_bundles[i]
        cache.pointers[n + j] = i
        cache.bias[n + j] = b[i]
    cache.num_used = n + a
    return a * host_bundles.shape[1] * host_bundles.dtype.itemsize


# --------------------------------------------------------------------------- FFN
def sparse_ffn(cache: NeuronCache, x, d_model: int, glu: bool = False, acc=np.float64):
    """y = sum over cached rows of relu(u.x + bias) * down  (GLU: relu(g.x + bias) * (u.x) * down).

    x [d] or [batch, d].  `acc` = np.float32 gives the fp32-accumulation variant
    that sizes the tolerance of the GPU comparison.
    """
    n, d = cache.num_used, d_model
    x = np.asarray(x, dtype=acc)
    rows = cache.matrix[:n].astype(acc)
    bias = cache.bias[:n].astype(acc)
    if glu:
        gate, up, down = rows[:, :d], rows[:, d:2 * d], rows[:, 2 * d:]
        h = np.maximum(x @ gate.T + bias, 0) * (x @ up.T)
    else:
        up, down = rows[:, :d], rows[:, d:]
        h = np.maximum(x @ up.T + bias, 0)
    return h @ down


def sparse_ffn_loops(cache: NeuronCache, x, d_model: int, glu: bool = False):
    """Same sum, one cached row at a time, in slot order (single token)."""
    d = d_model
    x = np.asarray(x, dtype=np.float64)
    y = np.zeros(d, dtype=np.float64)
    for s in range(cache.num_used):
        row = cache.matrix[s].astype(np.float64)
        if glu:
            h = max(float(row[:d] @ x) + float(cache.bias[s]), 0.0) * float(row[d:2 * d] @ x)
            y += h * row[2 * d:]
        else:
            h = max(float(row[:d] @ x) + float(cache.bias[s]), 0.0)
            y += h * row[d:]
    return y


def gate_predict_mask(x, w_gate, b, theta):
    """Appendix (Llama 2, alternative approaches): with the gate projection resident, the gate
    pre-activations a_i = gate_i . x + b_i are known before anything is loaded and a_i > theta names
    exactly the neurons that fire.  Returns (mask, margin, relu(a)) in fp64."""
    a = np.asarray(x, np.float64) @ np.asarray(w_gate, np.float64).T + np.asarray(b, np.float64)
    th = np.float64(np.float32(theta))
    margin = float(np.min(np.abs(a - th))) if np.isfinite(th) and a.size else float("inf")
    return a > th, margin, np.maximum(a, 0.0)


def sparse_ffn_resident_gate(cache: NeuronCache, gate_act, x, d_model: int):
    """FFN over the cached rows when bundles hold up row | down column and the gate activation
    relu(gate_i . x + b_i) comes from the resident gate projection (indexed by original neuron id):
    y = sum_s gate_act[pointers[s]] * (up_s . x) * down_s.  x [d] with gate_act [F], or a batch of tokens
    x [batch, d] with gate_act [batch, F] (one row of y per token, all over the same cached rows)."""
    n = cache.num_used
    m = cache.matrix[:n].astype(np.float64)
    up, down = m[:, :d_model], m[:, d_model:2 * d_model]
    h = np.asarray(gate_act, np.float64)[..., cache.pointers[:n]] * (np.asarray(x, np.float64) @ up.T)
    return h @ down


def preactivations(w_act, b, x):
    return np.asarray(w_act, dtype=np.float64) @ np.asarray(x, dtype=np.float64) + \
        np.asarray(b, dtype=np.float64)


def true_mask(w_act, b, x):
    """Neurons the ReLU keeps (w_act = up projection, or the gate projection if GLU)."""
    return preactivations(w_act, b, x) > 0


def dense_ffn(w_up, w_down, b, x, w_gate=None, only=None):
    """Dense FFN, neuron by neuron in ascending id.  `only` (bool [F]) restricts the sum."""
    x = np.asarray(x, dtype=np.float64)
    F, d = w_up.shape
    y = np.zeros(d, dtype=np.float64)
    for i in range(F):
        if only is not None and not only[i]:
            continue
        if w_gate is not None:
            h = max(float(w_gate[i].astype(np.float64) @ x) + float(b[i]), 0.0) * \
                float(w_up[i].astype(np.float64) @ x)
        else:
            h = max(float(w_up[i].astype(np.float64) @ x) + float(b[i]), 0.0)
        y += h * w_down[i].astype(np.float64)
    return y


# --------------------------------------------------------------------------- whole path
class OracleLayer:
    """One FFN layer driven token by token: predict -> window -> delete -> insert -> FFN."""

    def __init__(self, d_model, d_ffn, window_k, capacity_rows, glu, A, B, c, theta, b,
                 host_bundles, shrink=False, w_gate=None):
        """w_gate given: the resident gate projection is the predictor (A, B, c unused, glu False,
        bundles = up | down)."""
        self.shrink = shrink
        self.w_gate = w_gate
        self.gate_act = None
        self.d, self.F, self.k, self.glu = d_model, d_ffn, window_k, glu
        self.A, self.B, self.c, self.theta, self.b = A, B, c, theta, b
        self.host = host_bundles
        self.window = SlidingWindow(d_ffn, window_k)
        self.cache = NeuronCache(capacity_rows, host_bundles.shape[1], host_bundles.dtype)
        self.bytes_loaded = 0
        self.rows_moved = 0
        self.min_margin = float("inf")

    def predict(self, x):
        if self.w_gate is not None:
            mask, margin, self.gate_act = gate_predict_mask(x, self.w_gate, self.b, self.theta)
        else:
            mask, margin = predict_mask(x, self.A, self.B, self.c, self.theta)
        self.min_margin = min(self.min_margin, margin)
        return mask

    def update_window(self, mask):
        return self.window.push(step_mask(mask), self.cache.capacity, self.shrink)

    def load_bundles(self, added, removed):
        self.rows_moved += delete_neurons(self.cache, removed)
        loaded = insert_neurons(self.cache, added, self.host, self.b)
        self.bytes_loaded += loaded
        return loaded

    def sparse_ffn(self, x, acc=np.float64):
        if self.w_gate is not None:
            return sparse_ffn_resident_gate(self.cache, self.gate_act, x, self.d)
        return sparse_ffn(self.cache, x, self.d, self.glu, acc)

    def step_tokens(self, x, keep):
        """One speculative verification pass: x [n_tokens, d]; the first `keep` tokens enter the window."""
        masks = self.predict(x)
        added, removed = self.window.push_tokens(masks, keep, self.cache.capacity, self.shrink)
        loaded = self.load_bundles(added, removed)
        y = self.sparse_ffn(x)
        return dict(masks=masks, added=added, removed=removed, loaded=loaded, y=y,
                    num_used=self.cache.num_used)

    def step(self, x):
        """One token (or one batch of tokens).  Returns a dict with every intermediate."""
        masks = self.predict(x)
        added, removed = self.update_window(masks)
        loaded = self.load_bundles(added, removed)
        y = self.sparse_ffn(x)
        return dict(masks=masks, added=added, removed=removed, loaded=loaded, y=y,
                    num_used=self.cache.num_used)
