"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it leans on.  The expected values come from
hand-worked fixtures under tests/golden/, from closed forms, or from
independent brute force written here with Python sets and scalars.
"""
import json
import os

import numpy as np
import pytest
from scipy.stats import norm

import workloads as wl
from oracle import lif_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def cache_from_rows(rows, pointers, bias, capacity=None, dtype=np.float32):
    rows = np.asarray(rows, dtype=dtype)
    cap = capacity or max(len(rows), 1)
    c = O.NeuronCache(cap, rows.shape[1], dtype)
    c.matrix[:len(rows)] = rows
    c.pointers[:len(rows)] = pointers
    c.bias[:len(rows)] = bias
    c.num_used = len(rows)
    return c


# ----------------------------------------------------------------------------- bundles
def test_bundle_size_matches_paper_constants():
    g = golden("paper_constants.json")
    for key in ("opt_6p7b", "falcon_7b"):
        e = g[key]
        assert O.bundle_bytes(e["d_model"], e["num_bytes"]) == e["bundle_kib"] * 1024
    # bundling doubles the chunk (Section 3.2); the gated variant triples it
    assert O.bundle_bytes(4096, 2) == 2 * (4096 * 2)
    assert O.bundle_bytes(4096, 2, glu=True) == 3 * (4096 * 2)
    for name, w in wl.WORKLOADS.items():
        assert w.bundle_bytes == O.bundle_bytes(w.d_model, w.elem_bytes, w.glu and not w.gate_resident)


# ----------------------------------------------------------------------------- FFN
@pytest.mark.parametrize("fn", [O.sparse_ffn, O.sparse_ffn_loops])
def test_ffn_hand_worked(fn):
    g = golden("ffn_tiny.json")
    d = g["d_model"]
    p = g["plain"]
    rows = np.concatenate([np.array(p["up"], float), np.array(p["down"], float)], axis=1)
    cache = cache_from_rows(rows, [0, 1, 2], p["bias"])
    np.testing.assert_array_equal(fn(cache, g["x"], d), p["y"])
    q = g["glu"]
    rows = np.concatenate([np.array(q["gate"], float), np.array(q["up"], float),
                           np.array(q["down"], float)], axis=1)
    cache = cache_from_rows(rows, [0, 1, 2], q["bias"])
    np.testing.assert_array_equal(fn(cache, g["x"], d, glu=True), q["y"])
    assert list(O.true_mask(np.array(p["up"]), p["bias"], g["x"])) == p["true_mask"]


def test_dense_ffn_hand_worked():
    g = golden("ffn_tiny.json")
    p, q = g["plain"], g["glu"]
    y = O.dense_ffn(np.array(p["up"], float), np.array(p["down"], float), p["bias"], g["x"])
    np.testing.assert_array_equal(y, p["y"])
    y = O.dense_ffn(np.array(q["up"], float), np.array(q["down"], float), q["bias"], g["x"],
                    w_gate=np.array(q["gate"], float))
    np.testing.assert_array_equal(y, q["y"])


def _small_layer(glu=False, dtype="f32", d=64, F=192, r=16):
    w = wl.scaled(wl.WORKLOADS["C1"], d_model=d, d_ffn=F, rank=r, glu=glu, dtype=dtype,
                  capacity_rows=F, tokens=12, p_active=0.1)
    return w, wl.make_layer(w), wl.make_inputs(w)


@pytest.mark.parametrize("glu", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_sparse_over_true_set_equals_dense(glu, dtype):
    """ReLU-zeroed neurons contribute nothing (Section 3.1), so the sum over exactly the
    true-active neurons, taken in ascending id, is the dense FFN bit for bit."""
    w, L, X = _small_layer(glu, dtype)
    w_act = L.w_gate if glu else L.w_up
    for x in X[:4]:
        tm = O.true_mask(w_act, L.b, x)
        assert 0 < tm.sum() < w.d_ffn
        ids = np.flatnonzero(tm)
        cache = cache_from_rows(L.bundles[ids], ids, L.b[ids], dtype=L.bundles.dtype)
        y_dense = O.dense_ffn(L.w_up, L.w_down, L.b, x, L.w_gate)
        y_loop = O.sparse_ffn_loops(cache, x, w.d_model, glu)
        np.testing.assert_array_equal(y_loop, y_dense)
        np.testing.assert_array_equal(O.dense_ffn(L.w_up, L.w_down, L.b, x, L.w_gate, only=tm), y_dense)
        # matrix form and any slot order: equal up to fp64 rounding (Section 3.3 item 3:
        # the order of the cached neurons does not change the output)
        y_mat = O.sparse_ffn(cache, x, w.d_model, glu)
        perm = np.random.default_rng(1).permutation(len(ids))
        cache_p = cache_from_rows(L.bundles[ids[perm]], ids[perm], L.b[ids[perm]], dtype=L.bundles.dtype)
        y_perm = O.sparse_ffn(cache_p, x, w.d_model, glu)
        scale = np.linalg.norm(y_dense)
        assert np.linalg.norm(y_mat - y_dense) <= 1e-12 * scale
        assert np.linalg.norm(y_perm - y_dense) <= 1e-12 * scale


def test_all_rows_cached_equals_dense_and_empty_cache_is_zero():
    w, L, X = _small_layer()
    ids = np.arange(w.d_ffn)
    cache = cache_from_rows(L.bundles, ids, L.b)
    y = O.sparse_ffn(cache, X[0], w.d_model)
    y_dense = O.dense_ffn(L.w_up, L.w_down, L.b, X[0])
    assert np.linalg.norm(y - y_dense) <= 1e-12 * np.linalg.norm(y_dense)
    cache.num_used = 0
    assert not O.sparse_ffn(cache, X[0], w.d_model).any()
    assert not O.sparse_ffn_loops(cache, X[0], w.d_model).any()


def test_ffn_batch_rows_equal_single_token_calls():
    w, L, X = _small_layer(glu=True)
    ids = np.arange(0, w.d_ffn, 3)
    cache = cache_from_rows(L.bundles[ids], ids, L.b[ids])
    Y = O.sparse_ffn(cache, X[:5], w.d_model, True)
    for t in range(5):
        y1 = O.sparse_ffn_loops(cache, X[t], w.d_model, True)
        assert np.linalg.norm(Y[t] - y1) <= 1e-12 * np.linalg.norm(y1)


def test_fp32_accumulation_leaves_headroom_under_tolerance():
    """The GPU accumulates in fp32; the tolerance (1e-3 relative L2) must sit >= 10x above
    what fp32 accumulation alone costs."""
    w, L, X = _small_layer(dtype="f16", d=256, F=1024, r=16)
    ids = np.arange(0, w.d_ffn, 2)
    cache = cache_from_rows(L.bundles[ids], ids, L.b[ids], dtype=np.float16)
    for x in X[:3]:
        y64 = O.sparse_ffn(cache, x, w.d_model)
        y32 = O.sparse_ffn(cache, x, w.d_model, acc=np.float32)
        assert np.linalg.norm(y32 - y64) <= 1e-4 * np.linalg.norm(y64)


# ----------------------------------------------------------------------------- predictor
def test_predictor_hand_worked():
    g = golden("predictor_tiny.json")
    z = O.predictor_logits(g["x"], g["A"], g["B"], g["c"])
    np.testing.assert_array_equal(z, g["z"])
    mask, margin = O.predict_mask(g["x"], g["A"], g["B"], g["c"], g["theta"])
    assert list(mask) == g["mask"]
    assert margin == 0.0                      # z = 0 entries sit on the threshold: not active
    assert list(O.pack_mask(mask)) == g["packed"]


def test_pack_mask_bit_order():
    m = np.zeros(24, bool)
    m[[0, 9, 23]] = True
    assert list(O.pack_mask(m)) == [0x01, 0x02, 0x80]
    assert (O.unpack_mask(O.pack_mask(m), 24) == m).all()


def test_full_rank_predictor_reproduces_true_mask():
    """With r = d the truncated SVD is exact, so x A B = W x and, with c = b, the predicted
    mask is the true mask; the sparse FFN over the predicted set is then the dense FFN."""
    w = wl.scaled(wl.WORKLOADS["C1"], d_model=48, d_ffn=160, rank=48, p_active=0.1, dtype="f32",
                  capacity_rows=160)
    L = wl.make_layer(w)
    A64 = np.linalg.svd(L.w_up.astype(np.float64), full_matrices=False)[2].T   # [d, d]
    B64 = A64.T @ L.w_up.astype(np.float64).T
    X = wl.make_inputs(w, tokens=6)
    for x in X:
        mask, margin = O.predict_mask(x, A64, B64, L.b, 0.0)
        assert margin > 1e-9
        tm = O.true_mask(L.w_up, L.b, x)
        assert (mask == tm).all()
        ids = np.flatnonzero(mask)
        cache = cache_from_rows(L.bundles[ids], ids, L.b[ids])
        y = O.sparse_ffn(cache, x, w.d_model)
        y_dense = O.dense_ffn(L.w_up, L.w_down, L.b, x)
        assert np.linalg.norm(y - y_dense) <= 1e-12 * np.linalg.norm(y_dense)


def test_threshold_extremes_and_strictness():
    w, L, X = _small_layer()
    m, _ = O.predict_mask(X[0], L.A, L.B, L.c, -np.inf)
    assert m.all()
    m, _ = O.predict_mask(X[0], L.A, L.B, L.c, np.inf)
    assert not m.any()
    # strict comparison: a logit equal to the threshold is inactive
    A = np.eye(2); B = np.array([[1.0, 0, 0, 0, 0, 0, 0, 0], [0, 1.0, 0, 0, 0, 0, 0, 0]])
    m, _ = O.predict_mask([0.5, 0.75], A, B, None, 0.5)
    assert list(m[:2]) == [False, True]


def test_threshold_is_the_fp32_value_the_abi_carries():
    """theta crosses the C ABI as a float: both predictors compare against theta rounded to fp32 (0.1 rounds up
    to 0.100000001490116...), so a logit between the fp64 and the fp32 value of 0.1 is inactive, and the margin
    is measured from the rounded value."""
    th32 = float(np.float32(0.1))
    assert 0.1 < 0.1000000005 < th32
    z = [0.1000000005, 0.2]
    A = np.eye(2); B = np.array([[1.0, 0, 0, 0, 0, 0, 0, 0], [0, 1.0, 0, 0, 0, 0, 0, 0]])
    c = np.array([0, 0, 9, 9, 9, 9, 9, 9.0])
    m, margin = O.predict_mask(z, A, B, c, 0.1)
    assert list(m[:2]) == [False, True]
    assert margin == th32 - 0.1000000005
    gate = np.eye(2)
    m, margin, act = O.gate_predict_mask(z, gate, np.zeros(2), 0.1)
    assert list(m) == [False, True]
    assert margin == th32 - 0.1000000005
    assert list(act) == z                                       # the activation is relu(a), whatever theta is
    # infinite thresholds have no margin to report
    assert O.gate_predict_mask(z, gate, np.zeros(2), np.inf)[1] == float("inf")
    assert O.gate_predict_mask(z, gate, np.zeros(2), -np.inf)[0].all()


def test_batch_masks_and_step_mask():
    w, L, X = _small_layer()
    M, _ = O.predict_mask(X[:4], L.A, L.B, L.c, 0.0)
    for t in range(4):
        m, _ = O.predict_mask(X[t], L.A, L.B, L.c, 0.0)
        assert (M[t] == m).all()
    sm = O.step_mask(M)
    assert (sm == (M[0] | M[1] | M[2] | M[3])).all()


def test_calibrated_rates_match_closed_form():
    """Workload calibration: for stationary N(0, I) inputs the true and the predicted firing
    rates both equal p (normal quantile); AR(1) keeps unit variance since rho^2 + (1-rho^2) = 1."""
    w = wl.scaled(wl.WORKLOADS["C1"], tokens=400)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    assert abs(X.astype(np.float64).var() - 1.0) < 0.05
    M, _ = O.predict_mask(X, L.A, L.B, L.c, L.theta)
    T = np.stack([O.true_mask(L.w_up, L.b, x) for x in X])
    n = M.size
    tol = 6 * np.sqrt(w.p_active * (1 - w.p_active) / n) * 6   # tokens are correlated: wide band
    assert abs(M.mean() - w.p_active) < tol
    assert abs(T.mean() - w.p_active) < tol
    assert abs(norm.cdf(norm.ppf(1 - w.p_active)) - (1 - w.p_active)) < 1e-12


# ----------------------------------------------------------------------------- window
def test_window_hand_worked():
    g = golden("window_k3.json")
    win = O.SlidingWindow(g["d_ffn"], g["k"])
    for t, ids in enumerate(g["masks"]):
        m = np.zeros(g["d_ffn"], bool)
        m[ids] = True
        added, removed = win.push(m)
        assert list(added) == g["added"][t]
        assert list(removed) == g["removed"][t]
        assert list(np.flatnonzero(win.active_set())) == g["active"][t]


@pytest.mark.parametrize("k", [1, 2, 5, 100])
def test_window_equals_bruteforce_union_of_last_k(k):
    rng = np.random.default_rng(7)
    F, T = 96, 40
    sets = [set(np.flatnonzero(rng.random(F) < 0.08).tolist()) for _ in range(T)]
    win = O.SlidingWindow(F, k)
    prev = set()
    for t, s in enumerate(sets):
        m = np.zeros(F, bool)
        m[list(s)] = True
        added, removed = win.push(m)
        cur = set().union(*sets[max(0, t - k + 1):t + 1])
        assert set(np.flatnonzero(win.active_set()).tolist()) == cur
        assert list(added) == sorted(cur - prev)
        assert list(removed) == sorted(prev - cur)
        assert set(added.tolist()) <= s and not (set(removed.tolist()) & s)
        assert len(cur) == len(prev) + len(added) - len(removed)
        if t == 0:
            assert list(added) == sorted(s)          # the cache starts empty (Section 3.3)
        if k == 1:
            assert cur == s
        if k >= T:
            assert len(removed) == 0
        prev = cur


def test_window_overflow_leaves_state_unchanged():
    win = O.SlidingWindow(16, 2)
    m1 = np.zeros(16, bool); m1[[1, 2, 3]] = True
    win.push(m1, capacity=4)
    m2 = np.zeros(16, bool); m2[[4, 5]] = True
    with pytest.raises(OverflowError):
        win.push(m2, capacity=4)
    assert list(np.flatnonzero(win.active_set())) == [1, 2, 3]
    m3 = np.zeros(16, bool); m3[[4]] = True
    added, removed = win.push(m3, capacity=4)
    assert list(added) == [4] and list(removed) == []


# ----------------------------------------------------------------------------- cache
def test_delete_hand_worked_cases():
    for case in golden("delete_cases.json")["cases"]:
        ptr = case["pointers"]
        rows = np.array([[p, p + 0.5, -p] for p in ptr], dtype=np.float32).reshape(len(ptr), 3)
        cache = cache_from_rows(rows, ptr, [p * 0.25 for p in ptr])
        moved = O.delete_neurons(cache, case["removed"])
        n = cache.num_used
        assert list(cache.pointers[:n]) == case["after"]
        assert moved == case["moved"]
        for s in range(n):                         # rows and scalars travel with their pointer
            p = cache.pointers[s]
            assert list(cache.matrix[s]) == [p, p + 0.5, -p]
            assert cache.bias[s] == p * 0.25


def test_delete_matches_parallel_statement_and_bounds():
    """Equivalent closed statement: with n' = n - c, the dead slots below n' (ascending) are
    filled by the live slots at or above n' (descending).  At most c rows move, all into
    slots below n' (Section 3.3 item 1: rewrite of order c x d_model)."""
    rng = np.random.default_rng(3)
    for trial in range(200):
        n = int(rng.integers(0, 40))
        ptr = rng.permutation(1000)[:n].astype(np.int32)
        dead = rng.random(n) < rng.choice([0.0, 0.2, 0.6, 1.0])
        removed = ptr[dead]
        rows = np.stack([ptr, ptr * 2], axis=1).astype(np.float32).reshape(n, 2)
        cache = cache_from_rows(rows, ptr, ptr.astype(np.float32), capacity=64)
        before = cache.pointers[:n].copy()
        moved = O.delete_neurons(cache, removed)
        c = int(dead.sum()); n2 = n - c
        assert cache.num_used == n2
        holes = [s for s in range(n2) if dead[s]]
        fillers = [s for s in range(n2, n) if not dead[s]]
        assert len(holes) == len(fillers) == moved <= c
        expect = before.copy()
        for j, hslot in enumerate(holes):
            expect[hslot] = before[fillers[len(fillers) - 1 - j]]
        assert list(cache.pointers[:n2]) == list(expect[:n2])
        assert set(cache.pointers[:n2].tolist()) == set(before.tolist()) - set(removed.tolist())
        untouched = [s for s in range(n2) if not dead[s]]
        assert (cache.pointers[untouched] == before[untouched]).all()


def test_insert_appends_without_moving_rows_and_counts_bytes():
    w, L, _ = _small_layer()
    cache = O.NeuronCache(32, L.bundles.shape[1], L.bundles.dtype)
    first = np.array([3, 7, 20], np.int32)
    assert O.insert_neurons(cache, first, L.bundles, L.b) == 3 * w.bundle_bytes
    snap = cache.matrix[:3].copy()
    second = np.array([1, 100], np.int32)
    assert O.insert_neurons(cache, second, L.bundles, L.b) == 2 * w.bundle_bytes
    assert (cache.matrix[:3] == snap).all()
    assert list(cache.pointers[:5]) == [3, 7, 20, 1, 100]
    for s in range(5):
        i = cache.pointers[s]
        assert cache.matrix[s].tobytes() == L.bundles[i].tobytes()
        assert cache.bias[s] == L.b[i]
    with pytest.raises(OverflowError):
        O.insert_neurons(cache, np.arange(100, 130, dtype=np.int32), L.bundles, L.b)


# ----------------------------------------------------------------------------- whole path
def _run_layer(w, L, X, k=None):
    lay = O.OracleLayer(w.d_model, w.d_ffn, k or w.window_k, w.capacity_rows, w.glu,
                        L.A, L.B, L.c, L.theta, L.b, L.bundles)
    out = [lay.step(x) for x in X]
    return lay, out


def test_whole_path_invariants_C1():
    w = wl.WORKLOADS["C1"]
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    lay = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, w.glu,
                        L.A, L.B, L.c, L.theta, L.b, L.bundles)
    history = []
    total = 0
    for t, x in enumerate(X):
        r = lay.step(x)
        history.append(set(np.flatnonzero(r["masks"]).tolist()))
        S = set().union(*history[max(0, t - w.window_k + 1):])
        n = lay.cache.num_used
        ptr = lay.cache.pointers[:n]
        assert n == len(S) and set(ptr.tolist()) == S and len(set(ptr.tolist())) == n
        assert r["loaded"] == len(r["added"]) * w.bundle_bytes       # bytes = new neurons x bundle
        total += r["loaded"]
        assert (lay.cache.matrix[:n] == L.bundles[ptr]).all()
        assert (lay.cache.bias[:n] == L.b[ptr]).all()
        # FFN over the cache = dense FFN restricted to the cached neurons
        if t % 16 == 5:
            only = np.zeros(w.d_ffn, bool); only[ptr] = True
            yd = O.dense_ffn(L.w_up, L.w_down, L.b, x, only=only)
            assert np.linalg.norm(r["y"] - yd) <= 1e-12 * np.linalg.norm(yd)
    assert lay.bytes_loaded == total
    assert lay.min_margin > 1e-9
    first = len(history[0])
    assert lay.bytes_loaded >= first * w.bundle_bytes                # first token loads its whole mask


def test_bytes_and_occupancy_monotone_in_window_size():
    """Larger windows load fewer bytes per token and hold more rows (Section 3.1)."""
    w = wl.WORKLOADS["C1"]
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    loaded, held = [], []
    for k in (1, 2, 4, 8, 64):
        lay, out = _run_layer(w, L, X, k)
        loaded.append(lay.bytes_loaded)
        held.append(np.mean([o["num_used"] for o in out]))
    assert all(a >= b for a, b in zip(loaded, loaded[1:]))
    assert all(a <= b for a, b in zip(held, held[1:]))
    # k >= T: every neuron is loaded exactly once
    lay, out = _run_layer(w, L, X, 64)
    union = set()
    for o in out:
        union |= set(np.flatnonzero(o["masks"]).tolist())
    assert lay.bytes_loaded == len(union) * w.bundle_bytes


# ----------------------------------------------------------------------------- dynamic window
def test_dynamic_window_hand_worked():
    g = golden("window_shrink.json")
    win = O.SlidingWindow(g["d_ffn"], g["k"])
    for t, ids in enumerate(g["masks"]):
        m = np.zeros(g["d_ffn"], bool)
        m[ids] = True
        if g["active"][t] is None:
            before = list(np.flatnonzero(win.active_set()))
            with pytest.raises(OverflowError):
                win.push(m, capacity=g["capacity"], shrink=True)
            assert list(np.flatnonzero(win.active_set())) == before
            continue
        added, removed = win.push(m, capacity=g["capacity"], shrink=True)
        assert list(added) == g["added"][t] and list(removed) == g["removed"][t]
        assert list(np.flatnonzero(win.active_set())) == g["active"][t]
        assert len(win.masks) == g["window_len"][t]


def test_dynamic_window_is_the_largest_suffix_that_fits():
    """Against set arithmetic: after each step the window is the longest suffix of (previous window + new
    mask, at most k long) whose union fits; the active set never exceeds the capacity; with a capacity
    that is never reached the dynamic window equals the fixed one."""
    rng = np.random.default_rng(11)
    F, T, k, cap = 128, 60, 5, 30
    sets = [set(np.flatnonzero(rng.random(F) < rng.choice([0.03, 0.08, 0.15])).tolist()) for _ in range(T)]
    win, ref_win, fixed = O.SlidingWindow(F, k), [], O.SlidingWindow(F, k)
    for t, s in enumerate(sets):
        m = np.zeros(F, bool)
        m[list(s)] = True
        ref_win = (ref_win + [s])[-k:]
        while len(ref_win) > 1 and len(set().union(*ref_win)) > cap:
            ref_win = ref_win[1:]
        if len(set().union(*ref_win)) > cap:
            pytest.skip("mask alone above capacity: not the case under test")
        prev = set(np.flatnonzero(win.active_set()).tolist())
        added, removed = win.push(m, capacity=cap, shrink=True)
        cur = set().union(*ref_win)
        assert set(np.flatnonzero(win.active_set()).tolist()) == cur and len(cur) <= cap
        assert len(win.masks) == len(ref_win)
        assert list(added) == sorted(cur - prev) and list(removed) == sorted(prev - cur)
        a2, r2 = fixed.push(m, capacity=F, shrink=True)       # never shrinks
        assert len(fixed.masks) == min(k, t + 1)


# ----------------------------------------------------------------------------- several tokens per step
def test_window_tokens_hand_worked():
    g = golden("window_tokens.json")
    F = g["d_ffn"]
    win = O.SlidingWindow(F, g["k"])
    for p in g["passes"]:
        M = np.zeros((len(p["masks"]), F), bool)
        for i, ids in enumerate(p["masks"]):
            M[i, ids] = True
        added, removed = win.push_tokens(M, p["keep"])
        assert list(added) == p["added"] and list(removed) == p["removed"]
        assert list(np.flatnonzero(win.active_set())) == p["active"]
        assert len(win.masks) == p["window_len"]


def test_window_tokens_reduces_to_single_pushes():
    """keep = all tokens: the set held after the pass is the one that single pushes end with (union of the
    last k token masks); one token with keep = 1 is the ordinary push; keep = 0 leaves the window alone."""
    rng = np.random.default_rng(5)
    F, k = 64, 4
    a, b = O.SlidingWindow(F, k), O.SlidingWindow(F, k)
    for p in range(12):
        M = rng.random((3, F)) < 0.1
        a.push_tokens(M, 3)
        for m in M:
            b.push(m)
        assert (a.active_set() == b.active_set()).all()
    c, d = O.SlidingWindow(F, k), O.SlidingWindow(F, k)
    for p in range(12):
        m = rng.random(F) < 0.1
        r1 = c.push_tokens(m[None, :], 1)
        r2 = d.push(m)
        assert list(r1[0]) == list(r2[0]) and list(r1[1]) == list(r2[1])
    held = [x.copy() for x in c.masks]
    M = rng.random((2, F)) < 0.2
    c.push_tokens(M, 0)
    assert all((x == y).all() for x, y in zip(held, c.masks))
    assert (c.active_set() == (np.logical_or.reduce(held) | M[0] | M[1])).all()
    c.push_tokens(np.zeros((1, F), bool), 0)                       # the transient masks are gone again
    assert (c.active_set() == np.logical_or.reduce(held)).all()


def test_window_tokens_dynamic_hand_worked():
    g = golden("window_tokens_shrink.json")
    F = g["d_ffn"]
    win = O.SlidingWindow(F, g["k"])
    for p in g["passes"]:
        M = np.zeros((len(p["masks"]), F), bool)
        for i, ids in enumerate(p["masks"]):
            M[i, ids] = True
        if p.get("overflow"):
            with pytest.raises(OverflowError):
                win.push_tokens(M, p["keep"], g["capacity"], shrink=True)
        else:
            added, removed = win.push_tokens(M, p["keep"], g["capacity"], shrink=True)
            assert list(added) == p["added"] and list(removed) == p["removed"]
        assert list(np.flatnonzero(win.active_set())) == p["active"]
        assert len(win.masks) == p["window_len"]


def test_window_tokens_dynamic_is_the_longest_suffix_that_fits():
    """Brute force with Python sets: after a pass the window is the longest suffix of (old window, kept tokens), at
    most k masks, whose union with the masks of the pass fits; dropped masks never return; with room to spare
    the dynamic form is the fixed one; a pass of one kept token is the single-token dynamic push."""
    rng = np.random.default_rng(11)
    F, k, cap = 96, 5, 30
    win, fixed, big = O.SlidingWindow(F, k), O.SlidingWindow(F, k), O.SlidingWindow(F, k)
    ref = []                                            # list of sets, oldest first
    held_before = set()
    shrunk = 0
    for p in range(60):
        ntok = int(rng.integers(1, 5))
        keep = int(rng.integers(0, ntok + 1))
        M = rng.random((ntok, F)) < 0.07
        sets = [set(np.flatnonzero(m).tolist()) for m in M]
        T = set().union(*sets)
        cand = (ref + sets[:keep])[-k:]
        best = None
        for a in range(len(cand), -1, -1):              # longest suffix first
            u = set(T)
            for sset in cand[len(cand) - a:]:
                u |= sset
            if len(u) <= cap:
                best = (cand[len(cand) - a:], u)
                break
        if best is None:
            with pytest.raises(OverflowError):
                win.push_tokens(M, keep, cap, shrink=True)
            continue
        shrunk += len(best[0]) < len(cand)
        added, removed = win.push_tokens(M, keep, cap, shrink=True)
        ref = best[0]
        assert set(np.flatnonzero(win.active_set()).tolist()) == best[1]
        assert len(win.masks) == len(ref)
        assert all(set(np.flatnonzero(m).tolist()) == sset for m, sset in zip(win.masks, ref))
        assert list(added) == sorted(best[1] - held_before) and list(removed) == sorted(held_before - best[1])
        held_before = best[1]
        a1 = fixed.push_tokens(M, keep)
        a2 = big.push_tokens(M, keep, F, shrink=True)
        assert list(a1[0]) == list(a2[0]) and list(a1[1]) == list(a2[1])
    assert shrunk > 5, "the capacity never bound"
    a, b = O.SlidingWindow(F, k), O.SlidingWindow(F, k)
    for p in range(30):
        m = rng.random(F) < 0.12
        r1 = a.push_tokens(m[None, :], 1, cap, shrink=True)
        r2 = b.push(m, cap, shrink=True)
        assert list(r1[0]) == list(r2[0]) and list(r1[1]) == list(r2[1]) and len(a.masks) == len(b.masks)


# ----------------------------------------------------------------------------- resident gate as predictor
def _gate_layer(g, theta, k=2):
    gate, up, down = (np.array(g[n], np.float32) for n in ("gate", "up", "down"))
    b = np.array(g["b"], np.float32)
    bundles = np.concatenate([up, down], axis=1)
    return O.OracleLayer(2, 3, k, 3, False, None, None, None, theta, b, bundles, w_gate=gate)


def test_gate_predictor_hand_worked():
    """Appendix (Llama 2, alternative approaches): mask from the resident gate, bundles = up | down."""
    g = golden("gate_tiny.json")
    x = np.array(g["x"])
    for case in g["cases"]:
        lay = _gate_layer(g, case["theta"])
        r = lay.step(x)
        assert r["masks"].astype(int).tolist() == case["mask"]
        assert lay.min_margin == case["margin"]                         # min |a - theta|, worked by hand
        assert r["added"].tolist() == [i for i, m in enumerate(case["mask"]) if m]
        assert r["loaded"] == sum(case["mask"]) * 2 * 2 * 4           # up | down of d = 2 fp32 values
        np.testing.assert_allclose(r["y"], case["y"], rtol=0, atol=1e-12)
    # second token at theta = 0: neurons 0 and 1 fire (a = 2.5, 2.0); neuron 0 stays cached, 1 is loaded
    lay = _gate_layer(g, 0.0)
    lay.step(x)
    r = lay.step(np.array(g["second_x"]))
    assert r["added"].tolist() == [1] and r["removed"].tolist() == []
    np.testing.assert_allclose(lay.gate_act, np.maximum(g["second_a"], 0), rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["y"], g["second_y_theta0"], rtol=0, atol=1e-12)


def test_gate_predictor_reproduces_the_dense_gated_ffn():
    """The gate decides exactly which neurons fire, so at theta = 0 the windowed sparse path equals the
    dense gated FFN on every token (cached neurons that do not fire contribute exactly zero), and the
    bytes moved per new neuron are two thirds of the gate | up | down bundle."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="gate", d_model=64, d_ffn=192, rank=8, window_k=3, p_active=0.1,
                  glu=True, gate_resident=True, tokens=12, capacity_rows=192)
    wfull = wl.scaled(w, gate_resident=False)
    L = wl.make_layer(w)
    assert L.bundles.shape[1] == 2 * w.d_model and w.bundle_bytes * 3 == wfull.bundle_bytes * 2
    assert (L.bundles[:, :w.d_model] == L.w_up).all() and (L.bundles[:, w.d_model:] == L.w_down).all()
    lay = O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, False, None, None, None, 0.0, L.b,
                        L.bundles, w_gate=L.w_gate)
    for x in wl.make_inputs(w):
        r = lay.step(x)
        assert (r["masks"] == O.true_mask(L.w_gate, L.b, x)).all()
        dense = O.dense_ffn(L.w_up, L.w_down, L.b, x, w_gate=L.w_gate)
        np.testing.assert_allclose(r["y"], dense, rtol=1e-11, atol=1e-13)
        assert r["loaded"] == len(r["added"]) * w.bundle_bytes


def test_gate_predictor_batch_rows_equal_single_token_evaluation():
    """Several tokens per step with the resident gate as predictor: every token has its own gate activations, the
    step mask is the OR of the per-token masks, and row t of y is the dense gated FFN of token t (exact predictor:
    cached neurons that do not fire for token t contribute exactly zero), also in a pass of tokens of which only
    some stay in the window (Section 4.3)."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="gateb", d_model=48, d_ffn=160, rank=8, window_k=3, p_active=0.1,
                  glu=True, gate_resident=True, tokens=12, batch=3, capacity_rows=160)
    L = wl.make_layer(w)
    X = wl.make_batch_inputs(w)                                   # [T, 3, d]
    mk = lambda: O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, False, None, None, None, 0.0, L.b,
                               L.bundles, w_gate=L.w_gate)
    lay = mk()
    for xb in X[:6]:
        r = lay.step(xb)
        assert r["masks"].shape == (3, w.d_ffn) and r["y"].shape == (3, w.d_model)
        held = lay.window.active_set()
        for t in range(3):
            m1, _, act1 = O.gate_predict_mask(xb[t], L.w_gate, L.b, 0.0)
            assert (r["masks"][t] == m1).all() and (m1 <= held).all()
            np.testing.assert_allclose(lay.gate_act[t], act1, rtol=1e-12, atol=1e-14)   # matrix and vector products round apart
            dense = O.dense_ffn(L.w_up, L.w_down, L.b, xb[t], w_gate=L.w_gate)
            np.testing.assert_allclose(r["y"][t], dense, rtol=1e-11, atol=1e-13)
    lay = mk()
    for xb, keep in zip(X[6:], (3, 1, 0, 2, 3, 0)):
        r = lay.step_tokens(xb, keep)
        for t in range(3):
            dense = O.dense_ffn(L.w_up, L.w_down, L.b, xb[t], w_gate=L.w_gate)
            np.testing.assert_allclose(r["y"][t], dense, rtol=1e-11, atol=1e-13)


def test_layer_pass_of_tokens_equals_the_dense_ffn_restricted_to_the_held_set():
    """OracleLayer.step_tokens (Section 4.3): every token of a pass is computed over the same held set (kept
    window masks and all masks of the pass), so row i of y is the dense FFN restricted to that set; a pass of one
    kept token is the ordinary step; bytes loaded = |added| x bundle bytes."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="spec", d_model=48, d_ffn=128, rank=8, window_k=3, p_active=0.1,
                  tokens=40, capacity_rows=128)
    L = wl.make_layer(w)
    X = wl.make_inputs(w)
    mk = lambda: O.OracleLayer(w.d_model, w.d_ffn, w.window_k, w.capacity_rows, False, L.A, L.B, L.c, 0.0, L.b,
                               L.bundles)
    lay = mk()
    pos = 0
    for keep in (4, 2, 0, 1, 4, 3):
        xb = X[pos:pos + 4]
        pos += 4
        r = lay.step_tokens(xb, keep)
        held = lay.window.active_set()
        assert set(lay.cache.pointers[:lay.cache.num_used].tolist()) == set(np.flatnonzero(held).tolist())
        assert r["loaded"] == len(r["added"]) * w.bundle_bytes
        for i in range(4):
            assert (r["masks"][i] <= held).all()                     # every token's own mask is held
            ref = O.dense_ffn(L.w_up, L.w_down, L.b, xb[i], only=held)
            np.testing.assert_allclose(r["y"][i], ref, rtol=1e-11, atol=1e-13)
    a, b = mk(), mk()
    for x in X[:10]:
        ra, rb = a.step_tokens(x[None, :], 1), b.step(x)
        assert ra["added"].tolist() == rb["added"].tolist() and ra["removed"].tolist() == rb["removed"].tolist()
        assert (a.cache.pointers == b.cache.pointers).all()
        np.testing.assert_array_equal(ra["y"][0], rb["y"])
