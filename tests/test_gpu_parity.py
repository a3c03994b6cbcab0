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
    return O.OracleLayer(w.d_model, w.d_ffn, k or w.window_k, capacity or w.capacity_rows, w.glu,
                         L.A, L.B, L.c, L.theta, L.b, L.bundles)


def run_stream(w, L, X, ffn_mode=0, check_every=1):
    from tests.harness import GpuLayer, compare_step
    gpu = GpuLayer(w, L, ffn_mode=ffn_mode)
    ora = make_oracle(w, L)
    stats = []
    for t in range(len(X)):
        print(f"[{w.name}] token {t}", flush=True) if t % 32 == 0 else None
        stats.append(compare_step(gpu, ora, X[t], w, t, check_cache=(t % check_every == 0 or t == len(X) - 1)))
    cnt = gpu.layer.counters()
    assert cnt["h2d_bytes"] == ora.bytes_loaded
    assert cnt["rows_moved"] == ora.rows_moved
    assert cnt["steps"] == len(X)
    assert ora.min_margin > 1e-9
    return stats


@pytest.mark.parametrize("ffn_mode", [0, 1])
def test_c1_tiny_fp32_whole_path(ffn_mode):
    w = wl.WORKLOADS["C1"]
    stats = run_stream(w, wl.make_layer(w), wl.make_inputs(w), ffn_mode)
    assert max(s["err"] for s in stats) < 1e-5          # fp32 storage: far below the fp16 bar
    assert any(s["moved"] > 0 for s in stats) and any(s["removed"] > 0 for s in stats)


@pytest.mark.parametrize("ffn_mode", [0, 1])
@pytest.mark.parametrize("glu", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_ragged_shapes_whole_path(glu, dtype, ffn_mode):
    """Shapes that end in a partial tile everywhere: d = 71 x 8 (like 4544 = 71 x 64), F not a
    multiple of 128, rank not a power of two, capacity not a multiple of 1024."""
    w = wl.scaled(wl.WORKLOADS["C1"], name="ragged", d_model=568, d_ffn=1096, rank=40, window_k=3,
                  p_active=0.08, dtype=dtype, glu=glu, tokens=24, capacity_rows=700)
    run_stream(w, wl.make_layer(w), wl.make_inputs(w), ffn_mode)


def test_c2_opt_shape_fp16_whole_path():
    """OPT-6.7B FFN shape at full size, the launch configuration bench.py times (96 tokens)."""
    w = wl.WORKLOADS["C2"]
    L = wl.cached_layer("C2")
    X = wl.make_inputs(w, tokens=96)
    stats = run_stream(w, L, X, ffn_mode=0, check_every=8)
    assert np.mean([s["n"] for s in stats[10:]]) > 800         # window union of ~3 % active masks
    print("C2 max rel-L2 %.2e" % max(s["err"] for s in stats))


@pytest.mark.parametrize("ffn_mode", [1])
def test_c2_other_ffn_modes_match_oracle(ffn_mode):
    w = wl.WORKLOADS["C2"]
    L = wl.cached_layer("C2")
    X = wl.make_inputs(w, tokens=24)
    run_stream(w, L, X, ffn_mode=ffn_mode, check_every=8)
