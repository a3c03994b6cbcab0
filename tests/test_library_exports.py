"""The C-ABI library loads and exports every symbol include/lif.h declares (no GPU, no compute)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lif.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lif_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_hot_calls():
    syms = declared_symbols()
    for name in ("lif_predict", "lif_update_window", "lif_load_bundles", "lif_sparse_ffn",
                 "lif_create", "lif_reset", "lif_destroy"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    from paper_2312_11514_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2312_11514_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} is declared in lif.h but not exported"
    assert sorted(binding.EXPORTS) == declared_symbols()
    assert binding.load_library().lif_version() >= 1


def test_workspace_size_and_config_validation_without_gpu():
    from paper_2312_11514_amd import binding as b
    lib = b.load_library()
    ok = b.LifConfig(4096, 16384, 128, 5, 8192, 1, 0, b.LIF_F16, 0, 0, 0, 0.0)
    n = lib.lif_workspace_bytes(ctypes.byref(ok))
    assert n >= 8192 * 4 * 3 and n % 256 == 0
    bad_shapes = [
        dict(d_model=4090), dict(d_ffn=16385), dict(d_ffn=1 << 20), dict(rank=100), dict(window_k=0),
        dict(capacity_rows=0), dict(max_batch=9), dict(dtype=7), dict(glu=2), dict(ffn_mode=5), dict(shrink_window=3), dict(predictor=2), dict(predictor=1, glu=1),
    ]
    for ch in bad_shapes:
        cfg = b.LifConfig(4096, 16384, 128, 5, 8192, 1, 0, b.LIF_F16, 0, 0, 0, 0.0)
        for k, v in ch.items():
            setattr(cfg, k, v)
        assert lib.lif_workspace_bytes(ctypes.byref(cfg)) == 0, ch
    # null handles are rejected without touching a device
    assert lib.lif_reset(None, None) == b.LIF_INVALID_ARG
    assert lib.lif_destroy(None) == b.LIF_OK
    h = ctypes.c_void_p()
    assert lib.lif_create(ctypes.byref(ok), None, ctypes.byref(h)) == b.LIF_INVALID_ARG
    assert b"null" in lib.lif_last_error_string()
