"""Do the pins bite?  Each case plants one plausible mistake (a dropped term, a flipped sign, an index or an
order off by one) in a copy of the oracle's source, on the CPU, and checks that a named pin fails against it.
The real oracle is untouched."""
import os
import types

import pytest

from oracle import lif_oracle as O
from tests import test_oracle_pins as pins

SRC = open(os.path.join(os.path.dirname(O.__file__), "lif_oracle.py")).read()

# (what is planted, text in the oracle, replacement, pin that must fail, its arguments)
MUTATIONS = [
    ("predictor: > becomes >=", "mask = z > th", "mask = z >= th", "test_threshold_extremes_and_strictness", ()),
    ("predictor: offset dropped", "        z = z + np.asarray(c, dtype=np.float64)", "        z = z",
     "test_predictor_hand_worked", ()),
    ("predictor: offset sign", "        z = z + np.asarray(c, dtype=np.float64)",
     "        z = z - np.asarray(c, dtype=np.float64)", "test_full_rank_predictor_reproduces_true_mask", ()),
    ("window: one mask too many", "kept = self.masks[-(self.k - 1):] if self.k > 1 else []",
     "kept = self.masks[-self.k:]", "test_window_hand_worked", ()),
    ("window: one mask too few", "kept = self.masks[-(self.k - 1):] if self.k > 1 else []",
     "kept = self.masks[-(self.k - 2):] if self.k > 2 else []", "test_window_equals_bruteforce_union_of_last_k", (5,)),
    ("dynamic window: drops a newer mask",
     "int(union(new_masks).sum()) > capacity:\n                new_masks.pop(0)",
     "int(union(new_masks).sum()) > capacity:\n                new_masks.pop(-2 if len(new_masks) > 1 else 0)",
     "test_dynamic_window_hand_worked", ()),
    ("dynamic window: shrinks once too often",
     "while len(new_masks) > 1 and int(union(new_masks).sum()) > capacity:",
     "while len(new_masks) > 1 and int(union(new_masks).sum()) >= capacity:",
     "test_dynamic_window_is_the_largest_suffix_that_fits", ()),
    ("delete: bias stays behind", "        cache.bias[lo] = cache.bias[hi]\n", "", "test_delete_hand_worked_cases", ()),
    ("delete: pointer stays behind", "        cache.pointers[lo] = cache.pointers[hi]\n", "",
     "test_delete_matches_parallel_statement_and_bounds", ()),
    ("insert: descending ids", "    for j, i in enumerate(added):", "    for j, i in enumerate(list(added)[::-1]):",
     "test_insert_appends_without_moving_rows_and_counts_bytes", ()),
    ("insert: bias of the slot, not of the neuron", "        cache.bias[n + j] = b[i]",
     "        cache.bias[n + j] = b[min(n + j, len(b) - 1)]", "test_whole_path_invariants_C1", ()),
    ("insert: bytes per element", "    return a * host_bundles.shape[1] * host_bundles.dtype.itemsize",
     "    return a * host_bundles.shape[1]", "test_insert_appends_without_moving_rows_and_counts_bytes", ()),
    ("ffn: no relu", "        h = np.maximum(x @ up.T + bias, 0)\n", "        h = x @ up.T + bias\n",
     "test_all_rows_cached_equals_dense_and_empty_cache_is_zero", ()),
    ("ffn: no bias", "        h = np.maximum(x @ up.T + bias, 0)\n", "        h = np.maximum(x @ up.T, 0)\n",
     "test_sparse_over_true_set_equals_dense", (False, "f32")),
    ("ffn: gate and up swapped", "        h = np.maximum(x @ gate.T + bias, 0) * (x @ up.T)",
     "        h = np.maximum(x @ up.T + bias, 0) * (x @ gate.T)", "test_sparse_over_true_set_equals_dense", (True, "f16")),
    ("ffn: halves of the bundle swapped", "        up, down = rows[:, :d], rows[:, d:]\n",
     "        down, up = rows[:, :d], rows[:, d:]\n", "test_ffn_hand_worked", (None,)),
    ("bundle bytes: gate row forgotten", "return (3 if glu else 2) * d_model * num_bytes",
     "return 2 * d_model * num_bytes", "test_bundle_size_matches_paper_constants", ()),
    ("gate predictor: activation not rectified", "return a > th, margin, np.maximum(a, 0.0)",
     "return a > th, margin, a", "test_gate_predictor_reproduces_the_dense_gated_ffn", ()),
    ("gate predictor: margin measured from zero, not from theta",
     "    margin = float(np.min(np.abs(a - th))) if np.isfinite(th) and a.size else float(\"inf\")",
     "    margin = float(np.min(np.abs(a))) if np.isfinite(th) and a.size else float(\"inf\")",
     "test_gate_predictor_hand_worked", ()),
    ("gate predictor: threshold not rounded to the ABI's fp32", "    th = np.float64(np.float32(theta))\n    margin = float(np.min(np.abs(a - th)))",
     "    th = np.float64(theta)\n    margin = float(np.min(np.abs(a - th)))", "test_threshold_is_the_fp32_value_the_abi_carries", ()),
    ("predictor: threshold not rounded to the ABI's fp32", "    th = np.float64(np.float32(theta))\n    mask = z > th",
     "    th = np.float64(theta)\n    mask = z > th", "test_threshold_is_the_fp32_value_the_abi_carries", ()),
    ("pass of tokens: transient masks forgotten", "        for i in range(len(masks)):                    # also one that enters and leaves the window at once\n            transient |= masks[i]",
     "        for i in range(keep, keep):\n            transient |= masks[i]",
     "test_layer_pass_of_tokens_equals_the_dense_ffn_restricted_to_the_held_set", ()),
    ("dynamic window, pass of tokens: the newest mask leaves first",
     "            while new_masks and int(held(new_masks).sum()) > capacity:\n                new_masks.pop(0)",
     "            while new_masks and int(held(new_masks).sum()) > capacity:\n                new_masks.pop(-1)",
     "test_window_tokens_dynamic_hand_worked", ()),
    ("dynamic window, pass of tokens: the masks of the pass are not counted",
     "            while new_masks and int(held(new_masks).sum()) > capacity:",
     "            while new_masks and int(np.logical_or.reduce(new_masks).sum()) > capacity:",
     "test_window_tokens_dynamic_is_the_longest_suffix_that_fits", ()),
    ("gate ffn, batch: every token takes the first token's gate activations",
     "np.asarray(gate_act, np.float64)[..., cache.pointers[:n]]",
     "np.atleast_2d(np.asarray(gate_act, np.float64))[0, cache.pointers[:n]]",
     "test_gate_predictor_batch_rows_equal_single_token_evaluation", ()),
    ("gate ffn: activation looked up by slot", "np.asarray(gate_act, np.float64)[..., cache.pointers[:n]]",
     "np.asarray(gate_act, np.float64)[..., :n]", "test_gate_predictor_reproduces_the_dense_gated_ffn", ()),
]


def _pin(name):
    fn = getattr(pins, name)
    return getattr(fn, "__wrapped__", fn)


@pytest.mark.parametrize("what,old,new,pin,args", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_its_pin(what, old, new, pin, args, monkeypatch):
    assert SRC.count(old) >= 1, "the oracle no longer contains the text this case replaces"
    mutant = types.ModuleType("lif_oracle_mutant")
    exec(compile(SRC.replace(old, new, 1), "lif_oracle_mutant", "exec"), mutant.__dict__)
    takes_fn = args == (None,)                            # the pin takes one of the oracle's own functions
    _pin(pin)(*((O.sparse_ffn,) if takes_fn else args))   # sanity: the pin passes against the real oracle
    if takes_fn:
        args = (mutant.sparse_ffn,)
    for attr in dir(mutant):
        if not attr.startswith("__") and hasattr(O, attr):
            monkeypatch.setattr(O, attr, getattr(mutant, attr))
    with pytest.raises(Exception):
        _pin(pin)(*args)
