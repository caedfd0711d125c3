"""The pins must notice a plausible mistake anywhere in the oracle.  Each case below plants one
mistake in a private copy of the oracle module (on the CPU, never in the HIP path) and checks that
at least one of the pin tests fails on the mutant while passing on the real oracle."""
import importlib.util
import os
import sys
import types

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = os.path.join(ROOT, "oracle", "sdllm_oracle.py")

MUTATIONS = {
    # name: (text to replace, replacement)
    "scale_dropped": ("scale = 1.0 / math.sqrt(d) if scale is None else scale\n    cand =", "scale = 1.0\n    cand ="),
    "candidates_include_block": ("np.arange(block_off + block_len, seq_len)", "np.arange(block_off, seq_len)"),
    "softmax_over_queries_axis": ("a = a - a.max(axis=-1, keepdims=True)\n            e = np.exp(a)\n            w = e / e.sum(axis=-1, keepdims=True)",
                                  "a = a - a.max(axis=1, keepdims=True)\n            e = np.exp(a)\n            w = e / e.sum(axis=1, keepdims=True)"),
    "pool_window_off_by_one": ("lo, hi = max(0, c - half), min(n, c + half + 1)", "lo, hi = max(0, c - half), min(n, c + half)"),
    "ties_to_higher_position": ("key=lambda c: (-values[c], c)", "key=lambda c: (-values[c], -c)"),
    "smallest_instead_of_largest": ("key=lambda c: (-values[c], c)", "key=lambda c: (values[c], c)"),
    "floor_instead_of_ceil": ("k = math.ceil(x - 1e-9) if k_rounding == CEIL else math.floor(x + 1e-9)", "k = math.floor(x + 1e-9)"),
    "no_rounding_guard": ("k = math.ceil(x - 1e-9) if k_rounding == CEIL else math.floor(x + 1e-9)",
                          "k = math.ceil(x) if k_rounding == CEIL else math.floor(x)"),
    "suffix_positions_not_shifted": ("return cand[keep], int((keep < n_pre).sum())", "return keep, int((keep < n_pre).sum())"),
    "seam_ignored_in_per_segment": ("    if select_mode == JOINT:\n        return pool_1d(score, s, kind)\n", "    if True:\n        return pool_1d(score, s, kind)\n"),
    "gqa_head_mapping": ("        g = h // grp\n        a = (q[h] @ k[g].T) * scale", "        g = h % hkv\n        a = (q[h] @ k[g].T) * scale"),
    "values_transposed_heads": ("out[h] = p @ v[g]", "out[h] = p @ v[hkv - 1 - g]"),
    "attention_scale_squared": ("a = (q[h] @ k[g].T) * scale\n        a = a - a.max", "a = (q[h] @ k[g].T) * scale * scale\n        a = a - a.max"),
    "concat_block_first": ("k = np.concatenate([k_cache, k_blk], axis=1)\n    v = np.concatenate([v_cache, v_blk], axis=1)",
                           "k = np.concatenate([k_blk, k_cache], axis=1)\n    v = np.concatenate([v_cache, v_blk], axis=1)"),
    "delay_off_by_one": ("    if step_in_block > delay:\n        return 2\n    if step_in_block == delay:", "    if step_in_block >= delay:\n        return 2\n    if step_in_block == delay - 1:"),
    "mean_over_heads_dropped": ("return per_head.reshape(hkv, grp, -1).mean(axis=1)", "return per_head.reshape(hkv, grp, -1)[:, 0]"),
    "avg_pool_divides_by_window": ("out[c] = x[lo:hi].sum() / s", "out[c] = x[lo:hi].sum() / (hi - lo)"),
    "compaction_uses_keys_for_values": ("v_c = np.stack([v_full[g][idx[g]] for g in range(hkv)])", "v_c = np.stack([k_full[g][idx[g]] for g in range(hkv)])"),
    "prefix_only_drops_suffix": ("idx = np.concatenate([idx, np.broadcast_to(suffix, (hkv, suffix.size))], axis=1)", "idx = idx"),
}


def _load_mutant(name):
    src = open(ORACLE_SRC).read()
    if name is not None:
        old, new = MUTATIONS[name]
        assert src.count(old) >= 1, f"mutation target for {name} not found"
        src = src.replace(old, new, 1)
    mod = types.ModuleType("oracle.sdllm_oracle")
    mod.__file__ = ORACLE_SRC
    exec(compile(src, ORACLE_SRC, "exec"), mod.__dict__)
    return mod


def _pin_functions():
    """All pin tests of the two oracle test modules, as (name, callable taking the golden reader)."""
    from tests import conftest, test_oracle_attention, test_oracle_select
    out = []
    for m in (test_oracle_select, test_oracle_attention):
        for n in dir(m):
            if not n.startswith("test_") or "workload" in n or "even_pool" in n:
                continue
            f = getattr(m, n)
            marks = getattr(f, "pytestmark", [])
            params = [mk for mk in marks if mk.name == "parametrize"]
            out.append((m, n, f, params))
    return out, conftest.read_golden


def _run_all_pins(oracle_module):
    """Run every pin with `orc` swapped for the given module; returns the names that failed."""
    pins, golden = _pin_functions()
    failed = []
    for m, n, f, params in pins:
        saved = m.orc
        m.orc = oracle_module
        try:
            argnames = f.__code__.co_varnames[:f.__code__.co_argcount]
            if params:
                names = [a.strip() for a in params[0].args[0].split(",")]
                for vals in params[0].args[1]:
                    vals = vals if isinstance(vals, (tuple, list)) and len(names) > 1 else (vals,)
                    kw = dict(zip(names, vals))
                    if "golden" in argnames:
                        kw["golden"] = golden
                    f(**kw)
            elif "golden" in argnames:
                f(golden)
            else:
                f()
        except Exception:   # an assertion or an exception both count as "noticed"
            failed.append(n)
        finally:
            m.orc = saved
    return failed


def test_the_unmutated_oracle_passes_every_pin():
    assert _run_all_pins(_load_mutant(None)) == []


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    failed = _run_all_pins(_load_mutant(name))
    assert failed, f"no pin noticed the planted mistake '{name}'"
