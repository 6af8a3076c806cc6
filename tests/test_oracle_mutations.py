"""Plant plausible mistakes in a copy of the oracle (on the CPU) and check that
the pins notice every one of them.  This is what justifies trusting the pins.
"""
import importlib.util
import inspect
import os
import sys
import types

import pytest

import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "rpa_oracle.py")

MUTATIONS = {
    "mask_excludes_own_token": ("hidden = (j > (ctx + i))", "hidden = (j >= (ctx + i))"),
    "mask_one_too_many": ("hidden = (j > (ctx + i))", "hidden = (j > (ctx + i + 1))"),
    "mask_aligned_to_start": ("hidden = (j > (ctx + i))", "hidden = (j > i)"),
    "noncausal_flag_ignored": ("if causal else np.zeros((l_q, l_kv), dtype=bool)", "if True else None"),
    "noncausal_hides_new_tokens": ("if causal else np.zeros((l_q, l_kv), dtype=bool)",
                                   "if causal else (j >= ctx) & (j > ctx + i)"),
    "causal_flag_not_forwarded": ("res = attend_sequence(qq, kk, vv, sm_scale, heads=heads, causal=causal)",
                                  "res = attend_sequence(qq, kk, vv, sm_scale, heads=heads)"),
    "merged_causal_flag_not_forwarded": ("                              sm_scale, heads=heads, causal=causal)",
                                         "                              sm_scale, heads=heads)"),
    "merged_reads_halves_swapped": ("bf16_to_f64(rows[:, :, 0, :]), bf16_to_f64(rows[:, :, 1, :])",
                                    "bf16_to_f64(rows[:, :, 1, :]), bf16_to_f64(rows[:, :, 0, :])"),
    "merged_update_swaps_halves": ("kv_pages[pg, (ctx + t) % ps, :, 1, :] = v_new[q0 + t]",
                                   "kv_pages[pg, (ctx + t) % ps, :, 1, :] = k_new[q0 + t]"),
    "merged_update_at_wrong_position": ("pg = int(page_table[r, (ctx + t) // ps])", "pg = int(page_table[r, t // ps])"),
    "merged_gather_ignores_table": ("rows = kv_pages[np.asarray(page_table[r, :n_pages], dtype=np.int64)]",
                                    "rows = kv_pages[np.arange(n_pages)]"),
    "no_mask": ("s[hidden] = -np.inf", "pass"),
    "wrong_gqa_map": ("g = h // hg\n        s = scale", "g = h % hkv\n        s = scale"),
    "missing_scale": ("s = scale * (q[:, h, :] @ k[:, g, :].T)", "s = (q[:, h, :] @ k[:, g, :].T)"),
    "no_normalisation": ("p /= p.sum(axis=1, keepdims=True)", "pass"),
    "v_head_wrong": ("out[:, h, :] = p @ v[:, g, :]", "out[:, h, :] = p @ v[:, 0, :]"),
    "update_at_wrong_position": ("pos = ctx + t\n            pg", "pos = t\n            pg"),
    "update_wrong_slot": ("k_pages[pg, pos % ps] = k_new[q0 + t]", "k_pages[pg, t % ps] = k_new[q0 + t]"),
    "update_swaps_k_v": ("v_pages[pg, pos % ps] = v_new[q0 + t]", "v_pages[pg, pos % ps] = k_new[q0 + t]"),
    "update_ignores_seq_offset": ("k_pages[pg, pos % ps] = k_new[q0 + t]", "k_pages[pg, pos % ps] = k_new[t]"),
    "gather_ignores_table": ("ids = np.asarray(table_row[:n_pages], dtype=np.int64)",
                             "ids = np.arange(n_pages, dtype=np.int64)"),
    "no_update_before_attend": ("        update_cache(k_new, v_new, k_pages, v_pages, page_table, cu_q_lens, kv_lens, num_seqs)\n        decode_k = decode_v",
                                "        decode_k = decode_v"),
    "e4m3_wrong_bias": ("np.exp2((e - 7).astype(np.float64))", "np.exp2((e - 8).astype(np.float64))"),
    "e4m3_truncates": ("q = np.rint(a / step).astype(np.int64)", "q = np.floor(a / step).astype(np.int64)"),
    "e4m3_rounds_half_up": ("q = np.rint(a / step).astype(np.int64)", "q = np.floor(a / step + 0.5).astype(np.int64)"),
    "e4m3_no_saturation": ("a = np.minimum(np.abs(x.astype(np.float64)), E4M3_MAX)", "a = np.abs(x.astype(np.float64))"),
    "e4m3_flushes_subnormals": ("e_unb = np.maximum(expo - 1, -6)", "e_unb = expo - 1"),
    "e4m3_drops_sign": ("return (sign | code).astype(np.uint8)", "return code.astype(np.uint8)"),
    "fp8_multiplies_by_scale": ("inv = np.float32(1.0) / np.float32(scale)", "inv = np.float32(scale)"),
    "fp8_k_scale_not_applied": ("decode_k = lambda u: e4m3_to_f64(u) * k_scale", "decode_k = lambda u: e4m3_to_f64(u)"),
    "fp8_v_uses_k_scale": ("decode_v = lambda u: e4m3_to_f64(u) * v_scale", "decode_v = lambda u: e4m3_to_f64(u) * k_scale"),
    "fp8_update_skipped": ("        update_cache(quantize_rows(k_new, k_scale), quantize_rows(v_new, v_scale), k_pages, v_pages, page_table,\n                     cu_q_lens, kv_lens, num_seqs)\n", ""),
    "fp8_v_rows_use_k_scale": ("quantize_rows(v_new, v_scale)", "quantize_rows(v_new, k_scale)"),
    "merge_without_rescale": ("w = 0.0 if m == -np.inf else math.exp(m - big)", "w = 1.0"),
    "q_offset_ignored": ("qq = bf16_to_f64(q[q0:q0 + l_q])", "qq = bf16_to_f64(q[0:l_q])"),
}


def load_mutant(old, new):
    with open(SRC) as f:
        text = f.read()
    assert text.count(old) == 1, f"mutation anchor not unique: {old!r}"
    mod = types.ModuleType("rpa_oracle_mutant")
    exec(compile(text.replace(old, new), SRC + ":mutant", "exec"), mod.__dict__)
    return mod


PIN_TESTS = [(n, f) for n, f in inspect.getmembers(pins, inspect.isfunction)
             if n.startswith("test_") and n not in ("test_config_shapes",)]


def _calls(fn):
    """Expand pytest parametrisation (stacked marks included) by hand: a list of
    keyword dicts, one per case."""
    cases = [{}]
    for m in getattr(fn, "pytestmark", []):
        if m.name != "parametrize":
            continue
        names = [s.strip() for s in m.args[0].split(",")]
        expanded = []
        for v in m.args[1]:
            vals = v if len(names) > 1 else (v,)
            expanded += [dict(c, **dict(zip(names, vals))) for c in cases]
        cases = expanded
    return cases


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_mutation(name, monkeypatch):
    mutant = load_mutant(*MUTATIONS[name])
    monkeypatch.setattr(pins, "O", mutant)
    caught = []
    for tname, fn in PIN_TESTS:
        for args in _calls(fn):
            try:
                fn(**args)
            except (AssertionError, ValueError, IndexError, FloatingPointError):
                caught.append(tname)
                break
        if caught:
            break
    assert caught, f"no pin noticed the planted mistake {name}"
