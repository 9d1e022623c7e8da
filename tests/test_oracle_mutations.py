"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a COPY of the oracle's C
source (CPU only), build it, and require that at least one pin from test_oracle_pins.py fails.
The oracle that the rest of the suite uses is never modified."""
import importlib.util
import os
import subprocess
import sys

import numpy as np
import pytest

import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "emb_bag_oracle.c")
WRAP = os.path.join(ROOT, "oracle", "emb_bag_oracle.py")

MUTATIONS = {
    "weight dropped from the sum": ("acc += w * x;", "acc += x;"),
    "bound without abs": ("mag += fabs(w) * ax;", "mag += w * ax;"),
    "bound of a float element without abs": ("  *magnitude = fabs(x);\n  return x;", "  *magnitude = x;\n  return x;"),
    "quantised element without its bias": ("return sc + (double)bias;", "return sc;"),
    "quantised scale and bias swapped": ("memcpy(&scale, row + D, sizeof scale);\n    memcpy(&bias, row + D + 4, sizeof bias);",
                                         "memcpy(&bias, row + D, sizeof scale);\n    memcpy(&scale, row + D + 4, sizeof bias);"),
    "quantised row stride without the scale and bias": ("(const uint8_t*)tables + arena_row * (D + 8);", "(const uint8_t*)tables + arena_row * D;"),
    "quantised code read as signed": ("dtype == 3 ? (double)row[d] :", "dtype == 3 ? (double)(int8_t)row[d] :"),
    "quantised bound forgets the bias": ("*magnitude = fabs(sc) + fabs((double)bias);", "*magnitude = fabs(sc);"),
    "table base ignored": ("table_offsets[t] + indices[j], D, d, &ax)", "indices[j], D, d, &ax)"),
    "first lookup of a bag skipped": ("for (int64_t j = s; j < e; ++j) {", "for (int64_t j = s + 1; j < e; ++j) {"),
    "last lookup of a bag skipped": ("for (int64_t j = s; j < e; ++j) {", "for (int64_t j = s; j < e - 1; ++j) {"),
    "bags taken in (b, t) order": ("const int64_t t = g / B;\n    const int64_t b = g % B;",
                                   "const int64_t t = g % T;\n    const int64_t b = g / T;"),
    "output transposed within a table block": ("ref[b * out_ld + t * D + d] = acc;",
                                               "ref[b * out_ld + t * D + (D - 1 - d)] = acc;"),
    "output block of the wrong table": ("ref[b * out_ld + t * D + d] = acc;",
                                        "ref[b * out_ld + (T - 1 - t) * D + d] = acc;"),
    "mean divides by len + 1": ("acc /= (double)(e - s);", "acc /= (double)(e - s + 1);"),
    "mean of bound forgotten": ("          mag /= (double)(e - s);", ""),
    "columns reversed when reading a half row": ("x = half_bits_to_double(((const uint16_t*)tables)[arena_row * D + d]);",
                                                 "x = half_bits_to_double(((const uint16_t*)tables)[arena_row * D + (D - 1 - d)]);"),
    "fp32 rows read with the wrong stride": ("x = (double)((const float*)tables)[arena_row * D + d];",
                                             "x = (double)((const float*)tables)[arena_row * (D - 1) + d];"),
    "half exponent bias off by one": ("expo - 25", "expo - 24"),
    "half subnormal scale off by one": ("ldexp((double)frac, -24)", "ldexp((double)frac, -25)"),
    "half sign dropped": ("(1 + frac/1024) * 2^(expo-15) */\n  return sign ? -v : v;", "(1 + frac/1024) * 2^(expo-15) */\n  return v;"),
    "bfloat16 shifted one bit short": ("const uint32_t u = (uint32_t)h << 16;", "const uint32_t u = (uint32_t)h << 15;"),
    "max keeps the smaller element": ("if (j == s || x > acc) {", "if (j == s || x < acc) {"),
    "max starts from zero instead of the first element": ("if (j == s || x > acc) {", "if (x > acc) {"),
    "max bound not taken from the selected element": ("            acc = x;\n            mag = ax;", "            acc = x;\n            mag += ax;"),
    "e4m3 exponent bias off by one": ("ldexp((double)(8 + frac), expo - 10)", "ldexp((double)(8 + frac), expo - 11)"),
    "e4m3 subnormal scale off by one": ("ldexp((double)frac, -9)", "ldexp((double)frac, -10)"),
    "e4m3 sign dropped": ("(1 + frac/8) * 2^(expo-7) */\n  return sign ? -v : v;", "(1 + frac/8) * 2^(expo-7) */\n  return v;"),
    "e4m3 treats the whole top exponent as NaN": ("else if (expo == 15 && frac == 7)", "else if (expo == 15)"),
    "e4m3 codes read as integers": ("const double code = dtype == 3 ? (double)row[d] : e4m3_bits_to_double(row[d]);", "const double code = (double)row[d];"),
    "strict bound without abs": ("smag += fabs(w * x);", "smag += w * x;"),
    "strict bound charges the two terms": ("smag += fabs(w * x);", "smag += fabs(w) * ax;"),
    "strict bound of the mean forgotten": ("smag /= (double)(e - s);", ""),
    "weights applied in mean mode only": ("const double w = weights ? (double)weights[j] : 1.0;",
                                          "const double w = (weights && mode == 1) ? (double)weights[j] : 1.0;"),
}

PIN_FUNCS = [
    lambda o: pins.test_brute_force_exact_rational(o, "sum", np.float32),
    lambda o: pins.test_brute_force_exact_rational(o, "mean", np.float16),
    pins.test_brute_force_weighted,
    pins.test_hand_worked_example,
    pins.test_identity_tables_give_index_histograms,
    pins.test_table_base_is_respected,
    pins.test_one_item_case,
    pins.test_mean_is_sum_over_len_and_edge_lengths,
    pins.test_empty_and_len1_bags,
    pins.test_weights,
    pins.test_bound_is_sum_of_abs_terms,
    pins.test_strict_bound_equals_the_bound_for_unquantised_rows,
    pins.test_half_widening_is_exact,
    pins.test_bfloat16_widening_is_exact,
    pins.test_quantised_rows_brute_force,
    pins.test_quantised_rows_equal_their_dequantised_table,
    pins.test_e4m3_values_typed_in,
    pins.test_e4m3_every_code_against_torch,
    pins.test_e4m3_rows_brute_force,
    pins.test_max_hand_worked,
    lambda o: pins.test_max_brute_force(o, np.float32),
    pins.test_max_invariants,
]


def _load_mutant(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation {name!r}: pattern must occur exactly once"
    c_path = tmp_path / "mutant.c"
    so_path = tmp_path / "mutant.so"
    c_path.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so_path),
                    str(c_path), "-lm"], check=True, stderr=subprocess.DEVNULL)
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{abs(hash(name))}", WRAP)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.SRC, mod.LIB, mod._lib = str(c_path), str(so_path), None
    return mod


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTATIONS[name]
    mutant = _load_mutant(tmp_path, name, old, new)
    caught = []
    for f in PIN_FUNCS:
        try:
            f(mutant)
        except (AssertionError, ValueError) as ex:
            caught.append(type(ex).__name__)
    assert caught, f"no pin noticed: {name}"


def test_unmutated_copy_passes_every_pin(tmp_path):
    src = open(SRC).read()
    clean = _load_mutant(tmp_path, "identity", "acc += w * x;", "acc += w * x; ")
    for f in PIN_FUNCS:
        f(clean)


# ---- the two integer oracles written in Python (reuse profile, hot rows) ------------------------
PY_ORACLES = {"reuse_oracle": os.path.join(ROOT, "oracle", "reuse_oracle.py"),
              "hot_rows_oracle": os.path.join(ROOT, "oracle", "hot_rows_oracle.py")}

PY_MUTATIONS = {
    "reuse: repeats counted as distinct ids": ("reuse_oracle", "d = w - len(set(seg))", "d = len(set(seg))"),
    "reuse: the batch taken to be the window": ("reuse_oracle", "w, n_t = len(seg), e - s", "w, n_t = len(seg), len(seg)"),
    "reuse: share bar not strict": ("reuse_oracle", "few_repeats = n_t * d * 1000 * 128 < thr", "few_repeats = n_t * d * 1000 * 128 <= thr"),
    "reuse: cache bar not strict": ("reuse_oracle", "min(int(row_bytes), 128) > d * (1 << 36)", "min(int(row_bytes), 128) >= d * (1 << 36)"),
    "reuse: cache of half the size": ("reuse_oracle", "> d * (1 << 36)", "> d * (1 << 35)"),
    "reuse: rows per line ignored in the share": ("reuse_oracle", "thr * w * w * min(int(row_bytes), 128)", "thr * w * w * 128"),
    "reuse: rows per line ignored in the cache bar": ("reuse_oracle", "w * w * int(row_bytes) * min(int(row_bytes), 128) >", "w * w * int(row_bytes) * 128 >"),
    "reuse: threshold not capped": ("reuse_oracle", "thr = min(int(threshold_permille), 1_000_000)", "thr = int(threshold_permille)"),
    "reuse: an empty table is not streaming": ("reuse_oracle", "(w == 0 or beyond_cache or few_repeats)", "(beyond_cache or few_repeats)"),
    "reuse: the largest window refused": ("reuse_oracle", "if not 1 <= window <= MAX_WINDOW:", "if not 1 <= window < MAX_WINDOW:"),
    "reuse: window not applied": ("reuse_oracle", "indices[s:e][:window]", "indices[s:e]"),
    "reuse: table boundaries off by one bag": ("reuse_oracle", "int(offsets[t * B]), int(offsets[(t + 1) * B])", "int(offsets[t * B]), int(offsets[(t + 1) * B - 1])"),
    "hot rows: ties to the larger id": ("hot_rows_oracle", "(-int(counts[i]), int(ids[i]))", "(-int(counts[i]), -int(ids[i]))"),
    "hot rows: least frequent first": ("hot_rows_oracle", "(-int(counts[i]), int(ids[i]))", "(int(counts[i]), int(ids[i]))"),
    "hot rows: window not applied": ("hot_rows_oracle", "indices[s:e][:window]", "indices[s:e]"),
    "hot rows: the id 2^40 - 1 counted": ("hot_rows_oracle", "(seg >= 0) & (seg < ID_LIMIT)", "(seg >= 0) & (seg <= ID_LIMIT)"),
    "hot rows: negative ids counted": ("hot_rows_oracle", "seg[(seg >= 0) & (seg < ID_LIMIT)]", "seg[seg < ID_LIMIT]"),
    "hot rows: one row short": ("hot_rows_oracle", "[:k]\n", "[:k - 1]\n"),
    "hot rows: table boundaries off by one bag": ("hot_rows_oracle", "int(offsets[t * B]), int(offsets[(t + 1) * B])", "int(offsets[t * B]), int(offsets[(t + 1) * B - 1])"),
}

PY_PINS = {
    "reuse_oracle": [pins.test_reuse_profile_hand_worked, pins.test_reuse_profile_closed_forms,
                     pins.test_reuse_profile_counts_the_whole_batch,
                     pins.test_reuse_profile_rows_in_use_beyond_the_cache],
    "hot_rows_oracle": [pins.test_hot_rows_hand_worked, pins.test_hot_rows_closed_forms_and_second_route],
}


def _run_py_pins(monkeypatch, which, source):
    """Run the pins of one Python oracle against a module built from `source`; the names of the
    exception types they raised."""
    import types
    import oracle
    mod = types.ModuleType(f"oracle.{which}")
    mod.__file__ = PY_ORACLES[which]
    sys.modules[f"oracle.{which}_mutant"] = mod     # (dataclasses and typing look modules up by name)
    exec(compile(source, PY_ORACLES[which], "exec"), mod.__dict__)
    monkeypatch.setitem(sys.modules, f"oracle.{which}", mod)
    monkeypatch.setattr(oracle, which, mod, raising=False)
    caught = []
    for f in PY_PINS[which]:
        try:
            f()
        except (AssertionError, ValueError, IndexError) as ex:
            caught.append(type(ex).__name__)
    return caught


@pytest.mark.parametrize("name", sorted(PY_MUTATIONS))
def test_planted_mistake_in_a_python_oracle_is_caught(monkeypatch, name):
    which, old, new = PY_MUTATIONS[name]
    src = open(PY_ORACLES[which]).read()
    assert src.count(old) == 1, f"mutation {name!r}: pattern must occur exactly once"
    assert _run_py_pins(monkeypatch, which, src.replace(old, new)), f"no pin noticed: {name}"


@pytest.mark.parametrize("which", sorted(PY_ORACLES))
def test_unmutated_python_oracle_passes_its_pins(monkeypatch, which):
    assert _run_py_pins(monkeypatch, which, open(PY_ORACLES[which]).read()) == []
