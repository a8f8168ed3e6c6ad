"""Do the pins bite?  Every case here plants ONE plausible slip in a private copy of the CPU
oracle (a dropped accumulation, a wrong index, a missing offset, a sign, an unstable sort, a
dropped bias, ...), rebuilds that copy in a temporary directory, and runs the pins of
``test_oracle_pins.py`` against it: at least one pin has to fail.  The committed oracle is never
touched, and nothing here runs on a GPU.

Every planted slip keeps all memory accesses inside the arrays the pins pass (it reads a wrong
element, never one outside), so a mutant computes a wrong answer instead of crashing.
"""
import importlib.util
import inspect
import itertools
import os
import shutil

import pytest

import test_oracle_pins as pins

_ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")

# (name, file, text to replace, replacement, which occurrence of the text)
MUTANTS = [
    # forward product (Fig. 2 / Fig. 3 / Fig. 4 all reach C[r][j] += v * B[c][j])
    ("forward_overwrites_instead_of_adding", "c",
     "c[j] += v * (double)b[j];", "c[j] = v * (double)b[j];", 0),
    ("forward_gathers_the_row_s_first_column", "c",
     "const float* b = B + (b_row_off[i] + ci[p]) * ldb;",
     "const float* b = B + (b_row_off[i] + ci[rp[r]]) * ldb;", 0),
    ("forward_ignores_the_input_block_offset", "c",
     "const float* b = B + (b_row_off[i] + ci[p]) * ldb;",
     "const float* b = B + (int64_t)ci[p] * ldb;", 0),
    ("forward_drops_the_last_entry_of_a_row", "c",
     "p < rp[r + 1]; ++p)", "p < rp[r + 1] - 1; ++p)", 0),
    ("forward_ignores_the_output_block_offset", "c",
     "double* c = C + (c_row_off[i] + r) * ldc;", "double* c = C + (int64_t)r * ldc;", 0),
    ("forward_drops_the_value", "c",
     "c[j] += v * (double)b[j];", "c[j] += (double)b[j];", 0),
    ("scale_without_absolute_values", "c",
     "s[j] += fabs(v) * fabs((double)b[j]);", "s[j] += v * (double)b[j];", 0),
    # transposed product (Sec. IV-C backward pass: a scatter over the stored entries)
    ("transposed_with_the_wrong_sign", "c",
     "g[j] += v * (double)y[j];", "g[j] -= v * (double)y[j];", 0),
    ("transposed_reads_the_block_s_first_row", "c",
     "const float* y = dY + (c_row_off[i] + r) * ldy;",
     "const float* y = dY + c_row_off[i] * ldy;", 0),
    ("transposed_ignores_the_output_block_offset", "c",
     "double* g = G + (b_row_off[i] + ci[p]) * ldg;", "double* g = G + (int64_t)ci[p] * ldg;", 0),
    ("transposed_drops_the_last_entry_of_a_row", "c",
     "p < rp[r + 1]; ++p)", "p < rp[r + 1] - 1; ++p)", 2),
    # transposed CSR (stable counting sort)
    ("transpose_walks_the_rows_backwards", "c",
     "for (int32_t r = 0; r < rows[i]; ++r)\n            for (int32_t p = rp[r]; p < rp[r + 1]; ++p) {\n                const int32_t q",
     "for (int32_t r = rows[i] - 1; r >= 0; --r)\n            for (int32_t p = rp[r]; p < rp[r + 1]; ++p) {\n                const int32_t q", 0),
    ("transpose_keeps_the_column_index", "c", "ct[q] = r;", "ct[q] = ci[p];", 0),
    ("transpose_leaves_the_values_in_place", "c", "vt[q] = va[p];", "vt[p] = va[p];", 0),
    # COO product and conversion (Fig. 2; Sec. IV: entries are not sorted)
    ("coo_drops_the_last_entry", "c",
     "for (int32_t p = 0; p < nnz[i]; ++p) {\n            const int32_t rid",
     "for (int32_t p = 0; p < nnz[i] - 1; ++p) {\n            const int32_t rid", 0),
    ("coo_repeated_pairs_overwrite", "c",
     "y[j] += val * (double)x[j];", "y[j] = val * (double)x[j];", 0),
    ("coo_ignores_the_input_block_offset", "c",
     "const float* x = X + (in_off[i] + cid) * ldx;", "const float* x = X + (int64_t)cid * ldx;", 0),
    ("coo_to_csr_walks_the_entries_backwards", "c",
     "for (int32_t p = 0; p < nnz[i]; ++p) {\n            const int32_t q = cursor_scratch[id[2 * p]]++;",
     "for (int32_t p = nnz[i] - 1; p >= 0; --p) {\n            const int32_t q = cursor_scratch[id[2 * p]]++;", 0),
    ("coo_to_csr_stores_the_row_as_column", "c",
     "colids[nz_off[i] + q] = id[2 * p + 1];", "colids[nz_off[i] + q] = id[2 * p];", 0),
    # graph-convolution layer (Fig. 7: MatMul, Add, BatchedSpMM, ElementWiseAdd)
    ("layer_product_drops_the_value", "c", "c[j] += v * b[j];", "c[j] += b[j];", 0),
    ("layer_channels_overwrite_each_other", "c", "if (!accumulate)", "if (1)", 0),
    ("layer_matmul_drops_the_last_input_feature", "py",
     "U = X64 @ W64 ", "U = X64[:, :-1] @ W64[:-1] ", 0),
    ("layer_matmul_pairs_features_with_the_wrong_weight_rows", "py",
     "U = X64 @ W64 ", "U = X64[:, ::-1] @ np.roll(W64[::-1], 1, axis=0) ", 0),
    ("layer_matmul_is_elementwise_times_a_row_sum", "py",
     "U = X64 @ W64 ", "U = X64.sum(axis=1, keepdims=True) * W64.mean(axis=0, keepdims=True) ", 0),
    ("layer_without_bias", "py",
     "B = np.ascontiguousarray(U + bias64[None, :])", "B = np.ascontiguousarray(U)", 0),
    ("layer_bias_added_twice", "py",
     "B = np.ascontiguousarray(U + bias64[None, :])",
     "B = np.ascontiguousarray(U + 2.0 * bias64[None, :])", 0),
    ("layer_tolerance_without_absolute_values", "py",
     "np.abs(X64) @ np.abs(W64)", "X64 @ W64", 0),
    ("layer_rounds_its_input_to_half_precision", "py",
     "X64 = np.asarray(X, dtype=np.float32).astype(np.float64)",
     "X64 = np.asarray(X, dtype=np.float16).astype(np.float64)", 0),
]


def _replace_nth(text, old, new, nth):
    at = -1
    for _ in range(nth + 1):
        at = text.find(old, at + 1)
        assert at >= 0, f"mutation site not found: {old!r} (occurrence {nth})"
    return text[:at] + new + text[at + len(old):]


def _mutant_module(tmp_path, name, which, old, new, nth):
    """A private copy of oracle/ with one replacement, imported under its own module name."""
    d = tmp_path / name
    d.mkdir()
    for f in ("bspmm_oracle.c", "reference.py"):
        shutil.copy(os.path.join(_ORACLE_DIR, f), d / f)
    target = d / ("bspmm_oracle.c" if which == "c" else "reference.py")
    target.write_text(_replace_nth(target.read_text(), old, new, nth))
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{name}", d / "reference.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)       # _HERE inside the copy is the temporary directory
    assert os.path.dirname(mod._LIB) == str(d)
    mod.build(force=True)
    return mod


def _pin_calls():
    """Every pin that takes the oracle, once per combination of its parameters."""
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_") or "oracle" not in inspect.signature(fn).parameters:
            continue
        axes = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                names = [s.strip() for s in mark.args[0].split(",")]
                assert len(names) == 1
                axes.append([(names[0], v) for v in mark.args[1]])
        for combo in itertools.product(*axes):
            calls.append((name, fn, dict(combo)))
    return calls


def _first_failing_pin(mod):
    for name, fn, kw in _pin_calls():
        try:
            fn(oracle=mod, **kw)
        except Exception:       # an assertion, or the oracle refusing what it should accept
            return name
    return None


def test_the_pins_pass_on_an_unchanged_copy(tmp_path):
    """The harness itself: a copy with no slip passes every pin (so a failure below is the
    slip's, not the copying's), and the pins it runs are the ones pytest collects."""
    src = open(os.path.join(_ORACLE_DIR, "bspmm_oracle.c")).read()
    mod = _mutant_module(tmp_path, "unchanged", "c", src[:40], src[:40], 0)
    assert _first_failing_pin(mod) is None
    assert len(_pin_calls()) >= 35


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_slip_fails_a_pin(tmp_path, mutant):
    name, which, old, new, nth = mutant
    mod = _mutant_module(tmp_path, name, which, old, new, nth)
    caught_by = _first_failing_pin(mod)
    assert caught_by is not None, f"no pin notices the slip '{name}'"
