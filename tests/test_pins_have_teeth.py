"""The pins must be able to fail: plausible mistakes are planted in a COPY of the
oracle source (a dropped term, a wrong sign, index, comparison or operand), the
copy is compiled on the CPU (or, for the oracle's numpy functions, executed in
place of the function), and the pin tests are re-run against it -- at least one
pin has to object to every planted mistake."""
import ctypes
import inspect
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins
import test_workloads as wpins

# (what it breaks, text in oracle/groot_oracle.c, replacement)
MUTATIONS = [
    ("weight off by one", "1.0f / (float)deg : 1.0f", "1.0f / (float)(deg + 1) : 1.0f"),
    ("sign of a term", "y += term;", "y -= term;"),
    ("operand index (row instead of column)", "X[(int64_t)col[p] * F + k]", "X[(int64_t)i * F + k]"),
    ("dropped last entry of a row", "for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {\n                double term",
     "for (int64_t p = rowptr[i]; p < rowptr[i + 1] - 1; ++p) {\n                double term"),
    ("abs sum without abs", "s += fabs(term);", "s += term;"),
    ("no reverse edge", "if (flags & ORC_SYMMETRIC) { e[m].row = u;", "if (0) { e[m].row = u;"),
    ("polarity bit lost", "e[m].pol = (uint8_t)(inv | 2); ++m;", "e[m].pol = (uint8_t)2; ++m;"),
    ("duplicates kept", "if (w > 0 && e[w - 1].row == e[t].row && e[w - 1].col == e[t].col) e[w - 1].pol |= e[t].pol;\n        else e[w++] = e[t];",
     "e[w++] = e[t];"),
    ("batch offset on columns", "col[p] = (int32_t)((int64_t)c * n1 + e[t].col);", "col[p] = (int32_t)(e[t].col);"),
    ("threshold comparison", "row_class[i] = deg >= T;\n        if (deg >= T)", "row_class[i] = deg > T;\n        if (deg > T)"),
    ("degree sort descending", "for (int32_t d = 0; d < T; ++d) {\n        deg_offsets[d] = w;\n        for (int64_t i = 0; i < n; ++i)",
     "for (int32_t d = 0; d < T; ++d) {\n        deg_offsets[d] = w;\n        for (int64_t i = n - 1; i >= 0; --i)"),
    ("boundary misses neighbours with smaller ids", "if (col[q] != u) in_N[col[q]] = 1;", "if (col[q] > u) in_N[col[q]] = 1;"),
    ("boundary-boundary edges kept", "|| (i_owned != j_owned)                     /* C_p               */", "|| 1"),
    ("crossing counted from one side only", "if (!i_owned && j_owned && !has_entry(rowptr, col, j, i)) ++cross;", ""),
    ("AND evaluated as OR", "(type[v] == 1) ? (w0 & w1) : w0", "(type[v] == 1) ? (w0 | w1) : w0"),
    ("inverter ignored", "word[l1 >> 1] ^ ((l1 & 1) ? ~0ULL : 0ULL)", "word[l1 >> 1]"),
    ("transposed product scatters to the row", "out[j * F + k] += term;", "out[i * F + k] += term;"),
    ("transpose keeps the weight of another entry", "t_val[q] = val[p];", "t_val[q] = val[q];"),
    ("partition rule rounds up", "int64_t q = ((v % n1) * P) / n1;", "int64_t q = ((v % n1) * P + n1 - 1) / n1;"),
]

PIN_CALLS = [
    lambda: [pins.test_degree_histogram_closed_form(n) for n in (6, 8)],
    lambda: [pins.test_csr_structure(n) for n in (2, 3, 5)],
    lambda: pins.test_csr_flags_and_batch(),
    lambda: [pins.test_spmm_equals_dense_product(n) for n in (2, 3)],
    lambda: pins.test_spmm_ones_gives_row_sums(8, 1),
    lambda: pins.test_spmm_matches_scipy_on_stress_graph(),
    lambda: [pins.test_plan_on_multipliers(*a) for a in ((8, 1, 7), (8, 2, 9))],
    lambda: pins.test_plan_thresholds_on_stress_graph(),
    lambda: [pins.test_regrow_hand_cases(s) for s in (False, True)],
    lambda: [pins.test_regrow_on_multipliers(*a) for a in ((2, 2), (3, 3), (4, 3))],
    lambda: pins.test_regrow_one_way_edges_and_weight_modes(),
    lambda: pins.test_partition_rule_closed_form(),
    lambda: [pins.test_transposed_spmm_equals_dense_transpose(n, 7) for n in (2, 3)],
    lambda: pins.test_transposed_spmm_adjoint_identity(),
    lambda: wpins.test_two_bit_example_matches_paper(),
    lambda: wpins.test_multiplier_function_equals_integer_product(5),
    lambda: [pins.test_sage_layer_equals_dense_layer(n) for n in (2, 3)],
    lambda: pins.test_sage_layer_special_cases(),
    lambda: pins.test_sage_forward_is_two_layers(),
    lambda: pins.test_sage_forward_reduces_to_spmm(),
]

# mistakes planted in the oracle's numpy functions: (what, function, text, replacement)
PY_MUTATIONS = [
    ("layer: self term dropped", "sage_layer_f64", " + np.asarray(X, dtype=np.float64) @ Ws.astype(np.float64)", ""),
    ("layer: ReLU before the bias", "sage_layer_f64",
     "    if b is not None:\n        H = H + b.astype(np.float64)\n",
     "    if relu:\n        H = np.maximum(H, 0.0)\n    if b is not None:\n        H = H + b.astype(np.float64)\n"),
    ("layer: neighbour and self weights swapped", "sage_layer_f64",
     "A @ Wn.astype(np.float64) + np.asarray(X, dtype=np.float64) @ Ws.astype(np.float64)",
     "A @ Ws.astype(np.float64) + np.asarray(X, dtype=np.float64) @ Wn.astype(np.float64)"),
    ("layer: weight matrix transposed", "sage_layer_f64", "A @ Wn.astype(np.float64)", "A @ Wn.astype(np.float64).T"),
    ("layer: bias subtracted", "sage_layer_f64", "H = H + b.astype(np.float64)", "H = H - b.astype(np.float64)"),
    ("forward: no ReLU between the layers", "sage_forward_f64",
     "H1 = np.maximum(A1 @ W1n.astype(np.float64) + X64 @ W1s.astype(np.float64) + b1.astype(np.float64), 0.0)",
     "H1 = A1 @ W1n.astype(np.float64) + X64 @ W1s.astype(np.float64) + b1.astype(np.float64)"),
    ("forward: second layer aggregates the input again", "sage_forward_f64",
     "A2, _ = spmm_f64(rowptr, col, val, H1f, want_abs=False)", "A2, _ = spmm_f64(rowptr, col, val, X, want_abs=False)"),
]


ORACLE_SYMBOLS = ("orc_aig_simulate", "orc_csr_nnz", "orc_csr_build", "orc_spmm_f64", "orc_plan",
                  "orc_part_of_default", "orc_regrow_sizes", "orc_regrow_fill", "orc_spmm_t_f64", "orc_csr_transpose")


def test_symbol_list_covers_the_oracle_library():
    """Every function the oracle's C source exports gets its argument types copied onto a mutant."""
    src = open(os.path.join(os.path.dirname(oracle.__file__), "groot_oracle.c")).read()
    import re
    exported = set(re.findall(r"^(?:int32_t|void|int64_t|double)\s+(orc_\w+)\s*\(", src, flags=re.M))
    assert exported == set(ORACLE_SYMBOLS), exported ^ set(ORACLE_SYMBOLS)
    good = oracle._load()
    for name in ORACLE_SYMBOLS:
        assert getattr(good, name).argtypes is not None, name


def _build_mutant(tmp_path, idx, old, new):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "groot_oracle.c")).read()
    assert src.count(old) == 1, f"mutation {idx}: pattern must occur exactly once"
    c_path = tmp_path / f"mutant{idx}.c"
    so_path = tmp_path / f"mutant{idx}.so"
    c_path.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so_path), str(c_path), "-lm"],
                   check=True)
    return str(so_path)


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_every_planted_mistake_is_caught(idx, tmp_path, monkeypatch):
    what, old, new = MUTATIONS[idx]
    mutant = ctypes.CDLL(_build_mutant(tmp_path, idx, old, new))
    good = oracle._load()
    for name in ORACLE_SYMBOLS:
        getattr(mutant, name).restype = getattr(good, name).restype
        getattr(mutant, name).argtypes = getattr(good, name).argtypes
    monkeypatch.setattr(oracle, "_lib", mutant)
    caught = 0
    for call in PIN_CALLS:
        try:
            call()
        except (AssertionError, ValueError, IndexError):
            caught += 1
    assert caught > 0, f"no pin noticed: {what}"


@pytest.mark.parametrize("idx", range(len(PY_MUTATIONS)))
def test_every_planted_mistake_in_the_numpy_functions_is_caught(idx, monkeypatch):
    what, fn, old, new = PY_MUTATIONS[idx]
    src = inspect.getsource(getattr(oracle, fn))
    assert src.count(old) == 1, f"mutation {idx}: pattern must occur exactly once"
    scope = dict(vars(oracle))
    exec(compile(src.replace(old, new), f"<mutant of {fn}>", "exec"), scope)
    monkeypatch.setattr(oracle, fn, scope[fn])
    caught = 0
    for call in PIN_CALLS:
        try:
            call()
        except (AssertionError, ValueError, IndexError):
            caught += 1
    assert caught > 0, f"no pin noticed: {what}"
