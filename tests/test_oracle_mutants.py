"""Do the pins bite?  Each case below plants ONE plausible mistake in a copy of the oracle's C source (a dropped
factor, a wrong index, an off-by-one window, a transposed operand, a forgotten deletion), builds it, swaps it in
for the oracle library, and runs the pin tests: at least one of them must fail.  CPU only; the mistakes live in
copies under a temporary directory, the oracle itself is untouched."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_backward_pins as bwd
import test_oracle_pins as fwd

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "dgnn_oracle.c")
GOLDEN = os.path.join(HERE, "golden")

# (name, text in the oracle source, what a mistaken author might have written instead)
MUTANTS = [
    ("normalisation uses the row degree twice", "val[e] = 1.0 / sqrt(du * dv);", "val[e] = 1.0 / sqrt(du * du);"),
    ("normalisation without the square root", "val[e] = 1.0 / sqrt(du * dv);", "val[e] = 1.0 / (du * dv);"),
    ("degree counted without the self loop", "double dv = (double)(rowptr[v + 1] - rowptr[v]);",
     "double dv = (double)(rowptr[v + 1] - rowptr[v]) - 1.0 + (rowptr[v + 1] - rowptr[v] == 1);"),
    ("aggregation drops the edge weight", "zu[j] += val[e] * hv[j];", "zu[j] += hv[j];"),
    ("aggregation reads the row's own features", "const double *hv = h + (int64_t)colidx[e] * f;", "const double *hv = h + u * f;"),
    ("ReLU clamps the wrong side", "if (zu[j] < 0.0) zu[j] = 0.0;", "if (zu[j] > 0.0) zu[j] = 0.0;"),
    ("dense transform with W transposed", "s += x[i * f_in + k] * w[k * f_out + j];", "s += x[i * f_in + k] * w[(k % f_out) * f_out + (j % f_in)];"),
    ("window one step too long", "int64_t lo = t - w + 1 > 1 ? t - w + 1 : 1;", "int64_t lo = t - w > 1 ? t - w : 1;"),
    ("weights 1/w from the first step on", "double mn = (double)(w < t ? w : t);", "double mn = (double)w;"),
    ("M applied transposed", "s += M[t * T + k] * z[k * frame + i];", "s += M[k * T + t] * z[k * frame + i];"),
    ("deleted edges are kept", "if (!is_member(del, n_del, prev[e])) prev[m++] = prev[e];", "prev[m++] = prev[e];"),
    ("added edges are dropped", "else if (i >= m || add[j] < prev[i]) next[o++] = add[j++];", "else if (i >= m || add[j] < prev[i]) j++;"),
    ("adjoint aggregation not transposed", "out[(int64_t)colidx[e] * f + j] += val[e] * g[u * f + j];",
     "out[u * f + j] += val[e] * g[(int64_t)colidx[e] * f + j];"),
    ("weight gradient with the operands exchanged", "s += x[i * f_in + k] * g[i * f_out + j];",
     "s += x[i * f_in + (j % f_in)] * g[i * f_out + (k % f_out)];"),
    ("adjoint M-transform not transposed", "s += M[t * T + k] * g[t * frame + i];", "s += M[k * T + t] * g[t * frame + i];"),
    ("value updates ignored", "all[m].val = u >= 0 ? upd[u].val : val[e];", "all[m].val = val[e];"),
    ("added values not taken", "if (i == 0 || add[i].key != add[i - 1].key) all[m++] = add[i];",
     "if (i == 0 || add[i].key != add[i - 1].key) { all[m] = add[i]; all[m].val = 1.0; ++m; }"),
]


def pins():
    """Every pin test as a zero-argument callable."""
    calls = []
    for seed in (0, 1, 2):
        for sym in (True, False):
            calls.append(lambda s=seed, y=sym: fwd.test_delta_apply_matches_dense_boolean_brute_force(s, y))
    calls += [fwd.test_delta_apply_adversarial_tiny_cases, fwd.test_delta_apply_equals_from_scratch_every_step_c1,
              fwd.test_delta_involution_and_composition, fwd.test_csr_from_edges_handles_repeats_and_order,
              lambda: fwd.test_gcn_values_match_hand_worked_path(GOLDEN), fwd.test_xw_matches_numpy_rectangular,
              fwd.test_spmm_c1_whole_layer_vs_dense, fwd.test_spmm_sqrt_degree_is_fixed_vector, fwd.test_spmm_special_graphs,
              fwd.test_mproduct_closed_forms, fwd.test_c1_end_to_end_vs_dense_brute_force]
    for sym in (True, False):
        calls.append(lambda y=sym: fwd.test_gcn_values_match_dense_matrix_form(y))
        for relu in (False, True):
            calls.append(lambda y=sym, r=relu: fwd.test_spmm_matches_dense_brute_force(y, r))
    calls += [lambda: fwd.test_m_matrix_matches_hand_worked(GOLDEN, "m_matrix_T3_w2.txt", 3, 2),
              lambda: fwd.test_m_matrix_matches_hand_worked(GOLDEN, "m_matrix_T5_w3.txt", 5, 3)]
    for T, w in ((8, 3), (32, 8), (5, 1), (6, 9)):
        calls.append(lambda a=T, b=w: fwd.test_m_matrix_structure(a, b))
    for sym in (False, True):
        calls.append(lambda y=sym: bwd.test_spmm_t_matches_dense_transpose(y))
    calls += [bwd.test_spmm_t_is_the_adjoint_of_spmm, bwd.test_spmm_t_equals_spmm_on_undirected_graphs_only,
              bwd.test_spmm_t_closed_form_sqrt_degree, bwd.test_weight_grad_special_cases_and_numpy,
              bwd.test_input_grad_matches_numpy_and_adjoint, bwd.test_layer_backward_matches_finite_differences,
              bwd.test_weighted_delta_apply_trivial_cases, bwd.test_spmm_with_explicit_values_is_a_plain_sparse_product]
    for T, w in ((7, 3), (5, 1), (6, 9), (12, 4)):
        calls.append(lambda a=T, b=w: bwd.test_mproduct_t_adjoint_and_closed_forms(a, b))
    for seed in (0, 1, 2):
        calls.append(lambda s=seed: bwd.test_weighted_delta_apply_matches_dense_brute_force(s))
    return calls


def first_failure():
    for call in pins():
        try:
            call()
        except Exception as exc:          # an assertion, or an error the mistake provokes
            return exc
    return None


def test_the_unmodified_oracle_passes_every_pin_called_this_way():
    assert first_failure() is None


@pytest.mark.parametrize("name,good,bad", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, good, bad):
    text = open(SRC).read()
    assert text.count(good) == 1, f"the oracle source no longer contains exactly one: {good}"
    src, lib = tmp_path / "mutant.c", tmp_path / "libmutant.so"
    src.write_text(text.replace(good, bad))
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(lib), str(src), "-lm"])
    oracle._load()                                       # make sure the real one is loaded, then swap
    real = oracle._lib
    mutant = ctypes.CDLL(str(lib))
    for attr in dir(real):                               # same prototypes as the real library
        fn = getattr(real, attr, None)
        if attr.startswith("oracle_") and hasattr(fn, "argtypes"):
            getattr(mutant, attr).argtypes = fn.argtypes
            getattr(mutant, attr).restype = fn.restype
    oracle._lib = mutant
    try:
        caught = first_failure()
    finally:
        oracle._lib = real
    assert caught is not None, f"no pin noticed: {name}"


# ---- the same for the parts of the oracle written in Python (numpy) ---------------------------------------------
PY_SRC = os.path.join(os.path.dirname(HERE), "oracle", "__init__.py")

PY_MUTANTS = [
    ("weighted normalisation uses the row factor twice", "return val * dinv[rows] * dinv[colidx]", "return val * dinv[rows] * dinv[rows]"),
    ("weighted normalisation: a vertex without entries poisons its neighbours", "dinv = np.where(d > 0.0, 1.0 / np.sqrt(np.where(d > 0.0, d, 1.0)), 0.0)",
     "with np.errstate(all='ignore'):\n        dinv = 1.0 / np.sqrt(d)"),
    ("weighted normalisation counts entries instead of adding values", "d = np.array([val[rowptr[u]:rowptr[u + 1]].sum() for u in range(n)])",
     "d = np.array([float(rowptr[u + 1] - rowptr[u]) for u in range(n)])"),
    ("combination keeps entries that cancel", "keep = total != 0.0", "keep = np.ones(total.size, dtype=bool)"),
    ("combination: the diagonal rule is ignored", "    if diag != 0.0:\n        total = np.where(", "    if False:\n        total = np.where("),
    ("combination: the diagonal rule hits the whole matrix", "total = np.where((uniq >> 32) == (uniq & 0xffffffff), float(diag), total)",
     "total = np.where((uniq >> 32) >= 0, float(diag), total)"),
    ("combination ignores the weight of the removed snapshot", "wts.append(np.full(ci.size, float(scale)))", "wts.append(np.full(ci.size, abs(float(scale))))"),
    ("combination forgets the values of S", "wts.append(np.ones(ci.size) if len(op) < 3 or op[2] is None else _a(op[2], np.float64))",
     "wts.append(np.ones(ci.size))"),
    ("LSTM: forget and input gates exchanged", "c2 = _sig(af) * c + _sig(ai) * np.tanh(ag)\n    return", "c2 = _sig(ai) * c + _sig(af) * np.tanh(ag)\n    return"),
    ("LSTM backward: cell gradient without the carried part", "d_c2 = d_h * o * (1.0 - tc * tc) + (0.0 if d_c is None else _a(d_c, np.float64))",
     "d_c2 = d_h * o * (1.0 - tc * tc)"),
    ("LSTM backward: tanh derivative of the cell gate missing", "d_c2 * i * (1.0 - g * g)", "d_c2 * i"),
    ("LSTM backward: output gate's gradient uses the cell state, not its tanh", "d_h * tc * o * (1.0 - o)", "d_h * c2 * o * (1.0 - o)"),
    ("skip connection backward without the ReLU mask", "d_y = d_y * (np.concatenate([y0, y1], axis=1) > 0.0)", "d_y = d_y * 1.0"),
    ("skip connection backward drops the path through Y1", "spmm_t(rowptr, colidx, d_y0 + input_grad(d_y1, w))", "spmm_t(rowptr, colidx, d_y0)"),
    ("transpose: the entries of a new row come out in descending order", "order = np.lexsort((rows, colidx))", "order = np.lexsort((-rows, colidx))"),
    ("transpose: row pointers counted from the rows, not the columns", "np.cumsum(np.bincount(colidx, minlength=n), out=rowptr_t[1:])",
     "np.cumsum(np.bincount(rows, minlength=n), out=rowptr_t[1:])"),
    ("transposed list sorted by the old row", "order = np.lexsort((row, col))", "order = np.lexsort((col, row))"),
    ("evolving weights: gradient reaches W through one product only", "carry = d_x + d_hp", "carry = d_hp"),
    ("evolving weights: the cell state is not carried past the first step", "w, c = lstm_cell(ws[-1], ws[-1], cs[-1], u_x, u_h, bias)",
     "w, c = lstm_cell(ws[-1], ws[-1], cs[0], u_x, u_h, bias)"),
    ("evolving weights: the hidden state stays the initial weight", "w, c = lstm_cell(ws[-1], ws[-1], cs[-1], u_x, u_h, bias)",
     "w, c = lstm_cell(ws[-1], ws[0], cs[-1], u_x, u_h, bias)"),
    ("evolving weights: the input stays the initial weight", "w, c = lstm_cell(ws[-1], ws[-1], cs[-1], u_x, u_h, bias)",
     "w, c = lstm_cell(ws[0], ws[-1], cs[-1], u_x, u_h, bias)"),
]


def py_pins():
    calls = [bwd.test_weighted_normalisation_reduces_to_eqn_1_and_matches_the_dense_form, bwd.test_csr_combine_special_cases,
             bwd.test_sliding_window_sum_by_csr_combine_equals_the_windowed_sum, bwd.test_edge_life_smoothing_matches_hand_worked_series,
             bwd.test_summed_diagonal_is_the_m_transform_of_the_adjacency_tensor,
             bwd.test_lstm_cell_backward_matches_finite_differences, bwd.test_cdgcn_gcn_backward_matches_finite_differences,
             bwd.test_evolving_weights_backward_matches_finite_differences,
             bwd.test_evolving_weights_recurrence_beyond_the_first_step, bwd.test_transposed_snapshot_and_lists]
    for seed in (0, 1, 2):
        calls.append(lambda s=seed: bwd.test_csr_combine_matches_dense_matrices(s))
    calls += [getattr(bwd, n) for n in dir(bwd) if n.startswith("test_lstm_cell_matches") or n.startswith("test_cdgcn_gcn_matches")]
    return calls


def py_first_failure():
    for call in py_pins():
        try:
            call()
        except Exception as exc:
            return exc
    return None


def test_the_unmodified_python_oracle_passes_these_pins():
    assert py_first_failure() is None


@pytest.mark.parametrize("name,good,bad", PY_MUTANTS, ids=[m[0] for m in PY_MUTANTS])
def test_a_planted_mistake_in_the_python_oracle_is_caught(name, good, bad):
    import types
    text = open(PY_SRC).read()
    assert text.count(good) == 1, f"the oracle source no longer contains exactly one: {good}"
    mutant = types.ModuleType("oracle_mutant")
    mutant.__file__ = PY_SRC                              # it finds the same C library
    mutant.__package__ = "oracle"
    exec(compile(text.replace(good, bad), PY_SRC, "exec"), mutant.__dict__)
    saved = {}
    for attr, fn in vars(mutant).items():                 # the pins call oracle.<function>: hand them the mutant's
        if callable(fn) and not attr.startswith("_") and hasattr(oracle, attr) and getattr(fn, "__module__", None) == "oracle_mutant":
            saved[attr] = getattr(oracle, attr)
            setattr(oracle, attr, fn)
    try:
        caught = py_first_failure()
    finally:
        for attr, fn in saved.items():
            setattr(oracle, attr, fn)
    assert caught is not None, f"no pin noticed: {name}"
