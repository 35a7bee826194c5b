"""Python face of the CPU oracle (oracle/dgnn_oracle.c).

TEST INFRASTRUCTURE ONLY.  Importers are the tests, the smoke check and the CPU-baseline leg
of the benchmark; the product package never imports this and this never imports the product.
Arrays go in and out as numpy; real numbers are float64 throughout.

Passages followed: reconstruction from a graph difference -- Section "Graph-difference Based
Input Transfer"; normalised adjacency -- Eqn (1); GCN operation -- Eqn (2); M-transform and
its matrix M -- Section "TM-GCN"; gradient propagation through a block in the reverse direction
-- Section "Gradient Checkpoint" (the adjoint of each forward step); the sliding-window sum of
snapshots and its normalisation -- Section "Smoothening the Input Graphs" with Eqn (1); the GCN
operation with skip connection and the LSTM over time -- Section "CD-GCN"; the LSTM over the
weights -- Section "EvolveGCN"; and the adjoints of those; the transposed snapshot and lists the
reverse pass of a directed graph needs -- Section "Gradient Checkpoint".  The parts added in numpy below are
fp64 like the C part.  Parity status: every function here is pinned by tests that do not call
it to produce their own expectation (dense brute force, closed forms, hand-worked fixtures under
tests/golden/, a library LSTM cell, central differences); tests/test_oracle_mutants.py plants
mistakes in copies of both sources and requires those pins to fail.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgnn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_csr_from_edges.restype = _i64
        lib.oracle_csr_from_edges.argtypes = [_i64, _i32p, _i32p, _i64, _i32p, _i32p, _i64]
        lib.oracle_delta_apply.restype = _i64
        lib.oracle_delta_apply.argtypes = [_i64, _i32p, _i32p, _i32p, _i32p, _i64, _i32p, _i32p, _i64,
                                           _i32p, _i32p, _i64]
        lib.oracle_delta_apply_weighted.restype = _i64
        lib.oracle_delta_apply_weighted.argtypes = [_i64, _i32p, _i32p, _f64p, _i32p, _i32p, _f64p, _i64, _i32p, _i32p, _i64,
                                                    _i32p, _i32p, _f64p, _i64, _i32p, _i32p, _f64p, _i64]
        lib.oracle_gcn_values.restype = None
        lib.oracle_gcn_values.argtypes = [_i64, _i32p, _i32p, _f64p]
        lib.oracle_xw.restype = None
        lib.oracle_xw.argtypes = [_i64, _i64, _i64, _f64p, _f64p, _f64p]
        lib.oracle_spmm.restype = None
        lib.oracle_spmm.argtypes = [_i64, _i32p, _i32p, _f64p, _f64p, _i64, ctypes.c_int, _i64p, _i64, _f64p]
        lib.oracle_m_matrix.restype = None
        lib.oracle_m_matrix.argtypes = [_i64, _i64, _f64p]
        lib.oracle_mproduct.restype = None
        lib.oracle_mproduct.argtypes = [_i64, _i64, _f64p, _f64p, _f64p]
        lib.oracle_spmm_t.restype = None
        lib.oracle_spmm_t.argtypes = [_i64, _i32p, _i32p, _f64p, _f64p, _i64, _f64p]
        lib.oracle_weight_grad.restype = None
        lib.oracle_weight_grad.argtypes = [_i64, _i64, _i64, _f64p, _f64p, _f64p]
        lib.oracle_mproduct_t.restype = None
        lib.oracle_mproduct_t.argtypes = [_i64, _i64, _f64p, _f64p, _f64p]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _a(x, dt):
    return np.ascontiguousarray(np.asarray(x), dtype=dt)


def _p(a, ptype):
    return a.ctypes.data_as(ptype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(t: int) -> None:
    _load().oracle_set_threads(int(t))


def csr_from_edges(n: int, row, col) -> Tuple[np.ndarray, np.ndarray]:
    """Edge list (any order, repeats allowed) -> canonical CSR (rowptr int32[n+1], colidx int32)."""
    row, col = _a(row, np.int32), _a(col, np.int32)
    m = row.size
    rowptr = np.zeros(n + 1, np.int32)
    colidx = np.zeros(max(m, 1), np.int32)
    rc = _load().oracle_csr_from_edges(n, _p(row, _i32p), _p(col, _i32p), m, _p(rowptr, _i32p),
                                       _p(colidx, _i32p), colidx.size)
    if rc < 0:
        raise ValueError(f"oracle_csr_from_edges failed: {rc}")
    return rowptr, colidx[:rc].copy()


def delta_apply(n: int, rowptr, colidx, add_row, add_col, del_row, del_col) -> Tuple[np.ndarray, np.ndarray]:
    """E_{i+1} = (E_i minus deleted edges) union added edges, returned as canonical CSR."""
    rowptr, colidx = _a(rowptr, np.int32), _a(colidx, np.int32)
    ar, ac, dr, dc = (_a(x, np.int32) for x in (add_row, add_col, del_row, del_col))
    cap = int(rowptr[n]) + ar.size + 1
    rp = np.zeros(n + 1, np.int32)
    ci = np.zeros(cap, np.int32)
    rc = _load().oracle_delta_apply(n, _p(rowptr, _i32p), _p(colidx, _i32p), _p(ar, _i32p), _p(ac, _i32p),
                                    ar.size, _p(dr, _i32p), _p(dc, _i32p), dr.size, _p(rp, _i32p),
                                    _p(ci, _i32p), cap)
    if rc < 0:
        raise ValueError(f"oracle_delta_apply failed: {rc}")
    return rp, ci[:rc].copy()


def delta_apply_weighted(n: int, rowptr, colidx, val, add=None, dele=None, upd=None):
    """Snapshots with a value per stored entry: (prev minus deleted edges, values replaced where `upd` names the
    edge) plus the added edges with their values.  add = (row, col, val), dele = (row, col), upd = (row, col, val);
    returns (rowptr, colidx, val) in canonical order."""
    rowptr, colidx, val = _a(rowptr, np.int32), _a(colidx, np.int32), _a(val, np.float64)
    e_i, e_f = np.zeros(0, np.int32), np.zeros(0, np.float64)
    ar, ac, av = (_a(add[0], np.int32), _a(add[1], np.int32), _a(add[2], np.float64)) if add is not None else (e_i, e_i, e_f)
    dr, dc = (_a(dele[0], np.int32), _a(dele[1], np.int32)) if dele is not None else (e_i, e_i)
    ur, uc, uv = (_a(upd[0], np.int32), _a(upd[1], np.int32), _a(upd[2], np.float64)) if upd is not None else (e_i, e_i, e_f)
    cap = int(rowptr[n]) + ar.size + 1
    rp, ci, vo = np.zeros(n + 1, np.int32), np.zeros(cap, np.int32), np.zeros(cap, np.float64)
    rc = _load().oracle_delta_apply_weighted(n, _p(rowptr, _i32p), _p(colidx, _i32p), _p(val, _f64p),
                                             _p(ar, _i32p), _p(ac, _i32p), _p(av, _f64p), ar.size,
                                             _p(dr, _i32p), _p(dc, _i32p), dr.size,
                                             _p(ur, _i32p), _p(uc, _i32p), _p(uv, _f64p), ur.size,
                                             _p(rp, _i32p), _p(ci, _i32p), _p(vo, _f64p), cap)
    if rc < 0:
        raise ValueError(f"oracle_delta_apply_weighted failed: {rc}")
    return rp, ci[:rc].copy(), vo[:rc].copy()


def gcn_values(rowptr, colidx) -> np.ndarray:
    """Per stored entry (u,v) of A+I: 1/sqrt((1+deg_u)(1+deg_v)), Eqn (1)."""
    rowptr, colidx = _a(rowptr, np.int32), _a(colidx, np.int32)
    n = rowptr.size - 1
    val = np.zeros(max(colidx.size, 1), np.float64)
    _load().oracle_gcn_values(n, _p(rowptr, _i32p), _p(colidx, _i32p), _p(val, _f64p))
    return val[:colidx.size]


def xw(x, w) -> np.ndarray:
    x, w = _a(x, np.float64), _a(w, np.float64)
    n, fi = x.shape
    fo = w.shape[1]
    assert w.shape[0] == fi
    h = np.zeros((n, fo), np.float64)
    _load().oracle_xw(n, fi, fo, _p(x, _f64p), _p(w, _f64p), _p(h, _f64p))
    return h


def spmm(rowptr, colidx, h, relu: bool = False, rows=None, val: Optional[np.ndarray] = None) -> np.ndarray:
    """sigma?(A~ H).  `rows` (int64 indices) restricts the output to those rows, in that order."""
    rowptr, colidx, h = _a(rowptr, np.int32), _a(colidx, np.int32), _a(h, np.float64)
    n = rowptr.size - 1
    f = h.shape[1]
    assert h.shape[0] == n
    if val is None:
        val = gcn_values(rowptr, colidx)
    val = _a(val, np.float64)
    if rows is None:
        z = np.zeros((n, f), np.float64)
        rp, nr = None, 0
    else:
        rows = _a(rows, np.int64)
        z = np.zeros((rows.size, f), np.float64)
        rp, nr = _p(rows, _i64p), rows.size
    _load().oracle_spmm(n, _p(rowptr, _i32p), _p(colidx, _i32p), _p(val, _f64p), _p(h, _f64p), f,
                        int(bool(relu)), rp, nr, _p(z, _f64p))
    return z


def m_matrix(T: int, w: int) -> np.ndarray:
    """Dense T x T matrix of the M-transform: M[t][k] = 1/min(w,t) on max(1,t-w+1) <= k <= t (1-based)."""
    M = np.zeros((T, T), np.float64)
    _load().oracle_m_matrix(T, w, _p(M, _f64p))
    return M


def mproduct(z, M) -> np.ndarray:
    """Y = Z x_1 M for Z of shape [T, ...]; M is a dense T x T matrix."""
    z, M = _a(z, np.float64), _a(M, np.float64)
    T = z.shape[0]
    assert M.shape == (T, T)
    frame = int(np.prod(z.shape[1:]))
    y = np.zeros_like(z)
    _load().oracle_mproduct(T, frame, _p(M, _f64p), _p(z, _f64p), _p(y, _f64p))
    return y


def gcn_layer(rowptr, colidx, x, w, relu: bool = False, rows=None) -> np.ndarray:
    """sigma?(A~ (X W)), Eqn (2)."""
    return spmm(rowptr, colidx, xw(x, w), relu=relu, rows=rows)


# ---- backward of the same path (Section "Gradient Checkpoint") ------------------------------------

def spmm_t(rowptr, colidx, g, val: Optional[np.ndarray] = None) -> np.ndarray:
    """A~^T G: the adjoint of the aggregation of Eqn (2)."""
    rowptr, colidx, g = _a(rowptr, np.int32), _a(colidx, np.int32), _a(g, np.float64)
    n = rowptr.size - 1
    f = g.shape[1]
    assert g.shape[0] == n
    if val is None:
        val = gcn_values(rowptr, colidx)
    val = _a(val, np.float64)
    out = np.zeros((n, f), np.float64)
    _load().oracle_spmm_t(n, _p(rowptr, _i32p), _p(colidx, _i32p), _p(val, _f64p), _p(g, _f64p), f, _p(out, _f64p))
    return out


def weight_grad(x, g) -> np.ndarray:
    """dW = X^T G for H = X W and G = dL/dH."""
    x, g = _a(x, np.float64), _a(g, np.float64)
    n, fi = x.shape
    fo = g.shape[1]
    assert g.shape[0] == n
    dw = np.zeros((fi, fo), np.float64)
    _load().oracle_weight_grad(n, fi, fo, _p(x, _f64p), _p(g, _f64p), _p(dw, _f64p))
    return dw


def input_grad(g, w) -> np.ndarray:
    """dX = G W^T for H = X W and G = dL/dH."""
    return xw(g, _a(w, np.float64).T.copy())


def mproduct_t(g, M) -> np.ndarray:
    """G x_1 M^T: the adjoint of the M-transform; out_k = sum_t M[t][k] G_t."""
    g, M = _a(g, np.float64), _a(M, np.float64)
    T = g.shape[0]
    assert M.shape == (T, T)
    frame = int(np.prod(g.shape[1:]))
    out = np.zeros_like(g)
    _load().oracle_mproduct_t(T, frame, _p(M, _f64p), _p(g, _f64p), _p(out, _f64p))
    return out


def relu_grad(g, z) -> np.ndarray:
    """Gradient through Z = max(P, 0): G where Z > 0, else 0 (Z > 0 exactly where P > 0)."""
    return np.where(_a(z, np.float64) > 0.0, _a(g, np.float64), 0.0)


def gcn_layer_backward(rowptr, colidx, x, w, z, g_z):
    """Gradients of Z = relu(A~ (X W)) for upstream g_z = dL/dZ: returns (dW, dX)."""
    g_h = spmm_t(rowptr, colidx, relu_grad(g_z, z))
    return weight_grad(x, g_h), input_grad(g_h, w)


# ---- CD-GCN (Section "CD-GCN"): GCN operation with skip connection, LSTM over time ------------------

def cdgcn_gcn(rowptr, colidx, x, w) -> np.ndarray:
    """Y = relu(Y0 o Y1) with Y0 = A~ X and Y1 = Y0 W; F + F' features per vertex."""
    y0 = spmm(rowptr, colidx, _a(x, np.float64))
    y1 = xw(y0, w)
    return np.maximum(np.concatenate([y0, y1], axis=1), 0.0)


def _sig(a):
    return 1.0 / (1.0 + np.exp(-a))


def lstm_cell(x, h, c, w_x, w_h, bias):
    """One step of the standard LSTM (state (h, c)); gates in the order (input, forget, cell, output):
    a = x W_x + h W_h + b,  c' = sig(a_f) c + sig(a_i) tanh(a_g),  h' = sig(a_o) tanh(c')."""
    x, h, c = _a(x, np.float64), _a(h, np.float64), _a(c, np.float64)
    a = xw(x, w_x) + xw(h, w_h) + (0.0 if bias is None else _a(bias, np.float64)[None, :])
    hid = c.shape[1]
    ai, af, ag, ao = (a[:, q * hid:(q + 1) * hid] for q in range(4))
    c2 = _sig(af) * c + _sig(ai) * np.tanh(ag)
    return _sig(ao) * np.tanh(c2), c2


def gcn_values_weighted(rowptr, colidx, val) -> np.ndarray:
    """Eqn (1) for a snapshot with a value per stored entry: val(u,v) / sqrt(d_u d_v) with d_u the sum of the
    values of row u (self loop included); for values that are all 1 this is gcn_values."""
    rowptr, colidx, val = _a(rowptr, np.int32), _a(colidx, np.int32), _a(val, np.float64)
    n = rowptr.size - 1
    d = np.array([val[rowptr[u]:rowptr[u + 1]].sum() for u in range(n)])
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    # a vertex whose row sum is not positive has no normalisation: its factor is taken as 0 (it neither sends nor receives)
    dinv = np.where(d > 0.0, 1.0 / np.sqrt(np.where(d > 0.0, d, 1.0)), 0.0)
    return val * dinv[rows] * dinv[colidx]


def csr_combine(n: int, s, a_in=None, alpha: float = 1.0, a_out=None, beta: float = -1.0, diag: float = 0.0):
    """S + alpha * A_in + beta * A_out as sparse matrices, entries whose result is exactly 0 removed: one step of
    the sliding-window sum of Section "Smoothening the Input Graphs" (S_t = S_{t-1} + A_t - A_{t-l}).
    s = (rowptr, colidx, val or None for all ones); a_in, a_out = (rowptr, colidx) of unweighted snapshots, or
    None.  Returns (rowptr, colidx, val) with val in float64.  Written as the definition: every stored entry of
    the three operands is one term (row, col, weight), terms of equal (row, col) are added up.
    diag != 0: the operands hold A + I, the section smooths A and Eqn (1) adds I afterwards, once: every stored
    diagonal entry of the result is set to `diag` (1 for the edge-life sum) instead of the number of snapshots in
    the window."""
    keys, wts = [], []
    for op, scale in ((s, None), (a_in, alpha), (a_out, beta)):
        if op is None:
            continue
        rp, ci = _a(op[0], np.int32), _a(op[1], np.int32)
        rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rp))
        keys.append((rows << 32) | ci.astype(np.int64))
        if scale is None:
            wts.append(np.ones(ci.size) if len(op) < 3 or op[2] is None else _a(op[2], np.float64))
        else:
            wts.append(np.full(ci.size, float(scale)))
    keys, wts = np.concatenate(keys), np.concatenate(wts)
    uniq, inv = np.unique(keys, return_inverse=True)
    total = np.zeros(uniq.size)
    np.add.at(total, inv, wts)
    keep = total != 0.0
    uniq, total = uniq[keep], total[keep]
    if diag != 0.0:
        total = np.where((uniq >> 32) == (uniq & 0xffffffff), float(diag), total)
    rowptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(uniq >> 32, minlength=n), out=rowptr[1:])
    return rowptr, (uniq & 0xffffffff).astype(np.int32), total


def csr_transpose(n: int, rowptr, colidx, val=None):
    """CSR of the transposed matrix, canonical form (Section "Gradient Checkpoint": the reverse pass aggregates with
    A~^T).  The definition written out: the stored pairs (u, v) become (v, u), sorted by (v, u)."""
    rowptr, colidx = _a(rowptr, np.int32), _a(colidx, np.int32)
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    order = np.lexsort((rows, colidx))                    # by the old column, then by the old row
    rowptr_t = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(colidx, minlength=n), out=rowptr_t[1:])
    out = (rowptr_t, rows[order].astype(np.int32))
    return out if val is None else out + (_a(val, np.float64)[order],)


def coo_transpose(row, col):
    """The pairs (col, row), sorted ascending: a difference list of the transposed series."""
    row, col = _a(row, np.int32), _a(col, np.int32)
    order = np.lexsort((row, col))
    return col[order], row[order]


def lstm_cell_backward(x, h, c, w_x, w_h, bias, d_h, d_c=None):
    """Adjoint of lstm_cell: given dL/dh' (d_h) and dL/dc' (d_c, zero if None), returns
    (d_a, d_x, d_h_prev, d_c_prev, d_w_x, d_w_h, d_b), d_a being dL/d(pre-activations) [n, 4 hid].
    Chain rule on c' = sig(a_f) c + sig(a_i) tanh(a_g), h' = sig(a_o) tanh(c')."""
    x, h, c = _a(x, np.float64), _a(h, np.float64), _a(c, np.float64)
    w_x, w_h = _a(w_x, np.float64), _a(w_h, np.float64)
    a = xw(x, w_x) + xw(h, w_h) + (0.0 if bias is None else _a(bias, np.float64)[None, :])
    hid = c.shape[1]
    ai, af, ag, ao = (a[:, q * hid:(q + 1) * hid] for q in range(4))
    i, f, g, o = _sig(ai), _sig(af), np.tanh(ag), _sig(ao)
    c2 = f * c + i * g
    tc = np.tanh(c2)
    d_h = _a(d_h, np.float64)
    d_c2 = d_h * o * (1.0 - tc * tc) + (0.0 if d_c is None else _a(d_c, np.float64))
    d_a = np.concatenate([d_c2 * g * i * (1.0 - i), d_c2 * c * f * (1.0 - f), d_c2 * i * (1.0 - g * g),
                          d_h * tc * o * (1.0 - o)], axis=1)
    return (d_a, input_grad(d_a, w_x), input_grad(d_a, w_h), d_c2 * f, weight_grad(x, d_a), weight_grad(h, d_a),
            d_a.sum(axis=0))


def cdgcn_gcn_backward(rowptr, colidx, x, w, d_y):
    """Adjoint of cdgcn_gcn with respect to W and X: Y = relu(Y0 o Y1), Y0 = A~ X, Y1 = Y0 W.
    Returns (d_w, d_x)."""
    x, w, d_y = _a(x, np.float64), _a(w, np.float64), _a(d_y, np.float64)
    f = x.shape[1]
    y0 = spmm(rowptr, colidx, x)
    y1 = xw(y0, w)
    d_y = d_y * (np.concatenate([y0, y1], axis=1) > 0.0)
    d_y0, d_y1 = d_y[:, :f], d_y[:, f:]
    d_w = weight_grad(y0, d_y1)
    return d_w, spmm_t(rowptr, colidx, d_y0 + input_grad(d_y1, w))


def evolve_weights(w0, u_x, u_h, bias, T: int):
    """Section "EvolveGCN": W_t = LSTM(W_{t-1}), read as the EGCN-O variant it names: the weight matrix is the
    LSTM's input and its hidden state (rows = batch), with a cell state C of the same shape, C_0 = 0.
    Returns ([W_1 .. W_T], [C_0 .. C_T])."""
    ws, cs = [_a(w0, np.float64)], [np.zeros(np.shape(w0))]
    for _ in range(T):
        w, c = lstm_cell(ws[-1], ws[-1], cs[-1], u_x, u_h, bias)
        ws.append(w); cs.append(c)
    return ws[1:], cs


def evolve_weights_backward(w0, u_x, u_h, bias, d_w):
    """Adjoint of evolve_weights for L = sum_t <d_w[t-1], W_t>: (dU_x, dU_h, db, dW_0)."""
    T = len(d_w)
    ws, cs = evolve_weights(w0, u_x, u_h, bias, T)
    ws = [_a(w0, np.float64)] + ws
    d_ux = d_uh = d_b = 0.0
    carry, d_c = 0.0, None
    for t in range(T, 0, -1):
        _, d_x, d_hp, d_c, a, b, g = lstm_cell_backward(ws[t - 1], ws[t - 1], cs[t - 1], u_x, u_h, bias,
                                                       _a(d_w[t - 1], np.float64) + carry, d_c)
        d_ux, d_uh, d_b = d_ux + a, d_uh + b, d_b + g
        carry = d_x + d_hp                    # W_{t-1} is input and hidden state at once
    return d_ux, d_uh, d_b, carry
