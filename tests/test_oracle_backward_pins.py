"""Pins for the backward half of the CPU oracle (gradient propagation through a block, Section
"Gradient Checkpoint").  Each adjoint is checked against things that are not itself: the inner-product
identity <A^T g, h> = <g, A h> with the forward oracle (pinned elsewhere) on the other side, dense
transposes built here in numpy, closed forms, and central finite differences of the forward path in
double precision.  All CPU."""
import numpy as np
import pytest

import oracle
from test_oracle_pins import csr_from_dense, dense_gcn_matrix, random_graph_dense


def _graph(n, p, seed, symmetric):
    rng = np.random.default_rng(seed)
    a = random_graph_dense(n, p, rng, symmetric)
    rp, ci = csr_from_dense(a)
    return a, rp, ci, rng


# ----------------------------------------------------------------------------- A~^T G
@pytest.mark.parametrize("symmetric", [False, True])
def test_spmm_t_matches_dense_transpose(symmetric):
    a, rp, ci, rng = _graph(57, 0.1, 11, symmetric)
    g = rng.standard_normal((57, 5))
    want = dense_gcn_matrix(a).T @ g
    np.testing.assert_allclose(oracle.spmm_t(rp, ci, g), want, rtol=1e-12, atol=1e-13)


def test_spmm_t_is_the_adjoint_of_spmm():
    _, rp, ci, rng = _graph(200, 0.05, 12, False)
    g, h = rng.standard_normal((200, 7)), rng.standard_normal((200, 7))
    lhs = np.sum(oracle.spmm_t(rp, ci, g) * h)
    rhs = np.sum(g * oracle.spmm(rp, ci, h))
    assert abs(lhs - rhs) <= 1e-11 * (abs(lhs) + 1)


def test_spmm_t_equals_spmm_on_undirected_graphs_only():
    _, rp, ci, rng = _graph(80, 0.08, 13, True)
    g = rng.standard_normal((80, 3))
    np.testing.assert_allclose(oracle.spmm_t(rp, ci, g), oracle.spmm(rp, ci, g), rtol=1e-12, atol=1e-13)
    _, rp, ci, rng = _graph(80, 0.08, 14, False)
    g = rng.standard_normal((80, 3))
    assert np.max(np.abs(oracle.spmm_t(rp, ci, g) - oracle.spmm(rp, ci, g))) > 1e-3


def test_spmm_t_closed_form_sqrt_degree():
    # y_u = sqrt(1 + deg_u): every stored (u, v) sends 1 / sqrt(1 + deg_v) to v, so
    # (A~^T y)_v = (number of stored entries in column v) / sqrt(1 + deg_v), directed or not.
    a, rp, ci, _ = _graph(120, 0.06, 15, False)
    d = np.diff(rp).astype(np.float64)
    col_count = a.sum(axis=0).astype(np.float64)
    got = oracle.spmm_t(rp, ci, np.sqrt(d)[:, None])[:, 0]
    np.testing.assert_allclose(got, col_count / np.sqrt(d), rtol=1e-12)


# ----------------------------------------------------------------------------- X^T G and G W^T
def test_weight_grad_special_cases_and_numpy():
    rng = np.random.default_rng(16)
    g = rng.standard_normal((40, 6))
    x = np.zeros((40, 9))
    x[np.arange(9), np.arange(9)] = 1.0                       # X = [I; 0]  =>  X^T G = first rows of G
    np.testing.assert_array_equal(oracle.weight_grad(x, g), g[:9])
    x = rng.standard_normal((40, 9))
    np.testing.assert_allclose(oracle.weight_grad(x, g), x.T @ g, rtol=1e-12, atol=1e-13)
    # transposing the roles transposes the result: (X^T G)^T = G^T X
    np.testing.assert_allclose(oracle.weight_grad(g, x), oracle.weight_grad(x, g).T, rtol=1e-12, atol=1e-13)


def test_input_grad_matches_numpy_and_adjoint():
    rng = np.random.default_rng(17)
    g, w, x = rng.standard_normal((30, 6)), rng.standard_normal((9, 6)), rng.standard_normal((30, 9))
    np.testing.assert_allclose(oracle.input_grad(g, w), g @ w.T, rtol=1e-12, atol=1e-13)
    lhs, rhs = np.sum(oracle.input_grad(g, w) * x), np.sum(g * oracle.xw(x, w))   # <G W^T, X> = <G, X W>
    assert abs(lhs - rhs) <= 1e-11 * (abs(lhs) + 1)


# ----------------------------------------------------------------------------- G x_1 M^T
@pytest.mark.parametrize("T,w", [(7, 3), (5, 1), (6, 9), (12, 4)])
def test_mproduct_t_adjoint_and_closed_forms(T, w):
    rng = np.random.default_rng(18 + T)
    M = oracle.m_matrix(T, w)
    g, z = rng.standard_normal((T, 4, 3)), rng.standard_normal((T, 4, 3))
    got = oracle.mproduct_t(g, M)
    lhs, rhs = np.sum(got * z), np.sum(g * oracle.mproduct(z, M))
    assert abs(lhs - rhs) <= 1e-11 * (abs(lhs) + 1)
    # written out from the band: out_k = sum_{t=k}^{min(T, k+w-1)} g_t / min(w, t)   (1-based)
    want = np.zeros_like(g)
    for k in range(1, T + 1):
        for t in range(k, min(T, k + w - 1) + 1):
            want[k - 1] += g[t - 1] / min(w, t)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    if w == 1:
        np.testing.assert_array_equal(got, g)
    if w >= T:   # all-ones gradient: harmonic tail sums H_T - H_{k-1}
        ones = oracle.mproduct_t(np.ones((T, 1)), M)[:, 0]
        harm = np.cumsum(1.0 / np.arange(1, T + 1))
        np.testing.assert_allclose(ones, harm[-1] - np.concatenate([[0.0], harm[:-1]]), rtol=1e-12)


# ----------------------------------------------------------------------------- whole layer, finite differences
def _layer_loss(rp, ci, xs, w, M, c):
    z = np.stack([oracle.gcn_layer(rp_t, ci_t, x_t, w, relu=True) for rp_t, ci_t, x_t in zip(rp, ci, xs)])
    return float(np.sum(c * oracle.mproduct(z, M))), z


def test_layer_backward_matches_finite_differences():
    T, n, f, wdw = 4, 23, 3, 2
    rng = np.random.default_rng(19)
    rps, cis = [], []
    for t in range(T):
        a = random_graph_dense(n, 0.15, rng, False)
        r, c = csr_from_dense(a)
        rps.append(r)
        cis.append(c)
    xs = [rng.standard_normal((n, f)) for _ in range(T)]
    w = rng.standard_normal((f, f))
    c = rng.standard_normal((T, n, f))
    M = oracle.m_matrix(T, wdw)
    loss, z = _layer_loss(rps, cis, xs, w, M, c)
    pre = np.stack([oracle.gcn_layer(r, ci_, x, w, relu=False) for r, ci_, x in zip(rps, cis, xs)])
    assert np.min(np.abs(pre)) > 1e-4          # no pre-activation sits on the kink of the ReLU

    g_z = oracle.mproduct_t(c, M)               # dL/dZ
    dw = np.zeros_like(w)
    dxs = []
    for t in range(T):
        dw_t, dx_t = oracle.gcn_layer_backward(rps[t], cis[t], xs[t], w, z[t], g_z[t])
        dw += dw_t
        dxs.append(dx_t)

    eps = 1e-6
    for (i, j) in [(0, 0), (1, 2), (2, 1)]:
        wp, wm = w.copy(), w.copy()
        wp[i, j] += eps
        wm[i, j] -= eps
        fd = (_layer_loss(rps, cis, xs, wp, M, c)[0] - _layer_loss(rps, cis, xs, wm, M, c)[0]) / (2 * eps)
        assert abs(fd - dw[i, j]) <= 1e-6 * (abs(fd) + 1), (i, j, fd, dw[i, j])
    for (t, u, j) in [(0, 0, 0), (2, 7, 1), (3, 22, 2)]:
        xp = [x.copy() for x in xs]
        xm = [x.copy() for x in xs]
        xp[t][u, j] += eps
        xm[t][u, j] -= eps
        fd = (_layer_loss(rps, cis, xp, w, M, c)[0] - _layer_loss(rps, cis, xm, w, M, c)[0]) / (2 * eps)
        assert abs(fd - dxs[t][u, j]) <= 1e-6 * (abs(fd) + 1), (t, u, j, fd, dxs[t][u, j])


def test_relu_grad_masks_where_output_is_zero():
    g = np.array([[1.0, -2.0, 3.0]])
    z = np.array([[0.5, 0.0, 2.0]])
    np.testing.assert_array_equal(oracle.relu_grad(g, z), [[1.0, 0.0, 3.0]])


# ----------------------------------------------------------------------------- snapshots that carry values
def _dense_weighted(n, rp, ci, val):
    w = np.full((n, n), np.nan)
    for u in range(n):
        w[u, ci[rp[u]:rp[u + 1]]] = val[rp[u]:rp[u + 1]]
    return w


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_weighted_delta_apply_matches_dense_brute_force(seed):
    """Dense n x n arrays with NaN for "no edge": deleting writes NaN, updating and adding write the value."""
    n = 40
    a, rp, ci, rng = _graph(n, 0.12, 100 + seed, False)
    val = rng.uniform(0.5, 1.5, ci.size)
    dense = _dense_weighted(n, rp, ci, val)
    present = np.argwhere(a & ~np.eye(n, dtype=bool))
    absent = np.argwhere(~a)
    pick = rng.permutation(len(present))
    dele = present[pick[:15]]
    upd = present[pick[15:40]]
    add = absent[rng.permutation(len(absent))[:20]]
    add_v, upd_v = rng.uniform(2, 3, len(add)), rng.uniform(4, 5, len(upd))
    want = dense.copy()
    want[dele[:, 0], dele[:, 1]] = np.nan
    want[upd[:, 0], upd[:, 1]] = upd_v
    want[add[:, 0], add[:, 1]] = add_v
    # lists in arbitrary order: the oracle does not rely on their order
    rp2, ci2, v2 = oracle.delta_apply_weighted(n, rp, ci, val, add=(add[:, 0], add[:, 1], add_v),
                                               dele=(dele[:, 0], dele[:, 1]), upd=(upd[:, 0], upd[:, 1], upd_v))
    got = _dense_weighted(n, rp2, ci2, v2)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    np.testing.assert_array_equal(got[~np.isnan(want)], want[~np.isnan(want)])
    for u in range(n):
        assert np.all(np.diff(ci2[rp2[u]:rp2[u + 1]]) > 0)
    # the structure is what the unweighted rule gives
    rp3, ci3 = oracle.delta_apply(n, rp, ci, add[:, 0], add[:, 1], dele[:, 0], dele[:, 1])
    assert np.array_equal(rp2, rp3) and np.array_equal(ci2, ci3)
    # and it can be undone: re-adding the deleted edges with their old values, deleting the added ones, writing the
    # old values back
    back = oracle.delta_apply_weighted(n, rp2, ci2, v2, add=(dele[:, 0], dele[:, 1], dense[dele[:, 0], dele[:, 1]]),
                                       dele=(add[:, 0], add[:, 1]), upd=(upd[:, 0], upd[:, 1], dense[upd[:, 0], upd[:, 1]]))
    assert np.array_equal(back[0], rp) and np.array_equal(back[1], ci)
    np.testing.assert_array_equal(back[2], val)


def test_weighted_delta_apply_trivial_cases():
    n = 5
    rp, ci = oracle.csr_from_edges(n, [0, 1, 2, 3, 4, 0, 3], [0, 1, 2, 3, 4, 2, 1])
    val = np.arange(1.0, ci.size + 1)
    same = oracle.delta_apply_weighted(n, rp, ci, val)
    assert np.array_equal(same[0], rp) and np.array_equal(same[1], ci) and np.array_equal(same[2], val)
    only_upd = oracle.delta_apply_weighted(n, rp, ci, val, upd=([0], [2], [9.0]))
    assert np.array_equal(only_upd[1], ci) and only_upd[2][1] == 9.0 and only_upd[2].sum() == val.sum() - val[1] + 9.0


def test_spmm_with_explicit_values_is_a_plain_sparse_product():
    n = 60
    a, rp, ci, rng = _graph(n, 0.1, 200, False)
    val = rng.standard_normal(ci.size)
    h = rng.standard_normal((n, 4))
    dense = np.nan_to_num(_dense_weighted(n, rp, ci, val), nan=0.0)
    np.testing.assert_allclose(oracle.spmm(rp, ci, h, val=val), dense @ h, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.spmm_t(rp, ci, h, val=val), dense.T @ h, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- CD-GCN pieces
def test_lstm_cell_matches_the_library_cell_and_closed_forms():
    import torch
    rng = np.random.default_rng(300)
    n, fin, hid = 17, 6, 5
    x, h, c = rng.standard_normal((n, fin)), rng.standard_normal((n, hid)), rng.standard_normal((n, hid))
    w_x, w_h, b = rng.standard_normal((fin, 4 * hid)), rng.standard_normal((hid, 4 * hid)), rng.standard_normal(4 * hid)
    cell = torch.nn.LSTMCell(fin, hid).double()            # same gate order (input, forget, cell, output)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(w_x.T))
        cell.weight_hh.copy_(torch.from_numpy(w_h.T))
        cell.bias_ih.copy_(torch.from_numpy(b))
        cell.bias_hh.zero_()
        h_t, c_t = cell(torch.from_numpy(x), (torch.from_numpy(h), torch.from_numpy(c)))
    h2, c2 = oracle.lstm_cell(x, h, c, w_x, w_h, b)
    np.testing.assert_allclose(h2, h_t.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(c2, c_t.numpy(), rtol=1e-12, atol=1e-13)
    # all pre-activations zero: every gate is 1/2 and the candidate is 0
    z = np.zeros
    h3, c3 = oracle.lstm_cell(z((n, fin)), z((n, hid)), c, z((fin, 4 * hid)), z((hid, 4 * hid)), None)
    np.testing.assert_allclose(c3, 0.5 * c, rtol=1e-15)
    np.testing.assert_allclose(h3, 0.5 * np.tanh(0.5 * c), rtol=1e-15)


def test_cdgcn_gcn_on_special_graphs():
    rng = np.random.default_rng(301)
    n, f = 9, 3
    x, w = rng.standard_normal((n, f)), rng.standard_normal((f, 4))
    rp, ci = oracle.csr_from_edges(n, np.arange(n), np.arange(n))          # no edges: A~ = I
    y = oracle.cdgcn_gcn(rp, ci, x, w)
    np.testing.assert_allclose(y, np.maximum(np.concatenate([x, x @ w], axis=1), 0.0), rtol=1e-12, atol=1e-13)
    a, rp, ci, _ = _graph(n, 0.4, 302, False)
    dense = dense_gcn_matrix(a)
    y0 = dense @ x
    np.testing.assert_allclose(oracle.cdgcn_gcn(rp, ci, x, w), np.maximum(np.concatenate([y0, y0 @ w], axis=1), 0.0),
                               rtol=1e-12, atol=1e-13)


def test_weighted_normalisation_reduces_to_eqn_1_and_matches_the_dense_form():
    n = 50
    a, rp, ci, rng = _graph(n, 0.15, 400, False)
    np.testing.assert_allclose(oracle.gcn_values_weighted(rp, ci, np.ones(ci.size)), oracle.gcn_values(rp, ci), rtol=1e-14)
    val = rng.uniform(0.5, 3.0, ci.size)
    dense = np.nan_to_num(_dense_weighted(n, rp, ci, val), nan=0.0)
    d = dense.sum(axis=1)
    want = np.diag(d ** -0.5) @ dense @ np.diag(d ** -0.5)
    got = np.nan_to_num(_dense_weighted(n, rp, ci, oracle.gcn_values_weighted(rp, ci, val)), nan=0.0)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
    # a vertex without stored entries that others point to: the entries towards it weigh 0, nothing becomes infinite
    rp2 = np.array([0, 2, 2, 3], dtype=np.int32)                       # row 1 is empty
    ci2 = np.array([0, 1, 2], dtype=np.int32)                          # (0,0), (0,1), (2,2)
    got2 = oracle.gcn_values_weighted(rp2, ci2, np.array([2.0, 2.0, 3.0]))
    np.testing.assert_allclose(got2, [2.0 / 4.0, 0.0, 1.0], rtol=1e-15)
    # sqrt(d) is a fixed vector of the normalised matrix, as in the unweighted case
    np.testing.assert_allclose(oracle.spmm(rp, ci, np.sqrt(d)[:, None], val=oracle.gcn_values_weighted(rp, ci, val))[:, 0],
                               np.sqrt(d), rtol=1e-12)


def _dense_unweighted(n, rp, ci):
    d = np.zeros((n, n))
    for u in range(n):
        d[u, ci[rp[u]:rp[u + 1]]] = 1.0
    return d


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_csr_combine_matches_dense_matrices(seed):
    """S + alpha A_in + beta A_out with dense n x n arrays; entries that cancel must disappear from the structure."""
    n = 40
    rng = np.random.default_rng(seed)
    mats = []
    for p in (0.2, 0.15, 0.1):
        m = rng.random((n, n)) < p
        mats.append(oracle.csr_from_edges(n, *np.nonzero(m)))
    (s_rp, s_ci), a_in, a_out = mats
    s_val = rng.integers(1, 4, s_ci.size).astype(np.float64)
    s_dense = np.nan_to_num(_dense_weighted(n, s_rp, s_ci, s_val), nan=0.0)
    for alpha, beta in ((1.0, -1.0), (2.0, 0.5), (1.0, -2.0)):
        want = s_dense + alpha * _dense_unweighted(n, *a_in) + beta * _dense_unweighted(n, *a_out)
        rp, ci, val = oracle.csr_combine(n, (s_rp, s_ci, s_val), a_in, alpha, a_out, beta)
        assert np.all(val != 0.0)
        got = np.nan_to_num(_dense_weighted(n, rp, ci, val), nan=0.0)
        np.testing.assert_array_equal(got, want)
        assert ci.size == np.count_nonzero(want)                      # nothing stored that is zero, nothing missing
        for u in range(n):
            assert np.all(np.diff(ci[rp[u]:rp[u + 1]]) > 0)           # canonical order within each row


def test_csr_combine_special_cases():
    n = 30
    rng = np.random.default_rng(9)
    s = oracle.csr_from_edges(n, *np.nonzero(rng.random((n, n)) < 0.2))
    a = oracle.csr_from_edges(n, *np.nonzero(rng.random((n, n)) < 0.2))
    ones = np.ones(s[1].size)
    # nothing added, nothing removed: S itself (values all ones when none are given)
    rp, ci, val = oracle.csr_combine(n, s + (None,))
    assert np.array_equal(rp, s[0]) and np.array_equal(ci, s[1]) and np.array_equal(val, ones)
    # S - S is empty, S + S doubles every value
    rp, ci, val = oracle.csr_combine(n, s + (ones,), None, 1.0, s, -1.0)
    assert ci.size == 0 and np.all(rp == 0)
    rp, ci, val = oracle.csr_combine(n, s + (ones,), s, 1.0)
    assert np.array_equal(ci, s[1]) and np.array_equal(val, 2 * ones)
    # adding then removing the same snapshot gives S back
    rp, ci, val = oracle.csr_combine(n, s + (ones,), a, 1.0, a, -1.0)
    assert np.array_equal(rp, s[0]) and np.array_equal(ci, s[1]) and np.array_equal(val, ones)


def test_sliding_window_sum_by_csr_combine_equals_the_windowed_sum():
    """S_t = S_{t-1} + A_t - A_{t-l} carried over a series equals the sum of the last l snapshots formed
    directly (dense), Section "Smoothening the Input Graphs"."""
    n, life, T = 25, 3, 8
    rng = np.random.default_rng(4)
    snaps = [oracle.csr_from_edges(n, *np.nonzero((rng.random((n, n)) < 0.15) | np.eye(n, dtype=bool))) for _ in range(T)]
    s = snaps[0] + (None,)
    for t in range(2, T + 1):
        out = snaps[t - 1 - life] if t - life >= 1 else None
        s = oracle.csr_combine(n, s, snaps[t - 1], 1.0, out, -1.0)
        want = sum(_dense_unweighted(n, *snaps[i - 1]) for i in range(max(1, t - life + 1), t + 1))
        got = np.nan_to_num(_dense_weighted(n, *s), nan=0.0)
        np.testing.assert_array_equal(got, want)


def _central(fun, arr, eps=1e-6):
    """Central differences of the scalar fun() with respect to every entry of arr (changed in place, restored)."""
    out = np.zeros_like(arr)
    it = np.nditer(arr, flags=["multi_index"])
    for _ in it:
        k = it.multi_index
        keep = arr[k]
        arr[k] = keep + eps; up = fun()
        arr[k] = keep - eps; dn = fun()
        arr[k] = keep
        out[k] = (up - dn) / (2 * eps)
    return out


def test_lstm_cell_backward_matches_finite_differences():
    rng = np.random.default_rng(21)
    n, fx, hid = 5, 6, 4
    x, h, c = rng.normal(size=(n, fx)), rng.normal(size=(n, hid)), rng.normal(size=(n, hid))
    w_x, w_h, b = rng.normal(size=(fx, 4 * hid)) / 2, rng.normal(size=(hid, 4 * hid)) / 2, rng.normal(size=4 * hid)
    g_h, g_c = rng.normal(size=(n, hid)), rng.normal(size=(n, hid))

    def loss():
        h2, c2 = oracle.lstm_cell(x, h, c, w_x, w_h, b)
        return float((g_h * h2).sum() + (g_c * c2).sum())

    d_a, d_x, d_hp, d_cp, d_wx, d_wh, d_b = oracle.lstm_cell_backward(x, h, c, w_x, w_h, b, g_h, g_c)
    for got, arr in ((d_x, x), (d_hp, h), (d_cp, c), (d_wx, w_x), (d_wh, w_h), (d_b, b)):
        np.testing.assert_allclose(got, _central(loss, arr), rtol=1e-6, atol=1e-8)
    # without an upstream dL/dc' the cell state still carries gradient through h'
    g_c[:] = 0.0
    got = oracle.lstm_cell_backward(x, h, c, w_x, w_h, b, g_h, None)
    np.testing.assert_allclose(got[3], _central(loss, c), rtol=1e-6, atol=1e-8)


def test_cdgcn_gcn_backward_matches_finite_differences():
    n, f, f2 = 12, 3, 4
    a, rp, ci, rng = _graph(n, 0.3, 77, False)
    x, w, g = rng.normal(size=(n, f)), rng.normal(size=(f, f2)), rng.normal(size=(n, f + f2))

    def loss():
        return float((g * oracle.cdgcn_gcn(rp, ci, x, w)).sum())

    d_w, d_x = oracle.cdgcn_gcn_backward(rp, ci, x, w, g)
    np.testing.assert_allclose(d_w, _central(loss, w), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(d_x, _central(loss, x), rtol=1e-6, atol=1e-8)


def test_evolving_weights_backward_matches_finite_differences():
    rng = np.random.default_rng(31)
    f, f2, T = 5, 3, 4
    w0 = rng.normal(size=(f, f2))
    u_x, u_h, b = rng.normal(size=(f2, 4 * f2)) / 2, rng.normal(size=(f2, 4 * f2)) / 2, rng.normal(size=4 * f2) / 4
    g = [rng.normal(size=(f, f2)) for _ in range(T)]

    def loss():
        ws, _ = oracle.evolve_weights(w0, u_x, u_h, b, T)
        return float(sum((gt * wt).sum() for gt, wt in zip(g, ws)))

    d_ux, d_uh, d_b, d_w0 = oracle.evolve_weights_backward(w0, u_x, u_h, b, g)
    for got, arr in ((d_ux, u_x), (d_uh, u_h), (d_b, b), (d_w0, w0)):
        np.testing.assert_allclose(got, _central(loss, arr), rtol=1e-6, atol=1e-8)
    # the first step alone is one LSTM cell with the weight as input and state
    ws, cs = oracle.evolve_weights(w0, u_x, u_h, b, 1)
    h, c = oracle.lstm_cell(w0, w0, np.zeros_like(w0), u_x, u_h, b)
    assert np.array_equal(ws[0], h) and np.array_equal(cs[1], c)


def test_evolving_weights_recurrence_beyond_the_first_step():
    """W_t = LSTM(W_{t-1}) for t >= 2: what is fed forward.  (a) The closed form of tests/golden/
    evolve_cell_gate_bias_only.txt (no products, a bias on the cell gate): C_t = tanh(beta)(1 - 2^-t) only if the cell
    state is carried from step to step and starts at 0.  (b) A library LSTM cell in double precision applied T times
    with the previous weight as input AND hidden state and the previous cell state: every W_t and C_t."""
    import os
    import torch
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "evolve_cell_gate_bias_only.txt")
    rows = [line.split() for line in open(path) if not line.startswith("#")]
    f, f2, beta = 3, 2, 0.5
    bias = np.zeros(4 * f2)
    bias[2 * f2:3 * f2] = beta                                   # gate order (input, forget, cell, output)
    rng = np.random.default_rng(5)
    ws, cs = oracle.evolve_weights(rng.normal(size=(f, f2)), np.zeros((f2, 4 * f2)), np.zeros((f2, 4 * f2)), bias, len(rows))
    assert len(ws) == len(rows) and len(cs) == len(rows) + 1 and not cs[0].any()
    for t_s, c_s, w_s in rows:
        t = int(t_s)
        np.testing.assert_allclose(cs[t], float(c_s), rtol=1e-14)
        np.testing.assert_allclose(ws[t - 1], float(w_s), rtol=1e-14)
        assert abs(float(c_s) - np.tanh(beta) * (1.0 - 2.0 ** -t)) < 1e-15
    # (b) general parameters against the library cell, four steps
    f, f2, T = 4, 3, 4
    w0 = rng.normal(size=(f, f2))
    u_x, u_h, b = rng.normal(size=(f2, 4 * f2)) / 2, rng.normal(size=(f2, 4 * f2)) / 2, rng.normal(size=4 * f2) / 3
    cell = torch.nn.LSTMCell(f2, f2).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(u_x.T))
        cell.weight_hh.copy_(torch.from_numpy(u_h.T))
        cell.bias_ih.copy_(torch.from_numpy(b))
        cell.bias_hh.zero_()
        w, c = torch.from_numpy(w0), torch.zeros((f, f2), dtype=torch.float64)
        want = []
        for _ in range(T):
            w, c = cell(w, (w, c))
            want.append((w.numpy().copy(), c.numpy().copy()))
    ws, cs = oracle.evolve_weights(w0, u_x, u_h, b, T)
    for t in range(T):
        np.testing.assert_allclose(ws[t], want[t][0], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(cs[t + 1], want[t][1], rtol=1e-12, atol=1e-13)


def test_edge_life_smoothing_matches_hand_worked_series():
    """The hand-worked series in tests/golden/edge_life_n3.txt: sliding-window sums by csr_combine, then the weighted
    form of Eqn (1) on S_3."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "edge_life_n3.txt")
    want = [np.array([[float(x) for x in row.split()] for row in line.split(";")])
            for line in open(path) if not line.startswith("#")]
    n, life = 3, 2
    off = [[(0, 1)], [(0, 1), (1, 2)], [(1, 2), (2, 0)], [(2, 0)]]
    snaps = []
    for edges in off:
        rows = [u for u, _ in edges] + list(range(n))
        cols = [v for _, v in edges] + list(range(n))
        snaps.append(oracle.csr_from_edges(n, np.array(rows), np.array(cols)))
    s = snaps[0] + (None,)
    got = [s]
    for t in range(2, 5):
        s = oracle.csr_combine(n, s, snaps[t - 1], 1.0, snaps[t - 1 - life] if t - life >= 1 else None, -1.0, diag=1.0)
        got.append(s)
    for t, (g, w) in enumerate(zip(got, want), start=1):
        val = np.ones(g[1].size) if g[2] is None else g[2]
        dense = np.nan_to_num(_dense_weighted(n, g[0], g[1], val), nan=0.0)
        assert np.array_equal(dense, w), f"S_{t}"
        assert g[1].size == np.count_nonzero(w)               # an edge that left the window is not stored
    s3 = got[2]
    norm = oracle.gcn_values_weighted(s3[0], s3[1], s3[2])
    np.testing.assert_allclose(norm, [1 / 2, 1 / np.sqrt(6), 1 / 3, 2 / np.sqrt(6), 1 / 2, 1 / 2], rtol=1e-15)


def test_summed_diagonal_is_the_m_transform_of_the_adjacency_tensor():
    """Without the diagonal rule the window sum of the stored A_i + I carries min(l, t) on its diagonal.  After Eqn (1)
    that is the M-transform variant of the section: (1/min(l,t)) sum of the A_i, plus I, normalised -- formed here
    densely from the raw edge sets."""
    n, life, T = 14, 3, 6
    rng = np.random.default_rng(12)
    raw = [(rng.random((n, n)) < 0.2) & ~np.eye(n, dtype=bool) for _ in range(T)]
    snaps = [oracle.csr_from_edges(n, *np.nonzero(a | np.eye(n, dtype=bool))) for a in raw]
    s = snaps[0] + (None,)
    for t in range(2, T + 1):
        s = oracle.csr_combine(n, s, snaps[t - 1], 1.0, snaps[t - 1 - life] if t - life >= 1 else None, -1.0)
        c = min(life, t)
        b = sum(a.astype(np.float64) for a in raw[max(0, t - life):t]) / c + np.eye(n)
        d = b.sum(axis=1) ** -0.5
        want = d[:, None] * b * d[None, :]
        got = np.nan_to_num(_dense_weighted(n, s[0], s[1], oracle.gcn_values_weighted(*s)), nan=0.0)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
        # and with the rule: the plain edge-life sum plus I
        e = oracle.csr_combine(n, s, None, 1.0, None, -1.0, diag=1.0)
        b1 = sum(a.astype(np.float64) for a in raw[max(0, t - life):t]) + np.eye(n)
        np.testing.assert_array_equal(np.nan_to_num(_dense_weighted(n, *e), nan=0.0), b1)


def test_transposed_snapshot_and_lists():
    """csr_transpose / coo_transpose against dense transposes, the involution, the identity <A^T g, h> = <g, A h> through
    the aggregation oracle, and the snapshot rule: transposing the lists and applying them to A^T gives (A')^T."""
    n = 23
    rng = np.random.default_rng(90)
    a = (rng.random((n, n)) < 0.2) | np.eye(n, dtype=bool)
    a[:, 5] = False; a[5, 5] = True                      # a column with one entry; row 7 below gets none at all
    rp, ci = oracle.csr_from_edges(n, *np.nonzero(a))
    val = rng.normal(size=ci.size)
    rp_t, ci_t, val_t = oracle.csr_transpose(n, rp, ci, val)
    want = _dense_weighted(n, rp, ci, val).T
    got = _dense_weighted(n, rp_t, ci_t, val_t)
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(np.nan_to_num(got), np.nan_to_num(want))
    assert all(np.all(np.diff(ci_t[rp_t[u]:rp_t[u + 1]]) > 0) for u in range(n))          # canonical: columns ascending
    back = oracle.csr_transpose(n, rp_t, ci_t, val_t)
    assert np.array_equal(back[0], rp) and np.array_equal(back[1], ci) and np.array_equal(back[2], val)
    # an empty row and an empty column survive
    b = a.copy(); b[7, :] = False; b[:, 9] = False
    rp_b, ci_b = oracle.csr_from_edges(n, *np.nonzero(b))
    rp_bt, ci_bt = oracle.csr_transpose(n, rp_b, ci_b)
    assert np.array_equal(_dense_unweighted(n, rp_bt, ci_bt), _dense_unweighted(n, rp_b, ci_b).T)
    # the adjoint identity through the plain aggregation
    g, h = rng.normal(size=(n, 3)), rng.normal(size=(n, 3))
    lhs = (oracle.spmm(rp_t, ci_t, g, val=val_t) * h).sum()
    rhs = (g * oracle.spmm(rp, ci, h, val=val)).sum()
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(rhs))
    # lists: pairs exchanged and sorted; applied to A^T they give the transpose of the next snapshot
    off = a & ~np.eye(n, dtype=bool)
    dr, dc = np.nonzero(off)
    pick = rng.choice(dr.size, 9, replace=False); pick.sort()
    absent = np.argwhere(~a)
    add = absent[rng.choice(len(absent), 11, replace=False)]
    add = add[np.lexsort((add[:, 1], add[:, 0]))]
    lists = (add[:, 0], add[:, 1], dr[pick], dc[pick])
    nxt = oracle.delta_apply(n, rp, ci, *lists)
    t_add, t_del = oracle.coo_transpose(lists[0], lists[1]), oracle.coo_transpose(lists[2], lists[3])
    assert all(np.all(np.diff(r.astype(np.int64) * n + c) > 0) for r, c in (t_add, t_del))
    nxt_t = oracle.delta_apply(n, rp_t, ci_t, *t_add, *t_del)
    want_t = oracle.csr_transpose(n, *nxt)
    assert np.array_equal(nxt_t[0], want_t[0]) and np.array_equal(nxt_t[1], want_t[1])
