"""Pins for the CPU oracle: each oracle function is checked against something that is not the
oracle -- hand-worked fixtures with their citation, dense brute force written here in numpy,
numpy set algebra, closed forms and invariants that follow from the paper's definitions
(Eqn (1), Eqn (2), the graph-difference reconstruction rule, the matrix M of the M-transform).
All CPU; no GPU code is touched."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from dtdg_synth import WORKLOADS, DynamicGraph, features, glorot_weight


# ----------------------------------------------------------------------------- helpers (numpy only)
def dense_from_csr(rowptr, colidx, n):
    a = np.zeros((n, n), dtype=bool)
    for u in range(n):
        a[u, colidx[rowptr[u]:rowptr[u + 1]]] = True
    return a


def csr_from_dense(a):
    n = a.shape[0]
    rowptr = np.zeros(n + 1, np.int32)
    cols = []
    for u in range(n):
        c = np.nonzero(a[u])[0]
        rowptr[u + 1] = rowptr[u] + c.size
        cols.append(c)
    return rowptr, (np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32))


def dense_gcn_matrix(a_plus_i):
    """Eqn (1) from its matrix form: D^{-1/2} (A+I) D^{-1/2}, D[u,u] = 1 + deg_u, with deg_u the
    number of off-diagonal entries of row u."""
    m = a_plus_i.astype(np.float64)
    deg = m.sum(axis=1) - np.diag(m)
    d = np.diag(1.0 / np.sqrt(1.0 + deg))
    return d @ m @ d


def coo(pairs):
    pairs = sorted(set(pairs))
    r = np.array([p[0] for p in pairs], np.int32)
    c = np.array([p[1] for p in pairs], np.int32)
    return r, c


def check_canonical(rowptr, colidx, n):
    assert rowptr[0] == 0 and rowptr[n] == colidx.size
    assert np.all(np.diff(rowptr) >= 1)                      # diagonal always present
    for u in range(n):
        row = colidx[rowptr[u]:rowptr[u + 1]]
        assert np.all(np.diff(row) > 0)                      # strictly ascending: sorted, no repeats
        assert u in row


def random_graph_dense(n, p, rng, symmetric):
    a = rng.random((n, n)) < p
    if symmetric:
        a = a | a.T
    np.fill_diagonal(a, True)
    return a


# ----------------------------------------------------------------------------- structure: rebuild
@pytest.mark.parametrize("symmetric", [True, False])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_delta_apply_matches_dense_boolean_brute_force(seed, symmetric):
    rng = np.random.default_rng(seed)
    n = 48
    a = random_graph_dense(n, 0.15, rng, symmetric)
    off = ~np.eye(n, dtype=bool)
    dels = a & off & (rng.random((n, n)) < 0.3)
    adds = (~a) & off & (rng.random((n, n)) < 0.1)
    expect = (a & ~dels) | adds                              # the reconstruction rule, on dense booleans
    rp, ci = csr_from_dense(a)
    ar, ac = np.nonzero(adds)
    dr, dc = np.nonzero(dels)
    rp2, ci2 = oracle.delta_apply(n, rp, ci, ar, ac, dr, dc)
    erp, eci = csr_from_dense(expect)
    assert np.array_equal(rp2, erp) and np.array_equal(ci2, eci)
    check_canonical(rp2, ci2, n)
    assert ci2.size == ci.size + ar.size - dr.size


def test_delta_apply_adversarial_tiny_cases():
    n = 6
    base = [(u, u) for u in range(n)] + [(0, 1), (0, 5), (1, 0), (2, 3), (2, 4), (2, 5), (5, 0), (5, 4)]
    rp, ci = oracle.csr_from_edges(n, *coo(base))
    cases = {
        "empty": ([], []),
        "first_row_only": ([(0, 2), (0, 3)], [(0, 1)]),
        "last_row_only": ([(5, 1)], [(5, 4), (5, 0)]),
        "row_emptied_to_diagonal": ([], [(2, 3), (2, 4), (2, 5)]),
        "delete_next_to_insert": ([(2, 1), (0, 4)], [(2, 3), (0, 5)]),
        "first_and_last_column": ([(3, 0), (3, 5), (4, 0), (1, 5)], [(5, 0), (0, 5)]),
        "every_row": ([(0, 2), (1, 2), (2, 0), (3, 1), (4, 1), (5, 3)], [(0, 1), (1, 0), (2, 3), (5, 4)]),
    }
    for name, (adds, dels) in cases.items():
        ar, ac = coo(adds) if adds else (np.zeros(0, np.int32),) * 2
        dr, dc = coo(dels) if dels else (np.zeros(0, np.int32),) * 2
        rp2, ci2 = oracle.delta_apply(n, rp, ci, ar, ac, dr, dc)
        expect = sorted((set(base) - set(dels)) | set(adds))            # python set algebra
        got = [(u, int(v)) for u in range(n) for v in ci2[rp2[u]:rp2[u + 1]]]
        assert got == expect, name
        if name == "empty":
            assert np.array_equal(rp2, rp) and np.array_equal(ci2, ci)


def test_delta_apply_equals_from_scratch_every_step_c1():
    """Delta-applied snapshot == snapshot rebuilt from scratch from the generator's edge set,
    == numpy set algebra on keys, at every timestep of the tiny workload."""
    wl = WORKLOADS["c1"]
    g = DynamicGraph(wl)
    rp, ci = oracle.csr_from_edges(wl.n, (g.keys >> 32).numpy(), (g.keys & 0xFFFFFFFF).numpy())
    grp, gci = g.csr()
    assert np.array_equal(rp, grp.numpy()) and np.array_equal(ci, gci.numpy())
    for t in range(2, wl.T + 1):
        prev_keys = g.keys.numpy().copy()
        ar, ac, dr, dc = (x.numpy() for x in g.advance())
        rp2, ci2 = oracle.delta_apply(wl.n, rp, ci, ar, ac, dr, dc)
        # from scratch, edges handed over in a shuffled order
        keys = g.keys.numpy()
        perm = np.random.default_rng(t).permutation(keys.size)
        rp3, ci3 = oracle.csr_from_edges(wl.n, (keys >> 32)[perm], (keys & 0xFFFFFFFF)[perm])
        assert np.array_equal(rp2, rp3) and np.array_equal(ci2, ci3)
        # numpy set algebra on 64-bit keys
        addk = (ar.astype(np.int64) << 32) | ac
        delk = (dr.astype(np.int64) << 32) | dc
        expect = np.union1d(np.setdiff1d(prev_keys, delk), addk)
        got = (np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(rp2)) << 32) | ci2
        assert np.array_equal(got, expect)
        assert ci2.size == ci.size + ar.size - dr.size
        check_canonical(rp2, ci2, wl.n)
        rp, ci = rp2, ci2


def test_delta_involution_and_composition():
    wl = WORKLOADS["c3"].scaled(1 << 10, T=4)
    g = DynamicGraph(wl)
    rp1, ci1 = (x.numpy() for x in g.csr())
    d2 = [x.numpy() for x in g.advance()]
    rp2, ci2 = oracle.delta_apply(wl.n, rp1, ci1, *d2)
    # involution: swapping the roles of the two difference lists goes back
    rpb, cib = oracle.delta_apply(wl.n, rp2, ci2, d2[2], d2[3], d2[0], d2[1])
    assert np.array_equal(rpb, rp1) and np.array_equal(cib, ci1)
    # composition: two steps == one step with the canonical difference of the end points
    d3 = [x.numpy() for x in g.advance()]
    rp3, ci3 = oracle.delta_apply(wl.n, rp2, ci2, *d3)
    k1 = (np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(rp1)) << 32) | ci1
    k3 = g.keys.numpy()
    addk, delk = np.setdiff1d(k3, k1), np.setdiff1d(k1, k3)
    rpc, cic = oracle.delta_apply(wl.n, rp1, ci1, addk >> 32, addk & 0xFFFFFFFF, delk >> 32, delk & 0xFFFFFFFF)
    assert np.array_equal(rpc, rp3) and np.array_equal(cic, ci3)


def test_csr_from_edges_handles_repeats_and_order():
    n = 5
    pairs = [(4, 4), (0, 0), (3, 1), (3, 1), (1, 1), (2, 2), (3, 3), (0, 4), (3, 0), (0, 4)]
    r = np.array([p[0] for p in pairs], np.int32)
    c = np.array([p[1] for p in pairs], np.int32)
    rp, ci = oracle.csr_from_edges(n, r, c)
    assert rp.tolist() == [0, 2, 3, 4, 7, 8]
    assert ci.tolist() == [0, 4, 1, 2, 0, 1, 3, 4]


# ----------------------------------------------------------------------------- values of A~
def test_gcn_values_match_hand_worked_path(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "gcn_path3.txt")) if not l.startswith("#")]
    expect = np.array([[0.0 if x == "0" else 1.0 / np.sqrt(int(x)) for x in r] for r in rows])
    edges = [(0, 0), (1, 1), (2, 2), (0, 1), (1, 0), (1, 2), (2, 1)]
    rp, ci = oracle.csr_from_edges(3, *coo(edges))
    val = oracle.gcn_values(rp, ci)
    dense = np.zeros((3, 3))
    for u in range(3):
        for e in range(rp[u], rp[u + 1]):
            dense[u, ci[e]] = val[e]
    assert np.allclose(dense, expect, rtol=1e-15, atol=0)


@pytest.mark.parametrize("symmetric", [True, False])
def test_gcn_values_match_dense_matrix_form(symmetric):
    rng = np.random.default_rng(7)
    n = 40
    a = random_graph_dense(n, 0.2, rng, symmetric)
    rp, ci = csr_from_dense(a)
    val = oracle.gcn_values(rp, ci)
    dense = dense_gcn_matrix(a)
    got = np.zeros((n, n))
    for u in range(n):
        for e in range(rp[u], rp[u + 1]):
            got[u, ci[e]] = val[e]
    assert np.allclose(got, dense, rtol=1e-14, atol=0)
    if symmetric:
        assert np.allclose(got, got.T, rtol=0, atol=0)
        assert np.linalg.norm(got, 2) <= 1 + 1e-12


# ----------------------------------------------------------------------------- X W
def test_xw_matches_numpy_rectangular():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((37, 5))
    w = rng.standard_normal((5, 9))                           # rectangular: a transposed operand cannot pass
    assert np.allclose(oracle.xw(x, w), x @ w, rtol=1e-13, atol=1e-13)
    assert np.array_equal(oracle.xw(x, np.eye(5)), x)
    assert np.array_equal(oracle.xw(x, np.zeros((5, 3))), np.zeros((37, 3)))
    x2 = rng.standard_normal((37, 5))
    assert np.allclose(oracle.xw(2 * x + x2, w), 2 * oracle.xw(x, w) + oracle.xw(x2, w), rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- A~ H
@pytest.mark.parametrize("symmetric", [True, False])
@pytest.mark.parametrize("relu", [False, True])
def test_spmm_matches_dense_brute_force(symmetric, relu):
    rng = np.random.default_rng(11)
    n, f = 64, 7
    a = random_graph_dense(n, 0.12, rng, symmetric)
    rp, ci = csr_from_dense(a)
    h = rng.standard_normal((n, f))
    expect = dense_gcn_matrix(a) @ h
    if relu:
        expect = np.maximum(expect, 0.0)
    got = oracle.spmm(rp, ci, h, relu=relu)
    assert np.allclose(got, expect, rtol=1e-13, atol=1e-14)
    rows = np.array([5, 63, 0, 17], np.int64)
    assert np.array_equal(oracle.spmm(rp, ci, h, relu=relu, rows=rows), got[rows])


def test_spmm_c1_whole_layer_vs_dense():
    wl = WORKLOADS["c1"]
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    a = dense_from_csr(rp, ci, wl.n)
    x = features(wl, 1).double().numpy()
    w = glorot_weight(wl, 0).double().numpy()
    expect = np.maximum(dense_gcn_matrix(a) @ (x @ w), 0.0)
    got = oracle.gcn_layer(rp, ci, x, w, relu=True)
    assert np.allclose(got, expect, rtol=1e-12, atol=1e-13)


def test_spmm_sqrt_degree_is_fixed_vector():
    """x_u = sqrt(1+deg_u) is mapped to itself by A~ for any graph, directed or not: row u has
    1+deg_u entries, each contributing sqrt(1+deg_v) / sqrt((1+deg_u)(1+deg_v))."""
    wl = WORKLOADS["c3"].scaled(1 << 11)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    d = np.diff(rp).astype(np.float64)
    x = np.sqrt(d)[:, None] * np.array([[1.0, -2.0, 0.5]])
    got = oracle.spmm(rp, ci, x)
    assert np.allclose(got, x, rtol=1e-12, atol=0)


def test_spmm_special_graphs():
    rng = np.random.default_rng(5)
    n, f = 12, 4
    h = rng.standard_normal((n, f))
    # no edges: A~ = I
    rp, ci = csr_from_dense(np.eye(n, dtype=bool))
    assert np.array_equal(oracle.spmm(rp, ci, h), h)
    # complete graph: A~ = J/n, every output row is the column mean
    rp, ci = csr_from_dense(np.ones((n, n), dtype=bool))
    assert np.allclose(oracle.spmm(rp, ci, h), np.tile(h.mean(axis=0), (n, 1)), rtol=1e-13, atol=1e-15)
    # cycle: three-point moving average
    a = np.eye(n, dtype=bool)
    for u in range(n):
        a[u, (u + 1) % n] = a[u, (u - 1) % n] = True
    rp, ci = csr_from_dense(a)
    expect = (h + np.roll(h, 1, axis=0) + np.roll(h, -1, axis=0)) / 3.0
    assert np.allclose(oracle.spmm(rp, ci, h), expect, rtol=1e-13, atol=1e-15)


# ----------------------------------------------------------------------------- M-transform
@pytest.mark.parametrize("name,T,w", [("m_matrix_T3_w2.txt", 3, 2), ("m_matrix_T5_w3.txt", 5, 3)])
def test_m_matrix_matches_hand_worked(golden_dir, name, T, w):
    rows = [l.split() for l in open(os.path.join(golden_dir, name)) if not l.startswith("#")]
    expect = np.array([[float(Fraction(x)) for x in r] for r in rows])
    assert np.allclose(oracle.m_matrix(T, w), expect, rtol=1e-16, atol=0)


@pytest.mark.parametrize("T,w", [(8, 3), (32, 8), (128, 16), (5, 1), (6, 9)])
def test_m_matrix_structure(T, w):
    M = oracle.m_matrix(T, w)
    assert np.allclose(M.sum(axis=1), 1.0, rtol=1e-14)          # averaging: rows sum to one
    assert np.array_equal(M, np.tril(M))                         # lower triangular
    assert np.array_equal(np.triu(M, 0) * 0 + (np.tril(M, -w) != 0), np.zeros_like(M, dtype=bool))  # band of width w
    for t in range(T):
        assert np.count_nonzero(M[t]) == min(w, t + 1)


def test_mproduct_closed_forms():
    rng = np.random.default_rng(9)
    T, n, f = 9, 6, 3
    z = rng.standard_normal((T, n, f))
    # explicit tensor-times-matrix by einsum with an asymmetric M: catches a transposed M
    M = np.tril(rng.standard_normal((T, T)))
    assert np.allclose(oracle.mproduct(z, M), np.einsum("tk,knf->tnf", M, z), rtol=1e-13, atol=1e-13)
    # w = 1 is the identity
    assert np.array_equal(oracle.mproduct(z, oracle.m_matrix(T, 1)), z)
    # w >= T is the running mean
    run = np.cumsum(z, axis=0) / np.arange(1, T + 1)[:, None, None]
    assert np.allclose(oracle.mproduct(z, oracle.m_matrix(T, T + 3)), run, rtol=1e-13, atol=1e-14)
    # constant-in-time input is a fixed point
    c = np.tile(z[:1], (T, 1, 1))
    assert np.allclose(oracle.mproduct(c, oracle.m_matrix(T, 4)), c, rtol=1e-14, atol=0)
    # impulse at k0: 1/min(w,t) for k0 <= t <= k0+w-1, zero elsewhere (1-based)
    w, k0 = 3, 4
    imp = np.zeros((T, 1, 1))
    imp[k0 - 1] = 1.0
    y = oracle.mproduct(imp, oracle.m_matrix(T, w))[:, 0, 0]
    expect = np.array([1.0 / min(w, t) if k0 <= t <= k0 + w - 1 else 0.0 for t in range(1, T + 1)])
    assert np.allclose(y, expect, rtol=1e-15, atol=0)
    # commutes with a feature transform applied to every frame
    wmat = rng.standard_normal((f, f))
    Mw = oracle.m_matrix(T, 4)
    lhs = np.stack([oracle.xw(fr, wmat) for fr in oracle.mproduct(z, Mw)])
    rhs = oracle.mproduct(np.stack([oracle.xw(fr, wmat) for fr in z]), Mw)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- whole tiny pipeline
def test_c1_end_to_end_vs_dense_brute_force():
    """One GCN layer with ReLU on every snapshot (snapshots obtained by applying differences),
    then the M-transform with window 3, against dense numpy on from-scratch snapshots."""
    wl = WORKLOADS["c1"]
    g = DynamicGraph(wl)
    w = glorot_weight(wl, 0).double().numpy()
    rp, ci = (x.numpy() for x in g.csr())
    zs, dense_zs = [], []
    for t in range(1, wl.T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        x = features(wl, t).double().numpy()
        zs.append(oracle.gcn_layer(rp, ci, x, w, relu=True))
        keys = g.keys.numpy()
        a = np.zeros((wl.n, wl.n), dtype=bool)
        a[keys >> 32, keys & 0xFFFFFFFF] = True
        dense_zs.append(np.maximum(dense_gcn_matrix(a) @ x @ w, 0.0))
    y = oracle.mproduct(np.stack(zs), oracle.m_matrix(wl.T, wl.window))
    dz = np.stack(dense_zs)
    expect = np.zeros_like(dz)
    for t in range(1, wl.T + 1):
        lo = max(1, t - wl.window + 1)
        expect[t - 1] = dz[lo - 1:t].sum(axis=0) / min(wl.window, t)
    assert np.allclose(y, expect, rtol=1e-11, atol=1e-12)


# ----------------------------------------------------------------------------- the generator's promises
@pytest.mark.parametrize("name,n", [("c1", 1000), ("c2", 4096), ("c3", 1 << 12), ("c4", 5000), ("c5", 1 << 12)])
def test_generator_emits_canonical_differences(name, n):
    wl = WORKLOADS[name].scaled(n, T=4) if n != WORKLOADS[name].n else WORKLOADS[name]
    g = DynamicGraph(wl)
    for _ in range(3):
        prev = g.keys.numpy().copy()
        ar, ac, dr, dc = (x.numpy().astype(np.int64) for x in g.advance())
        addk, delk = (ar << 32) | ac, (dr << 32) | dc
        assert np.all(np.diff(addk) > 0) and np.all(np.diff(delk) > 0)         # sorted, unique
        assert np.all(np.isin(delk, prev)) and not np.any(np.isin(addk, prev))  # deleted present, added absent
        assert not np.any(ar == ac) and not np.any(dr == dc)                    # diagonal untouched
        assert np.array_equal(g.keys.numpy(), np.union1d(np.setdiff1d(prev, delk), addk))
        if wl.graph == "er":                                                     # undirected: both directions
            assert np.array_equal(np.sort((ac << 32) | ar), addk)
            assert np.array_equal(np.sort((dc << 32) | dr), delk)


def test_generator_is_deterministic_and_seeded():
    wl = WORKLOADS["c3"].scaled(1 << 10, T=3)
    a, b = DynamicGraph(wl), DynamicGraph(wl)
    assert torch.equal(a.keys, b.keys)
    assert all(torch.equal(x, y) for x, y in zip(a.advance(), b.advance()))
    from dataclasses import replace
    c = DynamicGraph(replace(wl, seed=wl.seed + 1))
    assert not torch.equal(a.keys[: c.keys.numel()], c.keys[: a.keys.numel()])
    assert torch.equal(features(wl, 2), features(wl, 2))
    assert not torch.equal(features(wl, 2), features(wl, 3))
