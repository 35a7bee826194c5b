"""GPU parity of the entry points for snapshots that carry a value per stored entry (Section "Graph-difference
Based Input Transfer": the values of the new snapshot travel with the index lists) against the CPU oracle:
structure and carried values bit for bit, aggregation within the floating-point bound."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph
from helpers import assert_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dtype):
    return torch.as_tensor(np.ascontiguousarray(a), dtype=dtype).to(DEV)


def gpu_rebuild_weighted(n, rp, ci, val, add, dele, upd, merged=False, expect_status=0):
    """add/dele as numpy tuples sorted by (row, col), upd in any order; returns numpy (rowptr, colidx, val).
    merged: the update list is sorted here and handed over as sorted, so that the streaming merge consumes it."""
    nnz_prev = int(ci.size)
    n_add, n_del = int(add[0].size), int(dele[0].size)
    cap = nnz_prev + n_add - n_del + 5
    rpn = torch.full((n + 1,), -7, dtype=torch.int32, device=DEV)
    cin = torch.full((cap,), -7, dtype=torch.int32, device=DEV)
    vn = torch.full((cap,), float("nan"), dtype=torch.float32, device=DEV)
    flags = dg.DGNN_VALIDATE
    if merged:
        if expect_status == 0:
            order = np.lexsort((upd[1], upd[0]))
            upd = tuple(x[order] for x in upd)
        flags |= dg.DGNN_UPDATES_SORTED
    ws = torch.empty(dg.delta_rebuild_workspace(n, nnz_prev, n_add, n_del), dtype=torch.uint8, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    nnz = dg.delta_rebuild_weighted(
        dev(rp, torch.int32), dev(ci, torch.int32), dev(val, torch.float32), nnz_prev,
        (dev(add[0], torch.int32), dev(add[1], torch.int32), dev(add[2], torch.float32)) if n_add else None,
        (dev(dele[0], torch.int32), dev(dele[1], torch.int32)) if n_del else None,
        (dev(upd[0], torch.int32), dev(upd[1], torch.int32), dev(upd[2], torch.float32)) if upd[0].size else None,
        rpn, cin, vn, ws, flags=flags, d_status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == expect_status
    assert torch.isnan(vn[nnz:]).all() and (cin[nnz:] == -7).all()      # nothing written beyond the result
    return rpn.cpu().numpy(), cin.cpu().numpy()[:nnz], vn.cpu().numpy()[:nnz]


def f32(x):
    return np.asarray(x, dtype=np.float32)


def step_lists(wl_graph, rng, upd_frac):
    """One step of the generator's structure plus seeded values: returns (add, dele, upd) for the current snapshot."""
    keys_before = wl_graph.keys.clone()
    ar, ac, dr, dc = (x.numpy() for x in wl_graph.advance())
    kb = keys_before.numpy()
    deleted = (dr.astype(np.int64) << 32) | dc.astype(np.int64)
    surv = kb[~np.isin(kb, deleted)]
    surv = surv[(surv >> 32) != (surv & 0xffffffff)]
    pick = rng.permutation(surv.size)[: int(upd_frac * surv.size)]
    ur, uc = (surv[pick] >> 32).astype(np.int32), (surv[pick] & 0xffffffff).astype(np.int32)
    return ((ar, ac, f32(rng.uniform(1, 2, ar.size))), (dr, dc), (ur, uc, f32(rng.uniform(3, 4, ur.size))))


@pytest.mark.parametrize("merged", [False, True])
@pytest.mark.parametrize("name,n,upd_frac", [("c1", 1000, 0.1), ("c3", 1 << 14, 0.05), ("c3", 1 << 14, 0.0), ("c2", 30_000, 0.3),
                                             ("c3", 1 << 14, 0.7), ("c2", 30_000, 1.0)])
def test_weighted_rebuild_chain(name, n, upd_frac, merged):
    wl = WORKLOADS[name].scaled(n, T=5) if n != WORKLOADS[name].n else WORKLOADS[name]
    g = DynamicGraph(wl)
    rng = np.random.default_rng(n)
    rp, ci = (x.numpy() for x in g.csr())
    val = f32(rng.uniform(0.1, 1.0, ci.size))
    for t in range(2, 6):
        add, dele, upd = step_lists(g, rng, upd_frac)
        want = oracle.delta_apply_weighted(wl.n, rp, ci, val, add=add, dele=dele, upd=upd)
        got = gpu_rebuild_weighted(wl.n, rp, ci, val, add, dele, upd, merged=merged)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), (name, t)
        assert np.array_equal(got[2], f32(want[2])), (name, t)                 # values are carried, not computed
        rp, ci, val = got


def test_weighted_rebuild_hub_rows_and_absent_updates():
    """Rows longer than a range of the merge (its wavefronts then begin in the middle of a row and have to find their
    place in the row's updates), with updates that name edges which are not stored (before, between and after a
    row's entries) or which the same step deletes: they change nothing."""
    n = 4096
    rng = np.random.default_rng(77)
    rows, cols = [np.arange(n)], [np.arange(n)]
    for hub, deg in ((5, 3000), (6, 1200), (4000, 4000)):
        rows.append(np.full(deg, hub)); cols.append(rng.choice(n, deg, replace=False))
    rows.append(rng.integers(0, n, 20000)); cols.append(rng.integers(0, n, 20000))
    rp, ci = oracle.csr_from_edges(n, np.concatenate(rows).astype(np.int32), np.concatenate(cols).astype(np.int32))
    val = f32(rng.uniform(0.1, 1.0, ci.size))
    r_of = np.repeat(np.arange(n, dtype=np.int32), np.diff(rp))
    off = np.flatnonzero(r_of != ci)
    dele_pos = np.sort(rng.choice(off, off.size // 10, replace=False))
    dele = (r_of[dele_pos], ci[dele_pos])
    stored = set(zip(r_of.tolist(), ci.tolist()))
    add_pairs = sorted({(int(r), int(c)) for r, c in zip(rng.choice([5, 6, 4000, 17, 99], 3000), rng.integers(0, n, 3000))
                        if (int(r), int(c)) not in stored and r != c})
    add = (np.array([p[0] for p in add_pairs], np.int32), np.array([p[1] for p in add_pairs], np.int32), f32(rng.uniform(1, 2, len(add_pairs))))
    # updates: 40 % of the stored entries (the deleted ones among them), and as many pairs drawn blindly
    some = rng.choice(ci.size, int(0.4 * ci.size), replace=False)
    blind_r = np.concatenate([rng.integers(0, n, 5000), np.full(5000, 5), np.full(5000, 4000)]).astype(np.int32)
    blind_c = rng.integers(0, n, blind_r.size).astype(np.int32)
    pairs = np.unique(np.concatenate([(r_of[some].astype(np.int64) << 32) | ci[some], (blind_r.astype(np.int64) << 32) | blind_c]))
    added = (add[0].astype(np.int64) << 32) | add[1]
    pairs = rng.permutation(pairs[~np.isin(pairs, added)])
    upd = ((pairs >> 32).astype(np.int32), (pairs & 0xffffffff).astype(np.int32), f32(rng.uniform(3, 4, pairs.size)))
    want = oracle.delta_apply_weighted(n, rp, ci, val, add=add, dele=dele, upd=upd)
    for merged in (False, True):
        got = gpu_rebuild_weighted(n, rp, ci, val, add, dele, upd, merged=merged)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), merged
        assert np.array_equal(got[2], f32(want[2])), merged


def test_weighted_rebuild_reports_an_unsorted_update_list():
    """Declared sorted, but not: the check says so, and nothing is written outside the result."""
    wl = WORKLOADS["c1"]
    g = DynamicGraph(wl)
    rng = np.random.default_rng(5)
    rp, ci = (x.numpy() for x in g.csr())
    val = f32(rng.uniform(0.1, 1.0, ci.size))
    add, dele, upd = step_lists(g, rng, 0.3)
    order = np.lexsort((upd[1], upd[0]))[::-1]
    upd = tuple(np.ascontiguousarray(x[order]) for x in upd)
    want = oracle.delta_apply_weighted(wl.n, rp, ci, val, add=add, dele=dele, upd=upd)
    got = gpu_rebuild_weighted(wl.n, rp, ci, val, add, dele, upd, merged=True, expect_status=2)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])      # the structure does not depend on the updates


def test_weighted_rebuild_edge_cases():
    n = 6
    base = [(u, u) for u in range(n)] + [(0, 1), (0, 5), (1, 0), (2, 3), (2, 4), (2, 5), (5, 0), (5, 4)]
    rows = np.array([p[0] for p in sorted(base)], np.int32)
    cols = np.array([p[1] for p in sorted(base)], np.int32)
    rp, ci = oracle.csr_from_edges(n, rows, cols)
    val = f32(np.arange(1, ci.size + 1))
    e_i, e_f = np.zeros(0, np.int32), np.zeros(0, np.float32)
    cases = {
        "nothing": ((e_i, e_i, e_f), (e_i, e_i), (e_i, e_i, e_f)),
        "only_updates_incl_diagonal": ((e_i, e_i, e_f), (e_i, e_i), (np.array([0, 3, 5], np.int32), np.array([5, 3, 0], np.int32), f32([9, 8, 7]))),
        "update_of_absent_edge_is_skipped": ((e_i, e_i, e_f), (e_i, e_i), (np.array([4], np.int32), np.array([0], np.int32), f32([5]))),
        "all_three": ((np.array([0, 3], np.int32), np.array([2, 0], np.int32), f32([20, 30])),
                      (np.array([2, 5], np.int32), np.array([4, 4], np.int32)),
                      (np.array([2], np.int32), np.array([3], np.int32), f32([40]))),
    }
    for name, (add, dele, upd) in cases.items():
        want = oracle.delta_apply_weighted(n, rp, ci, val, add=add, dele=dele, upd=upd)
        for merged in (False, True):
            got = gpu_rebuild_weighted(n, rp, ci, val, add, dele, upd, merged=merged)
            assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), (name, merged)
            assert np.array_equal(got[2], f32(want[2])), (name, merged)


@pytest.mark.parametrize("dtype,f", [(torch.float32, 16), (torch.float32, 32), (torch.float32, 128), (torch.bfloat16, 64),
                                     (torch.bfloat16, 128)])
@pytest.mark.parametrize("relu", [False, True])
def test_weighted_spmm(dtype, f, relu):
    wl = WORKLOADS["c3"].scaled(1 << 13, T=1)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    n = wl.n
    rng = np.random.default_rng(f)
    val = f32(rng.standard_normal(ci.size))
    h = torch.randn((n, f), generator=torch.Generator().manual_seed(f)).to(dtype)
    want = oracle.spmm(rp, ci, to_f64(h), relu=relu, val=val.astype(np.float64))
    ws = torch.empty(dg.spmm_workspace(n, int(ci.size), f), dtype=torch.uint8, device=DEV)
    z = torch.full((n, f), float("nan"), dtype=dtype, device=DEV)
    dg.spmm_weighted(dev(rp, torch.int32), dev(ci, torch.int32), dev(val, torch.float32), int(ci.size), h.to(DEV), z, ws,
                     flags=dg.DGNN_RELU if relu else 0)
    assert_close(to_f64(z), want, dtype, f"weighted spmm f={f}")
    # the paper's way of bringing the values: the normalised values of Eqn (1) shipped whole give the GCN aggregation
    if not relu:
        vals_eq1 = oracle.gcn_values(rp, ci)
        dg.spmm_weighted(dev(rp, torch.int32), dev(ci, torch.int32), dev(f32(vals_eq1), torch.float32), int(ci.size),
                         h.to(DEV), z, ws)
        assert_close(to_f64(z), oracle.spmm(rp, ci, to_f64(h)), dtype, "Eqn (1) values shipped whole")


@pytest.mark.parametrize("merged", [False, True])
@pytest.mark.parametrize("name,n,life,mode", [("c1", 1000, 3, "edge_life"), ("c3", 1 << 13, 4, "edge_life"),
                                              ("c3", 1 << 13, 3, "mproduct"), ("c2", 20_000, 2, "mproduct")])
def test_smoothed_series_through_the_weighted_path(name, n, life, mode, merged):
    """The smoothed graphs the paper's models are trained on (sum of the raw snapshots of the last `life`
    timesteps), carried from step to step by weighted differences.  The expected snapshots are built here from
    the raw oracle snapshots with numpy, not from the lists."""
    from dtdg_synth import SmoothedGraph
    wl = WORKLOADS[name].scaled(n, T=7) if n != WORKLOADS[name].n else WORKLOADS[name]
    raw = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in raw.csr())
    raw_keys = [(np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(rp)) << 32) | ci.astype(np.int64)]
    sm = SmoothedGraph(wl, life, mode)
    g_rp, g_ci, g_val = (x.numpy() for x in sm.csr())
    f = 32
    h = torch.randn((wl.n, f), generator=torch.Generator().manual_seed(3))
    for t in range(2, 8):
        rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in raw.advance()])
        raw_keys.append((np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(rp)) << 32) | ci.astype(np.int64))
        window = raw_keys[max(0, t - life):t]
        keys, counts = np.unique(np.concatenate(window), return_counts=True)
        want_val = f32(counts) / (np.float32(min(life, t)) if mode == "mproduct" else np.float32(1))
        add, dele, upd = sm.advance()
        add, dele, upd = tuple(x.numpy() for x in add), tuple(x.numpy() for x in dele), tuple(x.numpy() for x in upd)
        g_rp, g_ci, g_val = gpu_rebuild_weighted(wl.n, g_rp, g_ci, g_val, add, dele, upd, merged=merged)
        got_keys = (np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(g_rp)) << 32) | g_ci.astype(np.int64)
        assert np.array_equal(got_keys, keys), (name, t)
        assert np.array_equal(g_val, want_val), (name, t)
    # aggregation with the smoothed values of the last snapshot
    want = oracle.spmm(g_rp, g_ci, to_f64(h), relu=True, val=g_val.astype(np.float64))
    ws = torch.empty(dg.spmm_workspace(wl.n, int(g_ci.size), f), dtype=torch.uint8, device=DEV)
    z = torch.empty((wl.n, f), device=DEV)
    dg.spmm_weighted(dev(g_rp, torch.int32), dev(g_ci, torch.int32), dev(g_val, torch.float32), int(g_ci.size), h.to(DEV), z,
                     ws, flags=dg.DGNN_RELU)
    assert_close(to_f64(z), want, torch.float32, f"aggregation over the smoothed snapshot ({mode})")
    # and normalised as in Eqn (1), from the same carried values: nothing but the count changes travelled
    want = oracle.spmm(g_rp, g_ci, to_f64(h), relu=True, val=oracle.gcn_values_weighted(g_rp, g_ci, g_val.astype(np.float64)))
    rp_d, val_d = dev(g_rp, torch.int32), dev(g_val, torch.float32)
    dinv = torch.empty(wl.n, device=DEV)
    dg.csr_weighted_dinv(rp_d, val_d, int(g_ci.size), dinv, ws_dinv(int(g_ci.size)))
    hs = torch.empty((wl.n, f), device=DEV)
    dg.feature_transform(h.to(DEV), torch.eye(f, device=DEV), hs, row_scale=dinv)
    dg.spmm_weighted(rp_d, dev(g_ci, torch.int32), val_d, int(g_ci.size), hs, z, ws,
                     flags=dg.DGNN_RELU | dg.DGNN_H_PRESCALED, dinv=dinv)
    assert_close(to_f64(z), want, torch.float32, f"normalised aggregation over the smoothed snapshot ({mode})")


@pytest.mark.parametrize("dtype,f", [(torch.float32, 32), (torch.bfloat16, 128)])
def test_normalised_weighted_aggregation_recomputed_on_the_gpu(dtype, f):
    """D^(-1/2) V D^(-1/2) H from the raw values: weighted row sums -> dinv, rows of H pre-scaled by the dense
    transform, aggregation with the raw values; against the oracle's explicit normalised values."""
    wl = WORKLOADS["c3"].scaled(1 << 13, T=1)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    n = wl.n
    rng = np.random.default_rng(f)
    val = f32(rng.integers(1, 5, ci.size))                                  # counts, as a smoothed snapshot has
    x = torch.randn((n, f), generator=torch.Generator().manual_seed(f)).to(dtype)
    w = (torch.randn((f, f), generator=torch.Generator().manual_seed(f + 1)) / np.sqrt(f)).to(dtype)
    want = oracle.spmm(rp, ci, oracle.xw(to_f64(x), to_f64(w)), relu=True,
                       val=oracle.gcn_values_weighted(rp, ci, val.astype(np.float64)))
    rp_d, ci_d, val_d = dev(rp, torch.int32), dev(ci, torch.int32), dev(val, torch.float32)
    dinv = torch.empty(n, device=DEV)
    dg.csr_weighted_dinv(rp_d, val_d, int(ci.size), dinv, ws_dinv(int(ci.size)))
    d = np.array([val[rp[u]:rp[u + 1]].astype(np.float64).sum() for u in range(n)])
    np.testing.assert_allclose(to_f64(dinv), d ** -0.5, rtol=2e-6)
    h = torch.empty((n, f), dtype=dtype, device=DEV)
    dg.feature_transform(x.to(DEV), w.to(DEV), h, row_scale=dinv)
    z = torch.empty((n, f), dtype=dtype, device=DEV)
    ws = torch.empty(dg.spmm_workspace(n, int(ci.size), f), dtype=torch.uint8, device=DEV)
    dg.spmm_weighted(rp_d, ci_d, val_d, int(ci.size), h, z, ws, flags=dg.DGNN_RELU | dg.DGNN_H_PRESCALED, dinv=dinv)
    assert_close(to_f64(z), want, dtype, "normalised weighted aggregation")


def ws_dinv(nnz):
    return torch.empty(dg.csr_weighted_dinv_workspace(nnz), dtype=torch.uint8, device=DEV)


def test_weighted_row_sums_with_hub_rows_cut_into_pieces():
    """Row lengths around the piece length: rows that begin exactly on a piece boundary, end on one, span
    several pieces, follow each other directly, with empty rows between; against fp64 sums.  Twice: the
    result must repeat bit for bit."""
    piece = 4096
    lens = [5, 0, 20000, 3, piece, piece + 1, 0, 0, 40000, 64, 65, 1, 3 * piece, 7, 2 * piece + 1, 128, 129, 100000,
            piece - 1, 1, piece, 0, 2 * piece - 3, 3]
    pad = (-sum(lens[:2])) % piece                      # make the third row begin exactly on a piece boundary
    lens = lens[:1] + [pad + lens[1]] + lens[2:] + [3] * 150 + [9000] + [1] * 37 + [0] * 70
    rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    assert rp[2] % piece == 0
    nnz = int(rp[-1])
    rng = np.random.default_rng(5)
    val = f32(rng.uniform(0.5, 2.0, nnz))
    want = np.array([val[rp[u]:rp[u + 1]].astype(np.float64).sum() for u in range(len(lens))])
    rp_d, val_d = dev(rp, torch.int32), dev(val, torch.float32)
    outs = []
    for _ in range(2):
        dinv = torch.full((len(lens),), float("nan"), device=DEV)
        ws = ws_dinv(nnz)
        ws.fill_(0xff)
        dg.csr_weighted_dinv(rp_d, val_d, nnz, dinv, ws)
        outs.append(dinv.cpu())
    assert torch.equal(outs[0], outs[1])
    got = to_f64(outs[0])
    nz = want > 0
    np.testing.assert_allclose(got[nz], want[nz] ** -0.5, rtol=2e-6)
    assert np.all(got[~nz] == 0.0)                      # an empty row has no normalisation: factor 0


def test_normalised_aggregation_with_vertices_without_entries():
    """Rows without stored entries that other rows point to: their factor is 0 on both sides, nothing turns into
    inf or NaN, and the rest of the result is unaffected."""
    wl = WORKLOADS["c3"].scaled(1 << 12, T=1)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    n, f = wl.n, 32
    rng = np.random.default_rng(8)
    lens = np.diff(rp)
    drop = rng.choice(n, size=n // 10, replace=False)                     # a tenth of the rows lose all their entries
    keep = np.ones(ci.size, dtype=bool)
    for u in drop:
        keep[rp[u]:rp[u + 1]] = False
    lens[drop] = 0
    rp, ci = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), ci[keep]
    assert np.isin(ci, drop).any()                                        # emptied vertices are still pointed to
    val = f32(rng.integers(1, 4, ci.size))
    x = torch.randn((n, f), generator=torch.Generator().manual_seed(2))
    w = torch.randn((f, f), generator=torch.Generator().manual_seed(3)) / np.sqrt(f)
    want = oracle.spmm(rp, ci, oracle.xw(to_f64(x), to_f64(w)), relu=False, val=oracle.gcn_values_weighted(rp, ci, val.astype(np.float64)))
    assert np.isfinite(want).all() and np.all(want[drop] == 0.0)
    rp_d, ci_d, val_d = dev(rp, torch.int32), dev(ci, torch.int32), dev(val, torch.float32)
    dinv = torch.empty(n, device=DEV)
    dg.csr_weighted_dinv(rp_d, val_d, int(ci.size), dinv, ws_dinv(int(ci.size)))
    h = torch.empty((n, f), device=DEV)
    dg.feature_transform(x.to(DEV), w.to(DEV), h, row_scale=dinv)
    z = torch.full((n, f), float("nan"), device=DEV)
    ws = torch.empty(dg.spmm_workspace(n, int(ci.size), f), dtype=torch.uint8, device=DEV)
    dg.spmm_weighted(rp_d, ci_d, val_d, int(ci.size), h, z, ws, flags=dg.DGNN_H_PRESCALED, dinv=dinv)
    assert bool(torch.isfinite(z).all())
    assert_close(to_f64(z), want, torch.float32, "normalised aggregation with empty rows")
