"""GPU parity, kernel by kernel: every entry point of the C boundary against the CPU oracle on the
same seeded inputs, element by element, at sizes that span several tiles and a ragged tail."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph
from helpers import assert_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev_i32(a):
    return torch.as_tensor(np.ascontiguousarray(a), dtype=torch.int32).to(DEV)


def gpu_rebuild(n, rp, ci, ar, ac, dr, dc, validate=True, slack=0, shift=0):
    """shift: the row-pointer arrays and dinv begin `shift` elements into their allocations (1: not 16-byte aligned)."""
    ci_d = dev_i32(ci)
    rp_d = torch.empty(n + 1 + shift, dtype=torch.int32, device=DEV)[shift:]
    rp_d.copy_(torch.as_tensor(rp))
    lists = [dev_i32(x) for x in (ar, ac, dr, dc)]
    nnz_prev, n_add, n_del = int(ci.size), int(ar.size), int(dr.size)
    cap = nnz_prev + n_add - n_del + slack
    rpn = torch.full((n + 1 + shift,), -7, dtype=torch.int32, device=DEV)[shift:]
    cin = torch.full((max(cap, 1),), -7, dtype=torch.int32, device=DEV)
    dinv = torch.zeros(n + shift, dtype=torch.float32, device=DEV)[shift:]
    ws = torch.empty(dg.delta_rebuild_workspace(n, nnz_prev, n_add, n_del), dtype=torch.uint8, device=DEV)
    status = torch.full((1,), 99, dtype=torch.int32, device=DEV)
    nnz = dg.delta_rebuild(rp_d, ci_d, nnz_prev, lists[0], lists[1], n_add, lists[2], lists[3], n_del, rpn, cin, dinv,
                           ws, flags=dg.DGNN_VALIDATE if validate else 0, d_status=status)
    torch.cuda.synchronize()
    return rpn.cpu().numpy(), cin.cpu().numpy()[:nnz], dinv.cpu().numpy(), int(status.item()), cin.cpu().numpy()[nnz:]


def coo(pairs):
    pairs = sorted(set(pairs))
    return (np.array([p[0] for p in pairs], np.int32), np.array([p[1] for p in pairs], np.int32))


EMPTY = (np.zeros(0, np.int32), np.zeros(0, np.int32))


# ------------------------------------------------------------------------------- delta rebuild
def test_rebuild_adversarial_tiny_cases():
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
        "only_adds": ([(1, 3), (1, 4), (1, 5), (4, 2)], []),
        "only_dels": ([], [(0, 1), (5, 4)]),
    }
    for name, (adds, dels) in cases.items():
        a = coo(adds) if adds else EMPTY
        d = coo(dels) if dels else EMPTY
        erp, eci = oracle.delta_apply(n, rp, ci, *a, *d)
        grp, gci, dinv, status, tail = gpu_rebuild(n, rp, ci, *a, *d, slack=3)
        assert status == 0, name
        assert np.array_equal(grp, erp) and np.array_equal(gci, eci), name
        assert np.all(tail == -7), name                                   # nothing written past nnz
        assert np.allclose(dinv, 1.0 / np.sqrt(np.diff(erp)), rtol=3e-7, atol=0), name


@pytest.mark.parametrize("name,n,steps", [("c1", 1000, 7), ("c2", 50_000, 3), ("c3", 1 << 16, 3), ("c5", 1 << 15, 3),
                                          ("c4", 30_000, 3)])
def test_rebuild_matches_oracle_and_from_scratch(name, n, steps):
    wl = WORKLOADS[name] if WORKLOADS[name].n == n else WORKLOADS[name].scaled(n)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    for _ in range(steps):
        lists = [x.numpy() for x in g.advance()]
        erp, eci = oracle.delta_apply(wl.n, rp, ci, *lists)
        grp, gci, dinv, status, _ = gpu_rebuild(wl.n, rp, ci, *lists)
        assert status == 0
        assert np.array_equal(grp, erp) and np.array_equal(gci, eci)
        srp, sci = (x.numpy() for x in g.csr())                         # the generator's own E_t, from scratch
        assert np.array_equal(grp, srp) and np.array_equal(gci, sci)
        assert np.allclose(dinv, 1.0 / np.sqrt(np.diff(erp)), rtol=3e-7, atol=0)
        rp, ci = erp, eci


def test_rebuild_heavy_rows_and_many_adds_between_neighbours():
    """A hub row spanning several tiles that loses and gains thousands of entries, a row that grows from
    its diagonal alone, and rows of length one around them."""
    n = 20000
    rng = np.random.default_rng(3)
    hub, lone = 7, 11
    hub_cols = np.setdiff1d(rng.choice(n, 9000, replace=False), [hub])
    pairs_r = [np.full(hub_cols.size, hub), np.arange(n)]
    pairs_c = [hub_cols, np.arange(n)]
    other_r = rng.integers(100, n, 30000)
    other_c = rng.integers(0, n, 30000)
    rp, ci = oracle.csr_from_edges(n, np.concatenate(pairs_r + [other_r]).astype(np.int32),
                                   np.concatenate(pairs_c + [other_c]).astype(np.int32))
    present = set(zip(np.repeat(np.arange(n), np.diff(rp)).tolist(), ci.tolist()))
    dels = [(hub, int(c)) for c in hub_cols[::3]]
    adds = [(hub, int(c)) for c in rng.choice(n, 6000, replace=False) if (hub, int(c)) not in present]
    adds += [(lone, int(c)) for c in rng.choice(n, 5000, replace=False) if (lone, int(c)) not in present]
    a, d = coo(adds), coo(dels)
    erp, eci = oracle.delta_apply(n, rp, ci, *a, *d)
    grp, gci, _, status, _ = gpu_rebuild(n, rp, ci, *a, *d)
    assert status == 0
    assert np.array_equal(grp, erp) and np.array_equal(gci, eci)


@pytest.mark.parametrize("n", [1000, 1023, 4097, 70_001])
def test_rebuild_with_row_pointers_that_are_not_16_byte_aligned(n):
    """The row-pointer kernel moves four rows per access when its arrays allow it; here they do not, and n leaves a
    ragged last group of rows either way."""
    wl = WORKLOADS["c1"].scaled(n)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    lists = [x.numpy() for x in g.advance()]
    erp, eci = oracle.delta_apply(n, rp, ci, *lists)
    for shift in (0, 1, 2):
        grp, gci, dinv, status, _ = gpu_rebuild(n, rp, ci, *lists, shift=shift)
        assert status == 0, shift
        assert np.array_equal(grp, erp) and np.array_equal(gci, eci), shift
        assert np.allclose(dinv, 1.0 / np.sqrt(np.diff(erp)), rtol=3e-7, atol=0), shift


def test_rebuild_stretches_of_very_short_rows():
    """Thousands of consecutive rows that hold their diagonal alone, or one more entry: a 512-entry piece of the
    merge's stream then meets more rows than it fetches row pointers for ahead of time.  Hub rows in between."""
    n = 30_000
    rng = np.random.default_rng(21)
    rows, cols = [np.arange(n)], [np.arange(n)]
    second = np.arange(0, n, 3)                                  # every third row: one more entry
    rows.append(second); cols.append((second + 7) % n)
    for hub, deg in ((9000, 2000), (9001, 700), (20_000, 5000)):
        rows.append(np.full(deg, hub)); cols.append(rng.choice(n, deg, replace=False))
    rp, ci = oracle.csr_from_edges(n, np.concatenate(rows).astype(np.int32), np.concatenate(cols).astype(np.int32))
    r_of = np.repeat(np.arange(n), np.diff(rp))
    present = set(zip(r_of.tolist(), ci.tolist()))
    off = np.flatnonzero(r_of != ci)
    dele = np.sort(rng.choice(off, off.size // 3, replace=False))
    adds = {(int(r), int(c)) for r, c in zip(rng.integers(0, n, 9000), rng.integers(0, n, 9000))}
    adds |= {(9000, int(c)) for c in rng.integers(0, n, 800)} | {(12_345, int(c)) for c in rng.integers(0, n, 300)}
    a = coo([p for p in adds if p not in present and p[0] != p[1]])
    d = (r_of[dele].astype(np.int32), ci[dele].astype(np.int32))
    erp, eci = oracle.delta_apply(n, rp, ci, *a, *d)
    grp, gci, dinv, status, _ = gpu_rebuild(n, rp, ci, *a, *d)
    assert status == 0
    assert np.array_equal(grp, erp) and np.array_equal(gci, eci)
    assert np.allclose(dinv, 1.0 / np.sqrt(np.diff(erp)), rtol=3e-7, atol=0)


def test_rebuild_rows_that_hold_their_diagonal_alone():
    """Four thousand consecutive rows of one entry each: a 512-entry piece of the merge's stream meets 512 rows, the
    most it can, and needs the pointer of a 513th.  Some of those rows gain entries, and lose them again in a second
    step; rows with entries sit before and behind the stretch."""
    n = 12_000
    rng = np.random.default_rng(33)
    rows, cols = [np.arange(n)], [np.arange(n)]
    busy = np.concatenate([np.arange(0, 3000), np.arange(7000, n)])
    rows.append(rng.choice(busy, 40_000)); cols.append(rng.integers(0, n, 40_000))
    rp, ci = oracle.csr_from_edges(n, np.concatenate(rows).astype(np.int32), np.concatenate(cols).astype(np.int32))
    assert np.all(np.diff(rp)[3000:7000] == 1)
    lone = rng.choice(np.arange(3000, 7000), 900, replace=False)
    adds = sorted({(int(r), int(c)) for r in lone for c in rng.integers(0, n, 3) if int(c) != int(r)})
    a = coo(adds)
    erp, eci = oracle.delta_apply(n, rp, ci, *a, *EMPTY)
    grp, gci, dinv, status, _ = gpu_rebuild(n, rp, ci, *a, *EMPTY)
    assert status == 0
    assert np.array_equal(grp, erp) and np.array_equal(gci, eci)
    assert np.allclose(dinv, 1.0 / np.sqrt(np.diff(erp)), rtol=3e-7, atol=0)
    back_rp, back_ci = oracle.delta_apply(n, erp, eci, *EMPTY, *a)
    grp, gci, _, status, _ = gpu_rebuild(n, erp, eci, *EMPTY, *a)
    assert status == 0
    assert np.array_equal(grp, back_rp) and np.array_equal(gci, back_ci)
    assert np.array_equal(back_rp, rp) and np.array_equal(back_ci, ci)


def test_rebuild_many_changes_in_one_row_tile():
    """More than 16 list entries per row over a whole tile of 1024 rows (the row-pointer kernel then counts
    by searching instead of walking the list), next to tiles that get nothing."""
    n = 5000
    rng = np.random.default_rng(12)
    rows_r, rows_c = [np.arange(n)], [np.arange(n)]
    for u in range(300, 1500):
        cols = np.setdiff1d(rng.choice(n, 40, replace=False), [u])
        rows_r.append(np.full(cols.size, u)); rows_c.append(cols)
    rp, ci = oracle.csr_from_edges(n, np.concatenate(rows_r).astype(np.int32), np.concatenate(rows_c).astype(np.int32))
    adds, dels = [], []
    for u in range(300, 1500):
        old = ci[rp[u]:rp[u + 1]]
        dels += [(u, int(c)) for c in old[old != u][::2]]
        fresh = np.setdiff1d(rng.choice(n, 30, replace=False), old)
        adds += [(u, int(c)) for c in fresh]
    a, d = coo(adds), coo(dels)
    assert a[0].size > 16 * 1024 and d[0].size > 16 * 1024
    erp, eci = oracle.delta_apply(n, rp, ci, *a, *d)
    grp, gci, dinv, status, _ = gpu_rebuild(n, rp, ci, *a, *d)
    assert status == 0
    assert np.array_equal(grp, erp) and np.array_equal(gci, eci)
    assert np.allclose(dinv, 1.0 / np.sqrt(np.diff(erp)), rtol=3e-7, atol=0)


def test_rebuild_validation_codes():
    n = 6
    base = [(u, u) for u in range(n)] + [(0, 1), (1, 0), (2, 3), (3, 2)]
    rp, ci = oracle.csr_from_edges(n, *coo(base))

    def status(adds, dels, raw=False):
        a = adds if raw else (coo(adds) if adds else EMPTY)
        d = coo(dels) if dels else EMPTY
        return gpu_rebuild(n, rp, ci, *a, *d, slack=4)[3]

    assert status([(0, 2)], [(0, 1)]) == 0
    assert status([(0, 1)], []) == 5                                    # added edge present
    assert status([], [(0, 2)]) == 4                                              # deleted edge absent
    assert status([(4, 4)], []) == 3                                              # diagonal named
    assert status((np.array([0, 0], np.int32), np.array([3, 2], np.int32)), [], raw=True) == 2   # unsorted
    assert status((np.array([0, 0], np.int32), np.array([2, 2], np.int32)), [], raw=True) == 2   # repeated
    assert status((np.array([0], np.int32), np.array([6], np.int32)), [], raw=True) == 1         # out of range


def test_rebuild_is_deterministic():
    wl = WORKLOADS["c3"].scaled(1 << 14)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    lists = [x.numpy() for x in g.advance()]
    a = gpu_rebuild(wl.n, rp, ci, *lists)
    b = gpu_rebuild(wl.n, rp, ci, *lists)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])


def test_csr_dinv():
    wl = WORKLOADS["c3"].scaled(1 << 12)
    rp, _ = DynamicGraph(wl).csr()
    dinv = torch.zeros(wl.n, dtype=torch.float32, device=DEV)
    dg.csr_dinv(rp.to(DEV), dinv)
    assert np.allclose(dinv.cpu().numpy(), 1.0 / np.sqrt(np.diff(rp.numpy())), rtol=3e-7, atol=0)


# ------------------------------------------------------------------------------- X W
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f_in", [16, 32, 64, 128])
@pytest.mark.parametrize("f_out", [16, 32, 64, 128])
def test_feature_transform(dtype, f_in, f_out):
    gen = torch.Generator().manual_seed(f_in * 1000 + f_out)
    for n in (1, 33, 1000, 20497):
        x = torch.randn((n, f_in), generator=gen).to(dtype)
        w = (torch.rand((f_in, f_out), generator=gen) - 0.5).to(dtype)
        h = torch.full((n, f_out), float("nan"), dtype=dtype, device=DEV)
        dg.feature_transform(x.to(DEV), w.to(DEV), h)
        torch.cuda.synchronize()
        assert_close(to_f64(h), oracle.xw(to_f64(x), to_f64(w)), dtype, f"xw n={n} {f_in}x{f_out}")


@pytest.mark.parametrize("dtype,f", [(torch.float32, 32), (torch.bfloat16, 128)])
def test_feature_transform_more_rows_than_one_grid_pass(dtype, f):
    n = 600_001                                             # the launch caps its grid and loops over row tiles
    gen = torch.Generator().manual_seed(f)
    x = torch.randn((n, f), generator=gen).to(dtype)
    w = (torch.rand((f, f), generator=gen) - 0.5).to(dtype)
    h = torch.full((n, f), float("nan"), dtype=dtype, device=DEV)
    dg.feature_transform(x.to(DEV), w.to(DEV), h)
    assert_close(to_f64(h), oracle.xw(to_f64(x), to_f64(w)), dtype, f"xw n={n} f={f}")


@pytest.mark.parametrize("dtype,f", [(torch.float32, 32), (torch.float32, 64), (torch.bfloat16, 128), (torch.bfloat16, 16)])
def test_feature_transform_with_row_scale(dtype, f):
    n = 4099
    gen = torch.Generator().manual_seed(f + 1)
    x = torch.randn((n, f), generator=gen).to(dtype)
    w = (torch.rand((f, f), generator=gen) - 0.5).to(dtype)
    scale = torch.rand(n, generator=gen) + 0.1
    h = torch.full((n, f), float("nan"), dtype=dtype, device=DEV)
    dg.feature_transform(x.to(DEV), w.to(DEV), h, row_scale=scale.to(DEV))
    expect = oracle.xw(to_f64(x), to_f64(w)) * to_f64(scale)[:, None]      # diag(scale) (X W)
    assert_close(to_f64(h), expect, dtype, f"scaled xw f={f}")


def test_feature_transform_identity_is_exact():
    x = torch.randn((777, 64))
    h = torch.empty((777, 64), device=DEV)
    dg.feature_transform(x.to(DEV), torch.eye(64, device=DEV), h)
    assert torch.equal(h.cpu(), x)


# ------------------------------------------------------------------------------- A~ H
def gpu_spmm(rp, ci, h, relu, use_dinv=True, prescaled=False):
    n, f = h.shape
    rp_d, ci_d = dev_i32(rp), dev_i32(ci)
    dinv = None
    if use_dinv:
        dinv = torch.empty(n, dtype=torch.float32, device=DEV)
        dg.csr_dinv(rp_d, dinv)
    z = torch.full((n, f), float("nan"), dtype=h.dtype, device=DEV)
    ws = torch.empty(dg.spmm_workspace(n, int(ci.size), f), dtype=torch.uint8, device=DEV)
    flags = (dg.DGNN_RELU if relu else 0) | (dg.DGNN_H_PRESCALED if prescaled else 0)
    dg.spmm(rp_d, ci_d, int(ci.size), dinv, h.to(DEV), z, ws, flags=flags)
    torch.cuda.synchronize()
    return z


def graph_with_long_rows(n, seed):
    """Power-law snapshot plus planted rows of 513, 1024, 1025 and 5000 entries (the bin edges of the
    row-length split and of the long-row chunks)."""
    wl = WORKLOADS["c3"].scaled(n)
    g = DynamicGraph(wl)
    keys = g.keys.numpy()
    rng = np.random.default_rng(seed)
    extra_r, extra_c = [], []
    for row, length in ((3, 513), (n // 2, 1024), (n - 1, 1025), (17, 5000), (18, 512)):
        cols = rng.choice(n, length, replace=False)
        extra_r.append(np.full(length, row))
        extra_c.append(cols)
    r = np.concatenate([keys >> 32] + extra_r).astype(np.int32)
    c = np.concatenate([keys & 0xFFFFFFFF] + extra_c).astype(np.int32)
    return oracle.csr_from_edges(n, r, c)


@pytest.mark.parametrize("dtype,f", [(torch.float32, 16), (torch.float32, 32), (torch.float32, 64), (torch.float32, 128),
                                     (torch.bfloat16, 16), (torch.bfloat16, 32), (torch.bfloat16, 64), (torch.bfloat16, 128)])
@pytest.mark.parametrize("relu", [False, True])
def test_spmm_power_law_with_long_rows(dtype, f, relu):
    n = 1 << 13
    rp, ci = graph_with_long_rows(n, f)
    assert np.diff(rp).max() > 5000
    h = torch.randn((n, f), generator=torch.Generator().manual_seed(f)).to(dtype)
    z = gpu_spmm(rp, ci, h, relu)
    assert_close(to_f64(z), oracle.spmm(rp, ci, to_f64(h), relu=relu), dtype, f"spmm f={f}")


@pytest.mark.parametrize("dtype,f", [(torch.float32, 32), (torch.bfloat16, 128)])
def test_spmm_prescaled_rows(dtype, f):
    """With DGNN_H_PRESCALED the rows handed over are dinv[v] H[v]; the result is the same A~ H."""
    n = 1 << 13
    rp, ci = graph_with_long_rows(n, 2)
    h = torch.randn((n, f), generator=torch.Generator().manual_seed(3)).to(dtype)
    dinv = 1.0 / np.sqrt(np.diff(rp).astype(np.float64))
    pre = torch.tensor(to_f64(h) * dinv[:, None]).to(dtype)
    z = gpu_spmm(rp, ci, pre, True, prescaled=True)
    expect = np.maximum(dinv[:, None] * oracle.spmm(rp, ci, to_f64(pre), val=np.ones(ci.size)), 0.0)
    assert_close(to_f64(z), expect, dtype, "prescaled")
    assert_close(to_f64(z), oracle.spmm(rp, ci, to_f64(h), relu=True), dtype, "prescaled vs definition")


def test_spmm_rows_without_entries_give_zero():
    """Plain A H (no dinv) on a CSR with empty rows at the start, inside, at tile edges and at the end."""
    n, f = 5000, 32
    rng = np.random.default_rng(8)
    lens = rng.integers(0, 6, n)
    lens[:3] = 0
    lens[-4:] = 0
    lens[100:140] = 0
    lens[2000] = 3000                                                    # a row over several tiles, then empties
    lens[2001:2010] = 0
    rp = np.zeros(n + 1, np.int32)
    rp[1:] = np.cumsum(lens)
    ci = np.concatenate([np.sort(rng.choice(n, l, replace=False)) for l in lens if l]).astype(np.int32)
    h = torch.randn((n, f), generator=torch.Generator().manual_seed(6))
    z = gpu_spmm(rp, ci, h, False, use_dinv=False)
    expect = oracle.spmm(rp, ci, to_f64(h), val=np.ones(ci.size))
    assert_close(to_f64(z), expect, torch.float32, "empty rows")
    assert np.all(to_f64(z)[lens == 0] == 0.0)


def test_spmm_rows_ending_exactly_on_tile_edges():
    """fp32 F=32 uses tiles of 1024 entries: rows of 1024, 2048, 1 and 1023 entries laid end to end."""
    n, f = 4096, 32
    rng = np.random.default_rng(10)
    lens = np.ones(n, np.int64)
    lens[:8] = [1024, 2048, 1, 1023, 1024, 1, 1, 3070]
    rp = np.zeros(n + 1, np.int32)
    rp[1:] = np.cumsum(lens)
    ci = np.concatenate([np.sort(rng.choice(n, l, replace=False)) for l in lens]).astype(np.int32)
    h = torch.randn((n, f), generator=torch.Generator().manual_seed(7))
    z = gpu_spmm(rp, ci, h, True)
    assert_close(to_f64(z), oracle.spmm(rp, ci, to_f64(h), relu=True), torch.float32, "tile edges")


def test_spmm_uniform_graph_ragged_tail_and_closed_form():
    wl = WORKLOADS["c2"].scaled(10_007)
    rp, ci = (x.numpy() for x in DynamicGraph(wl).csr())
    h = torch.randn((wl.n, 32), generator=torch.Generator().manual_seed(1))
    z = gpu_spmm(rp, ci, h, False)
    assert_close(to_f64(z), oracle.spmm(rp, ci, to_f64(h)), torch.float32, "uniform")
    # sqrt(1 + deg) is a fixed vector of the normalised adjacency
    d = np.sqrt(np.diff(rp).astype(np.float64))
    x = torch.tensor(np.repeat(d[:, None], 16, axis=1), dtype=torch.float32)
    assert_close(to_f64(gpu_spmm(rp, ci, x, False)), to_f64(x), torch.float32, "fixed vector")


def test_spmm_without_normalisation_counts_neighbours():
    wl = WORKLOADS["c1"]
    rp, ci = (x.numpy() for x in DynamicGraph(wl).csr())
    z = gpu_spmm(rp, ci, torch.ones((wl.n, 16)), False, use_dinv=False)
    assert np.array_equal(to_f64(z), np.repeat(np.diff(rp).astype(np.float64)[:, None], 16, axis=1))


def test_spmm_is_deterministic():
    n = 1 << 13
    rp, ci = graph_with_long_rows(n, 5)
    h = torch.randn((n, 32), generator=torch.Generator().manual_seed(9))
    a, b = gpu_spmm(rp, ci, h, True), gpu_spmm(rp, ci, h, True)
    assert torch.equal(a, b)


# ------------------------------------------------------------------------------- M-transform
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,w", [(8, 3), (32, 8), (40, 16), (5, 1), (6, 9), (70, 32), (3, 2), (1, 4)])
def test_mproduct_paper_weights(dtype, T, w):
    n, f = 333, 32
    z = torch.randn((T, n, f), generator=torch.Generator().manual_seed(T * 100 + w)).to(dtype)
    expect = oracle.mproduct(to_f64(z), oracle.m_matrix(T, w))
    zd = z.to(DEV)
    y = torch.full_like(zd, float("nan"))
    dg.mproduct(zd, y, w)
    assert_close(to_f64(y), expect, dtype, f"mproduct T={T} w={w}")
    assert torch.equal(zd.cpu(), z)                                       # input untouched out of place
    dg.mproduct(zd, zd, w)                                               # in place
    torch.cuda.synchronize()
    assert torch.equal(zd, y)


def test_mproduct_explicit_band():
    T, w, n, f = 12, 4, 100, 16
    gen = torch.Generator().manual_seed(4)
    z = torch.randn((T, n, f), generator=gen)
    band = torch.randn((T, w), generator=gen)
    M = np.zeros((T, T))
    for t in range(T):
        for j in range(min(w, t + 1)):
            M[t, t - j] = float(band[t, j])
    y = torch.empty((T, n, f), device=DEV)
    dg.mproduct(z.to(DEV), y, w, m_band=band.to(DEV))
    assert_close(to_f64(y), oracle.mproduct(to_f64(z), M), torch.float32, "explicit band")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,w", [(40, 17), (50, 24), (70, 32), (20, 32), (33, 25)])
def test_mproduct_explicit_band_long_windows(dtype, T, w):
    """Explicit coefficients with windows beyond 16 (the kernels that keep the ring as raw pieces moving down one slot
    per step), forward and adjoint, out of place and in place."""
    n, f = 200, 32
    gen = torch.Generator().manual_seed(T * 37 + w)
    z = torch.randn((T, n, f), generator=gen).to(dtype)
    band = torch.randn((T, w), generator=gen) / w ** 0.5
    M = np.zeros((T, T))
    for t in range(T):
        for j in range(min(w, t + 1)):
            M[t, t - j] = float(band[t, j])
    zd, bd = z.to(DEV), band.to(DEV)
    y = torch.full_like(zd, float("nan"))
    dg.mproduct(zd, y, w, m_band=bd)
    assert_close(to_f64(y), oracle.mproduct(to_f64(z), M), dtype, f"explicit band T={T} w={w}")
    g = torch.full_like(zd, float("nan"))
    dg.mproduct_backward(zd, g, w, m_band=bd)
    assert_close(to_f64(g), oracle.mproduct_t(to_f64(z), M), dtype, f"adjoint, explicit band T={T} w={w}")
    dg.mproduct(zd, zd, w, m_band=bd)
    torch.cuda.synchronize()
    assert torch.equal(zd, y)


@pytest.mark.parametrize("w", [3, 8, 16])
def test_mproduct_running_sum_forgets_what_has_left_the_window(w):
    """The paper's weights are served by a running window sum.  What a frame leaves behind in it must not stay for the
    rest of the series: after a spike of 1e6 and after an infinity, every frame from two windows behind the event on
    is what the definition gives (exact zeros for a window of zeros, finite values after the infinity)."""
    T, n, f = 7 * w + 5, 64, 16
    z = torch.randn((T, n, f), generator=torch.Generator().manual_seed(w))
    z[2] *= 1.0e6                                                         # a spike among ordinary values ...
    z[4 * w + 1:] = 0.0                                                   # ... and, later, nothing but zeros
    zd = z.to(DEV)
    y = torch.empty_like(zd)
    dg.mproduct(zd, y, w)
    torch.cuda.synchronize()
    expect = oracle.mproduct(to_f64(z), oracle.m_matrix(T, w))
    assert_close(to_f64(y[:2 + w]), expect[:2 + w], torch.float32, "while the spike is in the window")
    assert_close(to_f64(y[2 + 2 * w:4 * w + 1]), expect[2 + 2 * w:4 * w + 1], torch.float32, "two windows behind the spike")
    assert float(y[6 * w + 1:].abs().max()) == 0.0                        # a window of zeros gives zeros, exactly
    z2 = torch.randn((T, n, f), generator=torch.Generator().manual_seed(w + 1))
    z2[3, 5, 7] = float("inf")
    y2 = torch.empty((T, n, f), device=DEV)
    dg.mproduct(z2.to(DEV), y2, w)
    torch.cuda.synchronize()
    clean = z2.clone(); clean[3, 5, 7] = 0.0
    late = slice(3 + 2 * w, T)
    assert bool(torch.isfinite(y2[late]).all())
    assert_close(to_f64(y2[late]), oracle.mproduct(to_f64(clean), oracle.m_matrix(T, w))[late], torch.float32, "after the infinity has left")
    g2 = torch.empty((T, n, f), device=DEV)
    dg.mproduct_backward(z2.to(DEV), g2, w)                               # going back the walk starts at the end
    torch.cuda.synchronize()
    early = slice(0, 3 - 2 * w) if 3 - 2 * w > 0 else slice(0, 0)
    assert bool(torch.isfinite(g2[early]).all())


def test_csr_validate_finds_what_is_wrong():
    """A canonical snapshot passes; each way of breaking it is reported with its code."""
    wl = WORKLOADS["c3"].scaled(1 << 12, T=1)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy().copy() for x in g.csr())
    n, nnz = wl.n, int(ci.size)
    status = torch.full((1,), -9, dtype=torch.int32, device=DEV)

    def code(rp_, ci_, nnz_=nnz, diag=True):
        dg.csr_validate(torch.from_numpy(rp_).to(DEV), torch.from_numpy(ci_).to(DEV), nnz_, status, require_diagonal=diag)
        return int(status.item())

    assert code(rp, ci) == 0
    u = int(np.argmax(np.diff(rp) >= 3))                                  # a row with at least three entries
    bad = ci.copy(); bad[rp[u]], bad[rp[u] + 1] = bad[rp[u] + 1], bad[rp[u]]
    assert code(rp, bad) == 8                                             # DGNN_BAD_ROW_ORDER
    bad = ci.copy(); bad[rp[u] + 1] = bad[rp[u]]
    assert code(rp, bad) == 8                                             # a repeated column
    bad = ci.copy(); bad[rp[u + 1] - 1] = n
    assert code(rp, bad) == 1                                             # DGNN_BAD_INDEX_RANGE
    bad = rp.copy(); bad[u + 1] = bad[u] - 1
    assert code(bad, ci) == 7                                             # DGNN_BAD_ROWPTR
    assert code(rp, ci, nnz_=nnz - 1) == 7                                # rowptr[n] != nnz
    bad = rp.copy(); bad[0] = 1
    assert code(bad, ci) == 7
    # a snapshot without one of its self loops: fine as a matrix, not as A + I
    keep = np.ones(nnz, dtype=bool)
    keep[rp[u] + int(np.searchsorted(ci[rp[u]:rp[u + 1]], u))] = False
    lens = np.diff(rp); lens[u] -= 1
    rp2 = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    assert code(rp2, ci[keep], nnz_=nnz - 1) == 9                         # DGNN_BAD_NO_DIAGONAL
    assert code(rp2, ci[keep], nnz_=nnz - 1, diag=False) == 0
