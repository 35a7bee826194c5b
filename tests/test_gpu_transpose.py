"""dgnn_csr_transpose and dgnn_coo_transpose (the transposed first snapshot and the transposed difference lists the
reverse pass of a directed graph needs, Section "Gradient Checkpoint") against the oracle, bit for bit; and the
transposed chain they feed: rebuilding A_t^T from A_1^T and the transposed lists gives the transpose of A_t."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def random_csr(n, density, rng, hubs=()):
    rows, cols = [], []
    for u in range(n):
        k = dict(hubs).get(u, rng.binomial(n, density))
        c = np.sort(rng.choice(n, size=min(k, n), replace=False))
        rows.append(np.full(c.size, u)); cols.append(c)
    return oracle.csr_from_edges(n, np.concatenate(rows), np.concatenate(cols))


@pytest.mark.parametrize("n,density,hubs", [(1, 1.0, ()), (37, 0.2, ()), (1000, 0.01, ((3, 900), (4, 0), (999, 1000))),
                                            (5000, 0.002, ((0, 0), (1, 0), (2, 0), (4999, 0))), (70000, 0.0002, ((5, 60000),))])
def test_csr_transpose(n, density, hubs):
    rng = np.random.default_rng(n)
    rp, ci = random_csr(n, density, rng, hubs)
    val = rng.normal(size=ci.size).astype(np.float32)
    want = oracle.csr_transpose(n, rp, ci, val)
    got = dg.csr_transpose(dev(rp), dev(ci), int(ci.size), dev(val))
    torch.cuda.synchronize()
    assert np.array_equal(got[0].cpu().numpy(), want[0]) and np.array_equal(got[1].cpu().numpy(), want[1])
    assert np.array_equal(got[2].cpu().numpy().astype(np.float64), want[2])
    plain = dg.csr_transpose(dev(rp), dev(ci), int(ci.size))
    assert len(plain) == 2 and torch.equal(plain[0], got[0]) and torch.equal(plain[1], got[1])
    back = dg.csr_transpose(got[0], got[1], int(ci.size))
    assert np.array_equal(back[0].cpu().numpy(), rp) and np.array_equal(back[1].cpu().numpy(), ci)


def test_csr_transpose_without_entries():
    n = 50
    rp = torch.zeros(n + 1, dtype=torch.int32, device=DEV)
    ci = torch.zeros(1, dtype=torch.int32, device=DEV)
    rp_t, ci_t = dg.csr_transpose(rp, ci, 0)
    assert int(rp_t.abs().sum()) == 0 and ci_t.numel() == 0


@pytest.mark.parametrize("n,m", [(10, 0), (10, 1), (1000, 5000), (1 << 20, 300000)])
def test_coo_transpose(n, m):
    rng = np.random.default_rng(m)
    keys = np.unique(rng.integers(0, n, m).astype(np.int64) * n + rng.integers(0, n, m))
    row, col = (keys // n).astype(np.int32), (keys % n).astype(np.int32)
    want = oracle.coo_transpose(row, col)
    got = dg.coo_transpose(n, dev(row), dev(col))
    torch.cuda.synchronize()
    assert np.array_equal(got[0].cpu().numpy(), want[0]) and np.array_equal(got[1].cpu().numpy(), want[1])


@pytest.mark.parametrize("name,n", [("c3", 1 << 13), ("c5", 1 << 15)])
def test_transposed_chain_follows_the_series(name, n):
    """A directed series: A_1^T by dgnn_csr_transpose, the lists by dgnn_coo_transpose, every A_t^T by dgnn_delta_rebuild;
    compared with the oracle's transpose of the oracle's A_t."""
    wl = WORKLOADS[name].scaled(n, T=5)
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    rp_t, ci_t = dg.csr_transpose(dev(rp), dev(ci), int(ci.size))
    nnz = int(ci.size)
    for t in range(2, wl.T + 1):
        lists = [x.numpy() for x in g.advance()]
        rp, ci = oracle.delta_apply(wl.n, rp, ci, *lists)
        ar, ac = dg.coo_transpose(wl.n, dev(lists[0]), dev(lists[1]))
        dr, dc = dg.coo_transpose(wl.n, dev(lists[2]), dev(lists[3]))
        rp_n = torch.empty(wl.n + 1, dtype=torch.int32, device=DEV)
        ci_n = torch.empty(int(ci.size), dtype=torch.int32, device=DEV)
        ws = torch.empty(dg.delta_rebuild_workspace(wl.n, nnz, int(ar.numel()), int(dr.numel())), dtype=torch.uint8, device=DEV)
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        got = dg.delta_rebuild(rp_t, ci_t, nnz, ar, ac, int(ar.numel()), dr, dc, int(dr.numel()), rp_n, ci_n, None, ws,
                               flags=dg.DGNN_VALIDATE, d_status=status)
        torch.cuda.synchronize()
        assert int(status) == 0 and got == ci.size
        want = oracle.csr_transpose(wl.n, rp, ci)
        assert np.array_equal(rp_n.cpu().numpy(), want[0]) and np.array_equal(ci_n.cpu().numpy(), want[1]), t
        rp_t, ci_t, nnz = rp_n, ci_n, int(ci.size)
