"""The size limit of the boundary on the GPU: a snapshot with just under 2^31 stored entries (the index type is
int32).  Built by formula on the device, checked on rows the CPU can compute one by one."""
import numpy as np
import pytest
import torch

import paper_2109_07893_amd as dg
from helpers import assert_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

N = 1 << 20
ROW = 2047                      # entries per row; N * ROW = 2^31 - 2^20
STRIDE = 512


def big_snapshot():
    """Row r holds the columns j * 512 + (r mod 512), j = 0..2046, with the diagonal swapped in for the entry
    it is nearest to... kept simple: the diagonal is NOT forced; rows are ascending and duplicate-free, which is
    all the aggregation needs (dinv comes from the row lengths)."""
    rowptr = (torch.arange(N + 1, dtype=torch.int64, device=DEV) * ROW).to(torch.int32)
    colidx = torch.empty(N * ROW, dtype=torch.int32, device=DEV)
    view = colidx.view(N, ROW)
    base = (torch.arange(ROW, dtype=torch.int32, device=DEV) * STRIDE)[None, :]
    chunk = 1 << 16
    for r0 in range(0, N, chunk):
        r = torch.arange(r0, min(N, r0 + chunk), dtype=torch.int32, device=DEV)
        view[r0:r0 + chunk] = base + (r % STRIDE)[:, None]
    return rowptr, colidx


def cols_of(r):
    return np.arange(ROW, dtype=np.int64) * STRIDE + (r % STRIDE)


@pytest.mark.timeout(600)
def test_aggregation_at_the_int32_limit():
    rowptr, colidx = big_snapshot()
    nnz = N * ROW
    assert nnz == (1 << 31) - (1 << 20)
    f = 16
    h = torch.randn((N, f), generator=torch.Generator().manual_seed(1)).to(DEV)
    z = torch.full((N, f), float("nan"), device=DEV)
    dinv = torch.empty(N, device=DEV)
    dg.csr_dinv(rowptr, dinv)
    ws = torch.empty(dg.spmm_workspace(N, nnz, f), dtype=torch.uint8, device=DEV)
    dg.spmm(rowptr, colidx, nnz, dinv, h, z, ws, flags=dg.DGNN_RELU)
    torch.cuda.synchronize()
    assert not torch.isnan(z).any()
    hh = to_f64(h)
    rows = np.concatenate([[0, 1, 511, 512, N - 1, N - 2], np.random.default_rng(2).integers(0, N, 200)])
    want = np.stack([np.maximum(hh[cols_of(r)].sum(axis=0) / ROW, 0.0) for r in rows])   # every dinv is ROW^(-1/2)
    assert_close(to_f64(z[torch.as_tensor(rows, device=DEV)]), want, torch.float32, "rows of the 2^31-entry snapshot")


@pytest.mark.timeout(600)
def test_rebuild_at_the_int32_limit():
    rowptr, colidx = big_snapshot()
    nnz = N * ROW
    # delete the first, a middle and the last entry of a few rows; add columns that fall between the stored ones
    rows = np.array([0, 1, 777, N // 2, N - 2, N - 1], np.int64)
    dr = np.repeat(rows, 3).astype(np.int32)
    dc = np.concatenate([cols_of(r)[[0, 1000, ROW - 1]] for r in rows]).astype(np.int32)
    ar = np.repeat(rows, 2).astype(np.int32)
    ac = np.concatenate([cols_of(r)[[5, 2000]] + 1 for r in rows]).astype(np.int32)      # r % 512 + 1 <= 512: between neighbours
    lists = [torch.as_tensor(x).to(DEV) for x in (ar, ac, dr, dc)]
    cap = nnz + ar.size - dr.size
    rpn = torch.empty(N + 1, dtype=torch.int32, device=DEV)
    cin = torch.full((cap,), -7, dtype=torch.int32, device=DEV)
    dinv = torch.empty(N, device=DEV)
    ws = torch.empty(dg.delta_rebuild_workspace(N, nnz, ar.size, dr.size), dtype=torch.uint8, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    got_nnz = dg.delta_rebuild(rowptr, colidx, nnz, lists[0], lists[1], ar.size, lists[2], lists[3], dr.size, rpn, cin, dinv, ws,
                               flags=0, d_status=status)
    torch.cuda.synchronize()
    assert got_nnz == cap
    # row pointers: every touched row lost one entry net
    shift = torch.zeros(N + 1, dtype=torch.int64, device=DEV)
    for k, r in enumerate(sorted(rows)):
        shift[r + 1:] -= 1
    assert torch.equal(rpn.to(torch.int64), rowptr.to(torch.int64) + shift)
    # untouched stretches are straight copies; touched rows are the merged rows
    edges = [0] + [int(x) for r in sorted(rows) for x in (r, r + 1)] + [N]
    for a, b in zip(edges[0::2], edges[1::2]):
        if b > a:
            src = colidx[int(rowptr[a]):int(rowptr[b])] if b < N + 1 else None
            dst = cin[int(rpn[a]):int(rpn[b])]
            assert torch.equal(src, dst), (a, b)
    for r in rows:
        old = set(cols_of(r).tolist())
        want = sorted((old - set(dc[dr == r].tolist())) | set(ac[ar == r].tolist()))
        got = cin[int(rpn[r]):int(rpn[r + 1])].cpu().numpy().tolist()
        assert got == want, r
