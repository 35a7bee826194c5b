"""dgnn_spmm_static, the aggregation for callers that cannot allocate (its scratch is a device array inside the
library), against dgnn_spmm through the C boundary: same kernels, so the two results must agree bit for bit, and
within the parity tolerance of the oracle.  Two calls in a row share the one scratch array, the second on a smaller
snapshot, so whatever the first call left there must not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph
from helpers import assert_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def power_law_snapshot(n, hub_rows, seed):
    """A c3-shaped snapshot with a few planted rows longer than a wavefront's range, so that rows are cut by range
    ends and the carry records in the scratch array are really used."""
    g = DynamicGraph(WORKLOADS["c3"].scaled(n))
    keys = g.keys.numpy()
    rng = np.random.default_rng(seed)
    rows, cols = [keys >> 32], [keys & 0xFFFFFFFF]
    for row, length in hub_rows:
        rows.append(np.full(length, row))
        cols.append(rng.choice(n, length, replace=False))
    return oracle.csr_from_edges(n, np.concatenate(rows).astype(np.int32), np.concatenate(cols).astype(np.int32))


def both_ways(rp, ci, h, flags):
    n, f = h.shape
    nnz = int(ci.size)
    rp_d = torch.from_numpy(rp).to(DEV)
    ci_d = torch.from_numpy(ci).to(DEV)
    dinv = torch.empty(n, dtype=torch.float32, device=DEV)
    dg.csr_dinv(rp_d, dinv)
    h_d = h.to(DEV)
    z_ws = torch.full((n, f), float("nan"), dtype=h.dtype, device=DEV)
    z_static = torch.full((n, f), float("nan"), dtype=h.dtype, device=DEV)
    ws = torch.empty(dg.spmm_workspace(n, nnz, f), dtype=torch.uint8, device=DEV)
    dg.spmm(rp_d, ci_d, nnz, dinv, h_d, z_ws, ws, flags=flags)
    before = torch.cuda.memory_allocated(DEV)
    dg.spmm_static(rp_d, ci_d, nnz, dinv, h_d, z_static, flags=flags)
    assert torch.cuda.memory_allocated(DEV) == before
    torch.cuda.synchronize()
    return z_ws, z_static


@pytest.mark.parametrize("dtype,f", [(torch.float32, 32), (torch.bfloat16, 128)])
def test_two_calls_in_a_row_second_one_smaller(dtype, f):
    cases = [
        (1 << 16, [(5, 40000), (1 << 14, 9000), ((1 << 16) - 1, 8193)], dg.DGNN_RELU),   # many ranges, rows cut by range ends
        (4096, [(7, 1500)], 0),                                                            # a handful of ranges
    ]
    for n, hubs, flags in cases:
        rp, ci = power_law_snapshot(n, hubs, seed=f)
        h = torch.randn((n, f), generator=torch.Generator().manual_seed(n)).to(dtype)
        z_ws, z_static = both_ways(rp, ci, h, flags)
        assert torch.equal(z_ws.view(torch.uint8), z_static.view(torch.uint8)), f"n={n}: differs from dgnn_spmm"
        expect = oracle.spmm(rp, ci, to_f64(h), relu=bool(flags & dg.DGNN_RELU))
        assert_close(to_f64(z_static), expect, dtype, f"dgnn_spmm_static n={n} f={f}")


def test_more_ranges_than_the_scratch_array_has_records_for():
    """8.8 M stored entries at width 128 in fp32: the usual ranges (192 entries at this size and width) would need 46
    thousand records of 1040 bytes, half as many again as the array holds, so this entry point makes its ranges longer.  Rows cut by a range's end are then summed in other pieces than in
    dgnn_spmm: same result within the rounding of the sums, and within the bound against the oracle."""
    n, f = 1 << 19, 128
    rp, ci = power_law_snapshot(n, [(3, 50_000), (77_777, 9_000)], seed=9)
    assert (16 + 8 * f) * (ci.size // 192) > dg.spmm_static_limit()
    h = torch.randn((n, f), generator=torch.Generator().manual_seed(5))
    z_ws, z_static = both_ways(rp, ci, h, dg.DGNN_RELU)
    assert_close(to_f64(z_static), to_f64(z_ws), torch.float32, "dgnn_spmm_static against dgnn_spmm")
    rows = np.unique(np.concatenate([np.random.default_rng(1).choice(n, 4096, replace=False), [3, 77_777]]))
    expect = oracle.spmm(rp, ci, to_f64(h), relu=True, rows=rows)
    assert_close(to_f64(z_static)[rows], expect, torch.float32, "dgnn_spmm_static, stretched ranges")


def test_sizes_beyond_the_scratch_array_are_refused():
    limit = dg.spmm_static_limit()
    assert limit == 32 << 20
    n, f = 1024, 128
    rp = torch.zeros(n + 1, dtype=torch.int32, device=DEV)
    ci = torch.zeros(16, dtype=torch.int32, device=DEV)
    h = torch.zeros((n, f), device=DEV)
    z = torch.zeros((n, f), device=DEV)
    nnz_too_many = 1 << 29                      # its carry records would take more than the array holds
    assert dg.spmm_workspace(n, nnz_too_many, f) > limit
    lib = dg.load_library()
    rc = lib.dgnn_spmm_static(n, nnz_too_many, rp.data_ptr(), ci.data_ptr(), None, h.data_ptr(), f, z.data_ptr(), 0, 0, None)
    assert rc == -3
