"""GPU parity of the whole forward pass over a block (rebuild -> X W -> A~ H per layer -> M-transform)
against the oracle, through the same caller-side plumbing the benchmark uses."""
import numpy as np
import pytest
import torch

import oracle
from dtdg_synth import WORKLOADS
from helpers import assert_close, oracle_block, to_f64
from dtdg_synth.blocks import make_block
from paper_2109_07893_amd.pipeline import BlockRunner

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_gpu(wl, T=None, pinned=False, from_pinned=False):
    blk = make_block(wl, DEV, gen_device="cpu", pinned=pinned, T=T)
    runner = BlockRunner(blk, keep_all_z=True)
    runner.load_first()
    csr = []
    if from_pinned:
        runner.run_from_pinned()
    else:
        runner.run_resident(validate=True, on_snapshot=lambda t, slot: csr.append(runner.snapshot_to_host(t)))
    torch.cuda.synchronize()
    assert int(runner.status.abs().sum()) == 0
    return runner, csr


@pytest.mark.parametrize("name,n,T", [("c1", 1000, 8), ("c2", 20_000, 10), ("c3", 1 << 14, 4), ("c4", 10_000, 20),
                                      ("c5", 1 << 14, 8)])
def test_block_forward_matches_oracle(name, n, T):
    wl = WORKLOADS[name] if WORKLOADS[name].n == n else WORKLOADS[name].scaled(n, T=T)
    runner, csr = run_gpu(wl, T=T)
    zs = []
    for t, (rp, ci, z) in enumerate(oracle_block(wl, T=T), start=1):
        grp, gci = csr[t - 1]
        assert np.array_equal(grp, rp) and np.array_equal(gci, ci), f"CSR differs at t={t}"
        zs.append(z)
    expect = np.stack(zs)
    if wl.window:
        expect = oracle.mproduct(expect, oracle.m_matrix(T, wl.window))
    assert_close(to_f64(runner.z), expect, runner.z.dtype, f"{wl.name} output")


def test_pinned_host_pipeline_equals_resident():
    wl = WORKLOADS["c5"].scaled(1 << 14)
    a, _ = run_gpu(wl)
    b, _ = run_gpu(wl, pinned=True, from_pinned=True)
    assert torch.equal(a.z, b.z)
    T = a.blk.T
    for t in (T - 1, T):
        slot, nnz = a.slot_of(t), a.blk.nnz[t - 1]
        assert torch.equal(a.rowptr[slot], b.rowptr[slot])
        assert torch.equal(a.colidx[slot][:nnz], b.colidx[slot][:nnz])


def test_pinned_host_pipeline_with_lists_requested_ahead():
    """A stream of passes in which the first lists of the next pass are requested while the current one finishes:
    every pass must leave what the resident pass leaves."""
    wl = WORKLOADS["c5"].scaled(1 << 14)
    a, _ = run_gpu(wl)
    blk = make_block(wl, DEV, gen_device="cpu", pinned=True)
    runner = BlockRunner(blk, keep_all_z=True)
    runner.load_first()
    for k in range(3):
        runner.z.fill_(float("nan"))
        runner.run_from_pinned(prefetch_next=True)
        torch.cuda.synchronize()
        assert torch.equal(a.z, runner.z), k
    runner.run_from_pinned()                      # takes up the outstanding request, asks for nothing more
    torch.cuda.synchronize()
    assert torch.equal(a.z, runner.z)
    runner.run_from_pinned()                      # and a pass that starts from scratch again
    torch.cuda.synchronize()
    assert torch.equal(a.z, runner.z)


def test_block_forward_is_deterministic():
    wl = WORKLOADS["c3"].scaled(1 << 13, T=3)
    a, _ = run_gpu(wl)
    b, _ = run_gpu(wl)
    assert torch.equal(a.z, b.z)


def test_transfer_size_of_graph_difference():
    """Bytes shipped per step: 8 per difference entry, against 4 (nnz + n + 1) for a whole CSR snapshot
    (the saving argued in Section "Graph-difference Based Input Transfer")."""
    wl = WORKLOADS["c5"].scaled(1 << 14)
    blk = make_block(wl, DEV, gen_device="cpu", pinned=True)
    for t, (lists, pins) in enumerate(zip(blk.deltas, blk.pinned), start=2):
        shipped = sum(p.numel() * p.element_size() for p in pins)
        assert shipped == 8 * (lists[0].numel() + lists[2].numel())
        whole = 4 * (blk.nnz[t - 1] + blk.n + 1)
        assert shipped < whole / 4


def test_forward_pass_as_a_hip_graph_repeats_the_eager_result():
    """The resident pass captured once and replayed several times, with eager work of the same program and
    synchronisations between the replays; every replay must leave exactly what the eager pass leaves."""
    wl = WORKLOADS["c1"]
    blk = make_block(wl, DEV, gen_device="cpu")
    runner = BlockRunner(blk)
    runner.load_first()
    runner.run_resident()
    torch.cuda.synchronize()
    want = runner.z.clone()
    want_rp, want_ci = runner.snapshot_to_host(wl.T)
    graph = runner.capture()
    for k in range(4):
        runner.z.fill_(float("nan"))
        runner.rowptr[wl.T % 2].fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(runner.z, want), k
        rp, ci = runner.snapshot_to_host(wl.T)
        assert np.array_equal(rp, want_rp) and np.array_equal(ci, want_ci), k
        runner.run_resident()                      # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(runner.z, want), k
