"""GPU parity of the sliding-window sum of snapshots (Section "Smoothening the Input Graphs") computed on the
device, C = S + alpha A_in + beta A_out, against the oracle: structure and values bit for bit (the values are
counts or dyadic fractions, exact in fp32 and fp64 alike, so the decision "is the result zero" is the same on
both sides)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(DEV)


def gpu_combine(n, s, a_in, alpha, a_out, beta, slack=0, diag=0.0, s_bound=None):
    """The result as the device leaves it: the number of stored entries read from rowptr_c[n].  s_bound: pass S's
    entry count as this upper bound instead of the exact figure (the kernels must take the last row pointer)."""
    rp_s, ci_s, val_s = s
    nnz_s = int(ci_s.size)
    pad = 0 if s_bound is None else s_bound - nnz_s
    ci_p = np.concatenate([ci_s, np.full(pad, 2**31 - 1, dtype=np.int32)]) if pad else ci_s          # poison behind the entries
    val_p = None if val_s is None else (np.concatenate([val_s, np.full(pad, np.nan)]) if pad else val_s)
    s_d = (dev(rp_s, torch.int32), dev(ci_p, torch.int32), None if val_p is None else dev(val_p, torch.float32), nnz_s + pad)
    ops = [None if a is None else (dev(a[0], torch.int32), dev(a[1], torch.int32), int(a[1].size)) for a in (a_in, a_out)]
    cap = nnz_s + sum(0 if a is None else int(a[1].size) for a in (a_in, a_out)) + slack
    out = (torch.full((n + 1,), -7, dtype=torch.int32, device=DEV), torch.full((max(cap, 1),), -7, dtype=torch.int32, device=DEV),
           torch.full((max(cap, 1),), float("nan"), device=DEV))
    ws = torch.empty(dg.csr_combine_workspace(nnz_s + pad), dtype=torch.uint8, device=DEV)
    status = torch.full((1,), 99, dtype=torch.int32, device=DEV)
    dg.csr_combine(s_d, ops[0], alpha, ops[1], beta, out, ws, diag_value=diag, status=status)
    torch.cuda.synchronize()
    assert int(status) == 0
    nnz = int(out[0][n])
    # nothing written behind the result
    assert bool((out[1][nnz:] == -7).all()) and bool(torch.isnan(out[2][nnz:]).all())
    return out[0].cpu().numpy(), out[1][:nnz].cpu().numpy(), out[2][:nnz].cpu().numpy()


def check(n, s, a_in, alpha, a_out, beta, what, diag=0.0, s_bound=None):
    want = oracle.csr_combine(n, s, a_in, alpha, a_out, beta, diag=diag)
    got = gpu_combine(n, s, a_in, alpha, a_out, beta, diag=diag, s_bound=s_bound)
    assert np.array_equal(got[0], want[0]), f"{what}: rowptr"
    assert np.array_equal(got[1], want[1]), f"{what}: colidx"
    assert np.array_equal(got[2].astype(np.float64), want[2]), f"{what}: values"


def random_csr(n, density, rng, hubs=()):
    """Rows of binomial length; `hubs` = (row, length) pairs get that many entries instead."""
    rows, cols = [], []
    for u in range(n):
        k = dict(hubs).get(u, rng.binomial(n, density))
        c = np.sort(rng.choice(n, size=min(k, n), replace=False))
        rows.append(np.full(c.size, u)); cols.append(c)
    return oracle.csr_from_edges(n, np.concatenate(rows), np.concatenate(cols))


@pytest.mark.parametrize("n,density,seed", [(300, 0.05, 0), (2000, 0.02, 1), (5000, 0.004, 2), (700, 0.3, 3)])
@pytest.mark.parametrize("alpha,beta", [(1.0, -1.0), (2.0, 0.5)])
def test_combine_random_operands(n, density, seed, alpha, beta):
    rng = np.random.default_rng(seed)
    s = random_csr(n, density, rng)
    a_in, a_out = random_csr(n, density, rng), random_csr(n, density / 2, rng)
    val = rng.integers(1, 4, s[1].size).astype(np.float64)
    check(n, s + (val,), a_in, alpha, a_out, beta, "three operands")
    check(n, s + (None,), a_in, alpha, None, beta, "no A_out, S unweighted")
    check(n, s + (val,), None, alpha, a_out, beta, "no A_in")
    check(n, s + (val,), None, alpha, None, beta, "S alone")
    check(n, s + (val,), a_in, alpha, a_out, beta, "diagonal entries take a given value", diag=1.0)
    check(n, s + (val,), a_in, alpha, a_out, beta, "S's entry count given as an upper bound", s_bound=int(s[1].size) + 777)


def test_combine_hub_rows_empty_rows_and_long_spans():
    """Rows much longer than a wavefront's range in each of the operands in turn (so a row is cut at columns,
    pieces are merged by all lanes, and spans of A_in / A_out exceed the staging area), next to empty rows."""
    n = 9000
    rng = np.random.default_rng(11)
    s = random_csr(n, 0.001, rng, hubs=((3, 5000), (4, 0), (5, 0), (100, 2047), (101, 1), (4000, 8999), (8999, 3000)))
    a_in = random_csr(n, 0.001, rng, hubs=((3, 4000), (4, 6000), (7, 0), (101, 7000), (4000, 10), (8998, 0), (8999, 2500)))
    a_out = random_csr(n, 0.0005, rng, hubs=((3, 4500), (5, 3000), (100, 2047), (4000, 8000)))
    val = rng.integers(1, 3, s[1].size).astype(np.float64)
    check(n, s + (val,), a_in, 1.0, a_out, -1.0, "hubs")
    check(n, s + (val,), a_in, 1.0, s, -1.0, "S partly cancelled by itself")
    check(n, a_in + (None,), s, 1.0, a_out, -1.0, "operands exchanged")


def csr_with_row_lengths(n, lengths, rng):
    """A CSR whose row u has lengths[u] entries at random columns."""
    rows = np.repeat(np.arange(n), lengths)
    cols = np.concatenate([np.sort(rng.choice(n, size=int(k), replace=False)) for k in lengths]) if rows.size else np.zeros(0, dtype=np.int64)
    return oracle.csr_from_edges(n, rows, cols)


@pytest.mark.parametrize("nnz_s", [256, 64 * 256, 64 * 256 + 1, 2 * 64 * 256 - 1, 2 * 64 * 256])
def test_combine_entry_counts_on_the_edges_of_ranges_and_boundary_tiles(nnz_s):
    """S with exactly as many entries as a whole number of wavefront ranges (256 entries each), and as a whole number
    of the boundary kernel's groups of 64 ranges (then the end of everything is the first boundary of a group of
    its own), and one more or less; rows of one entry (a boundary group meets more rows than it stages: 16384)
    next to long rows."""
    n = 40_000
    rng = np.random.default_rng(nnz_s)
    lengths = np.zeros(n, dtype=np.int64)
    ones = min(n - 100, nnz_s // 2)
    lengths[:ones] = 1                                       # a stretch of one-entry rows at the beginning
    rest = nnz_s - ones
    long_rows = rng.choice(np.arange(ones, n), size=40, replace=False)
    cut = np.sort(rng.choice(rest + 1, size=39, replace=True))
    lengths[long_rows] = np.diff(np.concatenate([[0], cut, [rest]]))
    assert int(lengths.sum()) == nnz_s and int(lengths.max()) <= n
    s = csr_with_row_lengths(n, lengths, rng)
    assert s[1].size == nnz_s
    a_in = random_csr(n, 0.0004, rng, hubs=((int(long_rows[0]), 3000), (5, 40)))
    a_out = csr_with_row_lengths(n, np.minimum(lengths, 3), rng)
    val = rng.integers(1, 3, s[1].size).astype(np.float64)
    check(n, s + (val,), a_in, 1.0, a_out, -1.0, f"{nnz_s} entries")
    check(n, s + (val,), a_in, 1.0, s, -1.0, f"{nnz_s} entries, S cancelled by itself where the value is 1")
    check(n, s + (val,), a_in, 1.0, a_out, -1.0, f"{nnz_s} entries, given as an upper bound", s_bound=nnz_s + 64 * 256)


def test_combine_empty_s_and_total_cancellation():
    n = 500
    rng = np.random.default_rng(5)
    a = random_csr(n, 0.05, rng)
    empty = (np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32))
    check(n, empty + (None,), a, 1.0, None, -1.0, "S empty")
    check(n, empty + (None,), None, 1.0, None, -1.0, "everything empty")
    check(n, a + (None,), None, 1.0, a, -1.0, "S - S")
    check(n, a + (None,), a, 1.0, a, -2.0, "S + S - 2 S")


def test_combine_reports_the_size_when_the_result_does_not_fit():
    n = 400
    rng = np.random.default_rng(6)
    s, a = random_csr(n, 0.05, rng), random_csr(n, 0.05, rng)
    want = oracle.csr_combine(n, s + (None,), a, 1.0)
    s_d = (dev(s[0], torch.int32), dev(s[1], torch.int32), None, int(s[1].size))
    a_d = (dev(a[0], torch.int32), dev(a[1], torch.int32), int(a[1].size))
    cap = int(want[1].size) - 1
    out = (torch.full((n + 1,), -7, dtype=torch.int32, device=DEV), torch.full((cap,), -7, dtype=torch.int32, device=DEV),
           torch.zeros(cap, device=DEV))
    ws = torch.empty(dg.csr_combine_workspace(int(s[1].size)), dtype=torch.uint8, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    dg.csr_combine(s_d, a_d, 1.0, None, -1.0, out, ws, status=status)            # enqueue-only: the verdict is on the device
    torch.cuda.synchronize()
    assert int(status) == 10                                                     # DGNN_BAD_CAPACITY
    assert int(out[0][n]) == want[1].size                                        # the size that would have been needed
    assert bool((out[0][:n] == -7).all()) and bool((out[1] == -7).all())         # nothing else written


@pytest.mark.parametrize("name,n,life,T", [("c1", 1000, 3, 10), ("c3", 1 << 13, 4, 10), ("c2", 20_000, 2, 10), ("c5", 1 << 13, 8, 10),
                                           ("c5", 1 << 17, 2, 4)])     # the last one: several tiles of the scan over ranges
def test_sliding_window_sum_on_the_device(name, n, life, T):
    """S_t = S_{t-1} + A_t - A_{t-l} carried on the device over a series; the expected S_t is formed here from the
    raw oracle snapshots (sorted keys of the window, counted with numpy), not step by step."""
    wl = WORKLOADS[name].scaled(n, T=T) if n != WORKLOADS[name].n else WORKLOADS[name]
    T = min(T, wl.T)
    raw = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in raw.csr())
    snaps = [(rp, ci)]
    s = (rp, ci, None)
    for t in range(2, T + 1):
        rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in raw.advance()])
        snaps.append((rp, ci))
        s = gpu_combine(wl.n, s, snaps[t - 1], 1.0, snaps[t - 1 - life] if t - life >= 1 else None, -1.0)
        keys = [(np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(p)) << 32) | c.astype(np.int64)
                for p, c in snaps[max(0, t - life):t]]
        want_keys, counts = np.unique(np.concatenate(keys), return_counts=True)
        got_keys = (np.repeat(np.arange(wl.n, dtype=np.int64), np.diff(s[0])) << 32) | s[1].astype(np.int64)
        assert np.array_equal(got_keys, want_keys), (name, t)
        assert np.array_equal(s[2], counts.astype(np.float32)), (name, t)


@pytest.mark.parametrize("name,n,T,life,diag", [("c3", 1 << 13, 6, 3, 1.0), ("c2", 20_000, 5, 2, 1.0), ("c4", 10_000, 9, 4, 1.0),
                                                ("c1", 1000, 8, 8, 1.0), ("c3", 1 << 13, 6, 3, 0.0), ("c1", 1000, 8, 4, 0.0)])
def test_forward_pass_on_smoothed_snapshots(name, n, T, life, diag):
    """The whole forward pass with the smoothing done on the device (rebuild, sliding-window sum, weighted
    normalisation, X W, aggregation, M-transform) against the oracle: the expected smoothed snapshot is the sum of
    the oracle's raw snapshots of the window, normalised by the weighted form of Eqn (1).  diag = 1: edge-life
    smoothing (the self loop counts once); diag = 0: the M-transform of the adjacency tensor."""
    from helpers import assert_close, to_f64
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.pipeline import SmoothedRunner
    wl = WORKLOADS[name].scaled(n, T=T) if n != WORKLOADS[name].n else WORKLOADS[name]
    T = min(T, wl.T)
    blk = make_block(wl, DEV, gen_device="cpu", T=T)
    runner = SmoothedRunner(blk, life, keep_all_z=True, diag_value=diag)
    runner.run_resident(validate=True)
    torch.cuda.synchronize()
    assert int(runner.status.abs().sum()) == 0 and int(runner.status_s.abs().sum()) == 0
    raw = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in raw.csr())
    snaps, zs = [(rp, ci)], []
    ws = [to_f64(w) for w in blk.w]
    for t in range(1, T + 1):
        if t >= 2:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in raw.advance()])
            snaps.append((rp, ci))
        s = snaps[max(0, t - life)] + (None,)
        for other in snaps[max(0, t - life) + 1:t]:
            s = oracle.csr_combine(wl.n, s, other, 1.0, diag=diag)
        val = oracle.gcn_values_weighted(s[0], s[1], np.ones(s[1].size) if s[2] is None else s[2])
        cur = to_f64(blk.x[t - 1])
        for w in ws:
            cur = oracle.spmm(s[0], s[1], oracle.xw(cur, w), relu=True, val=val)
        zs.append(cur)
    expect = np.stack(zs)
    if wl.window:
        expect = oracle.mproduct(expect, oracle.m_matrix(T, wl.window))
    assert_close(to_f64(runner.z), expect, runner.z.dtype, f"{wl.name} smoothed forward", stores=blk.layers + (1 if wl.window else 0))


@pytest.mark.parametrize("seed", range(80))
def test_combine_random_shapes(seed):
    """Seeded random operand shapes: sizes, densities, hub rows, empty stretches, weights, presence of A_in / A_out."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 3000))
    dens = [float(rng.choice([0.0, 0.001, 0.01, 0.1])) * min(1.0, 300.0 / n) * 3 for _ in range(3)]

    def operand(d):
        hubs = tuple((int(rng.integers(0, n)), int(rng.integers(0, n + 1))) for _ in range(int(rng.integers(0, 4))))
        rp, ci = random_csr(n, d, rng, hubs=hubs)
        if rng.random() < 0.3 and n > 10:                 # a stretch of empty rows
            a, b = sorted(rng.integers(0, n, 2))
            keep = np.ones(ci.size, dtype=bool)
            keep[rp[a]:rp[b]] = False
            lens = np.diff(rp); lens[a:b] = 0
            rp, ci = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), ci[keep]
        return rp, ci

    s, a_in, a_out = operand(dens[0]), operand(dens[1]), operand(dens[2])
    val = None if rng.random() < 0.3 else rng.integers(1, 5, s[1].size).astype(np.float64)
    alpha, beta = float(rng.choice([1.0, 2.0, 0.5])), float(rng.choice([-1.0, -2.0, 1.0]))
    check(n, s + (val,), a_in if rng.random() < 0.85 else None, alpha, a_out if rng.random() < 0.7 else None, beta, f"seed {seed}")


@pytest.mark.parametrize("name,n,T,life", [("c2", 20_000, 6, 3), ("c3", 1 << 12, 5, 2), ("c1", 1000, 8, 4)])
def test_training_step_on_smoothed_snapshots(name, n, T, life):
    """Forward and backward on smoothed snapshots (the graphs TM-GCN and EvolveGCN train on), smoothing on the
    device, every S_t (and S_t^T for the directed workload) kept resident; weight gradients against the oracle."""
    from dtdg_synth import gradient
    from helpers import assert_close, to_f64
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.training import make_smoothed_trainer
    wl = WORKLOADS[name].scaled(n, T=T) if n != WORKLOADS[name].n else WORKLOADS[name]
    T = min(T, wl.T)
    blk = make_block(wl, DEV, gen_device="cpu", T=T)
    tr = make_smoothed_trainer(wl, blk, life)
    g_y = torch.stack([gradient(wl, t, "cpu") for t in range(1, T + 1)]).to(DEV)
    for _ in range(2):
        y = tr.forward()
        tr.backward(g_y)
    torch.cuda.synchronize()
    # oracle
    raw = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in raw.csr())
    snaps, sm, zs = [(rp, ci)], [], []
    ws = [to_f64(w) for w in blk.w]
    for t in range(1, T + 1):
        if t >= 2:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in raw.advance()])
            snaps.append((rp, ci))
        s = snaps[max(0, t - life)] + (None,)
        for other in snaps[max(0, t - life) + 1:t]:
            s = oracle.csr_combine(wl.n, s, other, 1.0, diag=1.0)
        val = oracle.gcn_values_weighted(s[0], s[1], np.ones(s[1].size) if s[2] is None else s[2])
        sm.append((s[0], s[1], val))
        acts = [to_f64(blk.x[t - 1])]
        for w in ws:
            acts.append(oracle.spmm(s[0], s[1], oracle.xw(acts[-1], w), relu=True, val=val))
        zs.append(acts)
    top = np.stack([a[-1] for a in zs])
    M = oracle.m_matrix(T, wl.window) if wl.window else None
    assert_close(to_f64(y), oracle.mproduct(top, M) if wl.window else top, y.dtype, f"{name}: smoothed forward",
                 stores=blk.layers + (1 if wl.window else 0))
    g_top = oracle.mproduct_t(to_f64(g_y), M) if wl.window else to_f64(g_y)
    d_w = [0.0] * len(ws)
    for t in range(T, 0, -1):
        g = g_top[t - 1]
        for layer in range(len(ws) - 1, -1, -1):
            g_h = oracle.spmm_t(sm[t - 1][0], sm[t - 1][1], oracle.relu_grad(g, zs[t - 1][layer + 1]), val=sm[t - 1][2])
            d_w[layer] = d_w[layer] + oracle.weight_grad(zs[t - 1][layer], g_h)
            g = oracle.input_grad(g_h, ws[layer])
    for layer in range(len(ws)):
        err = np.abs(to_f64(tr.dw[layer]) - d_w[layer]).max()
        assert err <= 3e-4 * np.abs(d_w[layer]).max(), f"{name} dW[{layer}]: max err {err:.3e} against {np.abs(d_w[layer]).max():.3e}"


def test_evolvegcn_on_smoothed_snapshots():
    """The EvolveGCN model of the paper in one piece: edge-life smoothing on the device, one GCN weight per timestep
    produced by the LSTM over the weights, and the loss's gradient carried back through the GCN steps and the
    weight recurrence; against the oracle's chain."""
    from dtdg_synth import features, gradient
    from helpers import assert_close, to_f64
    from paper_2109_07893_amd.evolve import EvolvingWeights
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.training import make_smoothed_trainer
    wl = WORKLOADS["c3"].scaled(1 << 12, T=5)
    T, f, life = wl.T, wl.f, 3
    gen = torch.Generator().manual_seed(9)
    w0 = torch.randn((f, f), generator=gen) / np.sqrt(f)
    u_x, u_h = (torch.randn((f, 4 * f), generator=gen) / np.sqrt(f) for _ in range(2))
    bias = torch.randn(4 * f, generator=gen) * 0.1
    ev = EvolvingWeights(w0.to(DEV), u_x.to(DEV), u_h.to(DEV), bias.to(DEV), T)
    blk = make_block(wl, DEV, gen_device="cpu")
    blk.w_t = [[w] for w in ev.forward()]
    tr = make_smoothed_trainer(wl, blk, life)
    g_y = torch.stack([gradient(wl, t, "cpu") for t in range(1, T + 1)]).to(DEV)
    for _ in range(2):
        ev.forward()
        tr.forward()
        tr.backward(g_y)
        ev.backward([tr.dw_t[t][0] for t in range(T)])
    torch.cuda.synchronize()
    W0, UX, UH, Bv = (to_f64(x) for x in (w0, u_x, u_h, bias))
    ws, _ = oracle.evolve_weights(W0, UX, UH, Bv, T)
    raw = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in raw.csr())
    snaps, d_w = [(rp, ci)], []
    for t in range(1, T + 1):
        if t >= 2:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in raw.advance()])
            snaps.append((rp, ci))
        s = snaps[max(0, t - life)] + (None,)
        for other in snaps[max(0, t - life) + 1:t]:
            s = oracle.csr_combine(wl.n, s, other, 1.0, diag=1.0)
        val = oracle.gcn_values_weighted(s[0], s[1], np.ones(s[1].size) if s[2] is None else s[2])
        x = to_f64(features(wl, t))
        z = oracle.spmm(s[0], s[1], oracle.xw(x, ws[t - 1]), relu=True, val=val)
        assert_close(to_f64(tr.z[0, t - 1]), z, torch.float32, f"Z_{t}")
        g_h = oracle.spmm_t(s[0], s[1], oracle.relu_grad(to_f64(g_y[t - 1]), z), val=val)
        d_w.append(oracle.weight_grad(x, g_h))
    want = oracle.evolve_weights_backward(W0, UX, UH, Bv, d_w)
    for name, got, exp in (("dU_x", ev.du_x, want[0]), ("dU_h", ev.du_h, want[1]), ("db", ev.db, want[2]), ("dW_0", ev.dw0, want[3])):
        err = np.abs(to_f64(got) - exp).max()
        assert err <= 3e-4 * np.abs(exp).max(), f"{name}: max err {err:.3e} against max |.| {np.abs(exp).max():.3e}"


def test_smoothed_forward_with_lists_from_pinned_host_memory():
    """The smoothed forward pass with the raw difference lists streamed from pinned host memory (copies overlapped
    with the computation) leaves exactly what the pass with resident lists leaves."""
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.pipeline import SmoothedRunner
    wl = WORKLOADS["c5"].scaled(1 << 13, T=7)
    a = SmoothedRunner(make_block(wl, DEV, gen_device="cpu"), life=3, keep_all_z=True)
    a.run_resident()
    b = SmoothedRunner(make_block(wl, DEV, gen_device="cpu", pinned=True), life=3, keep_all_z=True)
    for _ in range(2):
        b.z.fill_(float("nan"))
        b.run_from_pinned()
        torch.cuda.synchronize()
        assert torch.equal(a.z, b.z)


@pytest.mark.parametrize("name,n,T,life", [("c5", 1 << 13, 9, 3), ("c2", 20_000, 6, 2), ("c3", 1 << 13, 7, 4), ("c4", 10_000, 12, 4)])
def test_smoothed_pass_on_two_streams_equals_the_pass_on_one(name, n, T, life):
    """overlap=True: rebuild, sliding-window sum, normalisation and X W of snapshot t+1 on a second stream beside the
    aggregation of snapshot t (S, its normalisation and H alternate with t).  Frames and the last smoothed snapshot
    must be those of the one-stream pass bit for bit: resident lists and pinned ones, passes back to back, and a
    one-stream pass in between."""
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.pipeline import SmoothedRunner
    wl = WORKLOADS[name].scaled(n, T=T)
    a = SmoothedRunner(make_block(wl, DEV, gen_device="cpu"), life=life, keep_all_z=True)
    a.run_resident()
    torch.cuda.synchronize()
    nnz = a.stored_entries()
    want_s = [x[:nnz].clone() if i else x.clone() for i, x in enumerate(a.cur[:3])]
    b = SmoothedRunner(make_block(wl, DEV, gen_device="cpu", pinned=True), life=life, keep_all_z=True)

    def same(what):
        torch.cuda.synchronize()
        assert int(b.status.abs().sum()) == 0 and int(b.status_s.abs().sum()) == 0
        assert torch.equal(a.z, b.z), what
        assert b.stored_entries() == nnz, what
        for i, (w, g) in enumerate(zip(want_s, b.cur[:3])):
            assert torch.equal(w, g[:nnz] if i else g), what
        b.z.fill_(float("nan"))

    b.run_resident(overlap=True)
    same("resident lists")
    b.run_resident(overlap=True)
    b.run_resident(overlap=True)
    same("two passes back to back")
    b.run_from_pinned(overlap=True)
    same("pinned lists")
    b.run_from_pinned(prefetch_next=True, overlap=True)
    b.run_from_pinned(prefetch_next=True, overlap=True)
    same("pinned lists requested ahead")
    b.run_from_pinned()
    same("one-stream pass after two-stream passes")
    b.run_resident(overlap=True)
    same("and a two-stream pass again")


def test_smoothed_pass_as_a_hip_graph_repeats_the_eager_result():
    """Every call of the smoothed pass only enqueues (the sliding-window sum leaves its size on the device), so the
    pass can be recorded as a HIP graph: replayed several times with eager passes and synchronisations in between,
    every replay must leave exactly what the eager pass leaves -- frames, the smoothed snapshot, its size."""
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.pipeline import SmoothedRunner
    wl = WORKLOADS["c3"].scaled(1 << 13, T=6)
    blk = make_block(wl, DEV, gen_device="cpu")
    runner = SmoothedRunner(blk, 3, keep_all_z=True)
    runner.run_resident()
    torch.cuda.synchronize()
    want_z = runner.z.clone()
    nnz = runner.stored_entries()
    want_s = [x.clone() for x in runner.cur[:3]]
    graph = runner.capture()
    for k in range(4):
        runner.z.fill_(float("nan"))
        for x in runner.cur[:3]:
            x.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        assert int(runner.status_s.abs().sum()) == 0
        assert torch.equal(runner.z.view(torch.int32), want_z.view(torch.int32)), k
        assert runner.stored_entries() == nnz
        assert torch.equal(runner.cur[0], want_s[0]) and torch.equal(runner.cur[1][:nnz], want_s[1][:nnz]), k
        assert torch.equal(runner.cur[2][:nnz], want_s[2][:nnz]), k
        runner.run_resident()                      # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(runner.z.view(torch.int32), want_z.view(torch.int32)), k
