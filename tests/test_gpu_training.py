"""GPU parity of a whole training step over a block (forward keeping activations, then gradient
propagation in the reverse direction, Section "Gradient Checkpoint") against the CPU oracle: weight
gradients of every layer, the input gradient, and the snapshots met on the way back."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph, features, glorot_weight, gradient
from helpers import assert_close, to_f64
from dtdg_synth.blocks import make_block
from paper_2109_07893_amd.training import make_trainer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = {
    "undirected_1layer_window": WORKLOADS["c1"],
    "undirected_2layers_window": replace(WORKLOADS["c1"], layers=2, f=32, name="c1-2l"),
    "directed_1layer": WORKLOADS["c3"].scaled(4096, T=5),
    "directed_2layers_window": replace(WORKLOADS["c3"].scaled(4096, T=6), layers=2, window=3, name="c3-2l-w"),
    "bf16_window": replace(WORKLOADS["c4"].scaled(3000, T=6), window=4, name="c4-small"),
    "bf16_directed_2layers": replace(WORKLOADS["c3"].scaled(2048, T=4), layers=2, dtype="bf16", f=64, name="c3-bf16"),
}


def oracle_training_step(wl):
    """Forward and backward of the block in float64; returns (dW per layer, dX per frame, Y, snapshots,
    stored activations).  Which gradient elements the ReLU lets through is a yes/no decision taken on the
    activations as they are STORED (float32 or bfloat16): the backward half therefore starts from the oracle's
    activations rounded to the storage type, and the GPU is handed the same stored activations, so that both
    sides take that decision on identical numbers."""
    T, L = wl.T, wl.layers
    store = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    ws = [to_f64(glorot_weight(wl, layer)) for layer in range(L)]
    snaps, acts, xs = [], [], []
    for t in range(1, T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        snaps.append((rp, ci))
        cur = to_f64(features(wl, t))
        xs.append(cur)
        layer_out = []
        for layer in range(L):
            cur = oracle.gcn_layer(rp, ci, cur, ws[layer], relu=True)
            layer_out.append(cur)
        acts.append(layer_out)
    z_top = np.stack([a[-1] for a in acts])
    stored = [[torch.from_numpy(a).to(store) for a in layer_out] for layer_out in acts]
    g_y = np.stack([to_f64(gradient(wl, t)) for t in range(1, T + 1)])
    if wl.window:
        M = oracle.m_matrix(T, wl.window)
        y = oracle.mproduct(z_top, M)
        g_z = oracle.mproduct_t(g_y, M)
    else:
        y, g_z = z_top, g_y
    dws = [np.zeros_like(w) for w in ws]
    dxs = []
    for t in range(T, 0, -1):
        rp, ci = snaps[t - 1]
        gin = g_z[t - 1]
        for layer in range(L - 1, -1, -1):
            below = xs[t - 1] if layer == 0 else to_f64(stored[t - 1][layer - 1])
            dw, gin = oracle.gcn_layer_backward(rp, ci, below, ws[layer], to_f64(stored[t - 1][layer]), gin)
            dws[layer] += dw
        dxs.append(gin)
    return dws, dxs[::-1], y, snaps, stored


@pytest.mark.parametrize("case", sorted(CASES))
def test_training_step_matches_oracle(case):
    wl = CASES[case]
    dtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    dws, dxs, y, snaps, stored = oracle_training_step(wl)
    blk = make_block(wl, DEV, gen_device="cpu")
    tr = make_trainer(wl, blk, want_dx=True)
    out = tr.forward()
    assert_close(to_f64(out), y, dtype, f"{case}: forward output")
    for t in range(wl.T):                     # the stored activations the backward half starts from (see above)
        for layer in range(wl.layers):
            tr.z[layer, t].copy_(stored[t][layer])
    g_y = torch.stack([gradient(wl, t) for t in range(1, wl.T + 1)]).to(DEV)
    tr.backward(g_y)
    torch.cuda.synchronize()
    # after the walk back, the two alternating slots hold A_2 and A_3 again, bit for bit
    for t in (2, 3):
        if t <= wl.T:
            slot = tr.a.slot_of(t)
            rp, ci = snaps[t - 1]
            assert np.array_equal(tr.a.rowptr[slot].cpu().numpy(), rp), (case, t)
            assert np.array_equal(tr.a.colidx[slot][: ci.size].cpu().numpy(), ci), (case, t)
    for layer in range(wl.layers):
        assert_close(to_f64(tr.dw[layer]), dws[layer], dtype, f"{case}: dW of layer {layer}")
    # dX has gone through three stored tensors per layer (masked gradient, aggregated gradient, input gradient)
    for t in range(wl.T):
        assert_close(to_f64(tr.dx[t]), dxs[t], dtype, f"{case}: dX of frame {t + 1}", stores=3 * wl.layers)


def test_training_step_repeats_bit_for_bit():
    wl = CASES["directed_2layers_window"]
    blk = make_block(wl, DEV, gen_device="cpu")
    g_y = torch.stack([gradient(wl, t) for t in range(1, wl.T + 1)]).to(DEV)
    runs = []
    for _ in range(2):
        tr = make_trainer(wl, blk)
        tr.forward()
        tr.backward(g_y)
        torch.cuda.synchronize()
        runs.append([d.clone() for d in tr.dw])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("case,bsize", [("undirected_2layers_window", 3), ("directed_2layers_window", 2),
                                        ("directed_2layers_window", 4), ("undirected_1layer_window", 1),
                                        ("directed_1layer", 2), ("bf16_window", 4)])
def test_checkpointed_training_equals_the_one_block_step(case, bsize):
    """The series cut into checkpoint blocks (forward keeping only the hand-over, then per block a rerun and the
    backward pass, last block first) must give the gradients of the whole series."""
    from paper_2109_07893_amd.training import CheckpointedTrainer
    wl = CASES[case]
    dtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    dws, _, y, _, _ = oracle_training_step(wl)
    series = make_block(wl, DEV, gen_device="cpu")
    ck = CheckpointedTrainer(wl, series, bsize)
    outs = {}
    ck.forward(on_block=lambda b, a, e, yb: outs.__setitem__((a, e), yb.clone()))
    got_y = torch.cat([outs[k] for k in sorted(outs)])
    assert_close(to_f64(got_y), y, dtype, f"{case}: forward output in blocks of {bsize}")
    g_y = torch.stack([gradient(wl, t) for t in range(1, wl.T + 1)]).to(DEV)
    ck.backward(g_y)
    torch.cuda.synchronize()
    # here both sides decide the ReLU mask on their own activations: a result rounded once through fp32 storage
    # leaves the mask alone except for pre-activations within rounding of zero, of which these cases have none;
    # with bf16 storage the mask differs in a fraction of a percent of the elements, so dW is only required to
    # agree with the one-block GPU step, bit for bit, and that one is checked against the oracle above
    one = make_trainer(wl, series)
    one.forward()
    one.backward(g_y)
    torch.cuda.synchronize()
    for layer in range(wl.layers):
        if dtype == torch.float32:
            assert_close(to_f64(ck.dw[layer]), dws[layer], dtype, f"{case}: dW of layer {layer}, blocks of {bsize}")
        assert_close(to_f64(ck.dw[layer]), to_f64(one.dw[layer]), torch.float32, f"{case}: blocks vs one block, layer {layer}")


def test_one_weight_per_timestep():
    """Section "EvolveGCN": the GCN weight differs from timestep to timestep; the library takes W per call, the
    driver passes W_t, and every timestep gets a weight gradient of its own."""
    from paper_2109_07893_amd.pipeline import BlockRunner
    wl = replace(WORKLOADS["c3"].scaled(4096, T=4), layers=2, name="c3-evolving")
    blk = make_block(wl, DEV, gen_device="cpu")
    blk.w_t = [[glorot_weight(wl, layer, t=t).to(DEV) for layer in range(wl.layers)] for t in range(1, wl.T + 1)]
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    snaps, acts = [], []
    for t in range(1, wl.T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        snaps.append((rp, ci))
        cur, outs = to_f64(features(wl, t)), []
        for layer in range(wl.layers):
            cur = oracle.gcn_layer(rp, ci, cur, to_f64(blk.w_t[t - 1][layer]), relu=True)
            outs.append(cur)
        acts.append(outs)
    runner = BlockRunner(blk, keep_all_z=True)
    runner.load_first()
    runner.run_resident()
    for t in range(wl.T):
        assert_close(to_f64(runner.z[t]), acts[t][-1], torch.float32, f"forward with W_t, t={t + 1}")
    tr = make_trainer(wl, blk)
    tr.forward()
    stored = [[torch.from_numpy(a).to(torch.float32) for a in outs] for outs in acts]
    for t in range(wl.T):
        for layer in range(wl.layers):
            tr.z[layer, t].copy_(stored[t][layer])
    g_y = torch.stack([gradient(wl, t) for t in range(1, wl.T + 1)]).to(DEV)
    tr.backward(g_y)
    for t in range(wl.T):
        rp, ci = snaps[t]
        gin = to_f64(g_y[t])
        for layer in range(wl.layers - 1, -1, -1):
            below = to_f64(features(wl, t + 1)) if layer == 0 else to_f64(stored[t][layer - 1])
            dw, gin = oracle.gcn_layer_backward(rp, ci, below, to_f64(blk.w_t[t][layer]), to_f64(stored[t][layer]), gin)
            assert_close(to_f64(tr.dw_t[t][layer]), dw, torch.float32, f"dW_t t={t + 1} layer {layer}")


def test_gradient_descent_on_the_weights_reduces_a_loss():
    """End to end: the weight gradients drive plain gradient descent on L = 1/2 |Y - Y*|^2, where Y* comes from a
    hidden weight pair; the loss layer (Y - Y*) is the caller's, everything below it is the library's."""
    wl = replace(WORKLOADS["c1"], layers=2, f=32, name="c1-descent")
    blk = make_block(wl, DEV, gen_device="cpu")
    tr = make_trainer(wl, blk)
    target = tr.forward().clone()                           # outputs under the generator's weights
    blk.w = [w + 0.3 * torch.randn(w.shape, generator=torch.Generator().manual_seed(k)).to(DEV) for k, w in enumerate(blk.w)]
    losses = []
    lr = 2e-5
    for _ in range(40):
        y = tr.forward()
        g_y = (y - target).contiguous()
        losses.append(float(0.5 * (g_y.double() ** 2).sum()))
        tr.backward(g_y)
        blk.w = [(w - lr * dw).contiguous() for w, dw in zip(blk.w, tr.dw)]
    assert losses[-1] < 0.2 * losses[0], losses[::8]
    assert all(b <= a * 1.001 for a, b in zip(losses, losses[1:])), losses


def test_evolving_weights_end_to_end():
    """EvolveGCN (Section "EvolveGCN"): W_t = LSTM(W_{t-1}) produced on the device, used by the GCN steps of a
    block, and the loss's gradient carried back through the GCN steps AND the weight recurrence to U_x, U_h, b and
    W_0; against the oracle's chain (every link pinned by finite differences)."""
    import oracle
    from paper_2109_07893_amd.evolve import EvolvingWeights
    wl = WORKLOADS["c3"].scaled(1 << 12, T=5)
    T, f = wl.T, wl.f
    gen = torch.Generator().manual_seed(5)
    w0 = torch.randn((f, f), generator=gen) / np.sqrt(f)
    u_x = torch.randn((f, 4 * f), generator=gen) / np.sqrt(f)
    u_h = torch.randn((f, 4 * f), generator=gen) / np.sqrt(f)
    bias = torch.randn(4 * f, generator=gen) * 0.1
    ev = EvolvingWeights(w0.to(DEV), u_x.to(DEV), u_h.to(DEV), bias.to(DEV), T)
    w_t = ev.forward()
    blk = make_block(wl, DEV, gen_device="cpu")
    blk.w_t = [[w] for w in w_t]
    tr = make_trainer(wl, blk)
    g_y = torch.randn((T, wl.n, f), generator=gen)
    for _ in range(2):
        ev.forward()
        tr.forward()
        tr.backward(g_y.to(DEV))
        ev.backward([tr.dw_t[t][0] for t in range(T)])
    torch.cuda.synchronize()
    # oracle
    W0, UX, UH, Bv = (to_f64(x) for x in (w0, u_x, u_h, bias))
    ws, _ = oracle.evolve_weights(W0, UX, UH, Bv, T)
    for t in range(T):
        assert_close(to_f64(w_t[t]), ws[t], torch.float32, f"W_{t + 1}")
    from dtdg_synth import DynamicGraph, features
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    d_w = []
    for t in range(1, T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        x = to_f64(features(wl, t))
        z = oracle.gcn_layer(rp, ci, x, ws[t - 1], relu=True)
        d_w.append(oracle.gcn_layer_backward(rp, ci, x, ws[t - 1], z, to_f64(g_y[t - 1]))[0])
    want = oracle.evolve_weights_backward(W0, UX, UH, Bv, d_w)
    for name, got, exp in (("dU_x", ev.du_x, want[0]), ("dU_h", ev.du_h, want[1]), ("db", ev.db, want[2]), ("dW_0", ev.dw0, want[3])):
        err = np.abs(to_f64(got) - exp).max()
        assert err <= 2e-4 * np.abs(exp).max(), f"{name}: max err {err:.3e} against max |.| {np.abs(exp).max():.3e}"


@pytest.mark.parametrize("name", ["c1", "c3"])
def test_training_step_with_all_snapshots_resident(name):
    """keep_snapshots: every A_t (and A_t^T) of the block stays in a slot of its own and the backward pass rebuilds
    nothing; the gradients are bit for bit those of the trainer that walks the snapshots back by reverse rebuilds."""
    wl = WORKLOADS[name] if name == "c1" else WORKLOADS[name].scaled(1 << 12, T=5)
    blk = make_block(wl, DEV, gen_device="cpu")
    g_y = torch.stack([gradient(wl, t, "cpu") for t in range(1, wl.T + 1)]).to(DEV)
    ref, kept = make_trainer(wl, blk), make_trainer(wl, blk, keep_snapshots=True)
    for tr in (ref, kept):
        for _ in range(2):
            tr.forward()
            tr.backward(g_y)
    torch.cuda.synchronize()
    for a, b in zip(ref.dw, kept.dw):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["c1", "c3"])
def test_training_step_as_a_hip_graph_repeats_the_eager_result(name):
    """The training step captured once and replayed several times, with eager steps and synchronisations between the
    replays; every replay must leave exactly the gradients the eager step leaves."""
    from paper_2109_07893_amd.training import capture_training_step
    wl = WORKLOADS[name] if name == "c1" else WORKLOADS[name].scaled(1 << 12, T=4)
    blk = make_block(wl, DEV, gen_device="cpu")
    g_y = torch.stack([gradient(wl, t, "cpu") for t in range(1, wl.T + 1)]).to(DEV)
    tr = make_trainer(wl, blk)
    tr.forward(); tr.backward(g_y)
    torch.cuda.synchronize()
    want = [d.clone() for d in tr.dw]
    graph = capture_training_step(tr, g_y)
    for k in range(4):
        for d in tr.dw:
            d.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(tr.dw, want):
            assert torch.equal(a, b), k
        tr.forward(); tr.backward(g_y)                 # eager work between replays
        torch.cuda.synchronize()
        for a, b in zip(tr.dw, want):
            assert torch.equal(a, b), k
