"""GPU parity of the CD-GCN pieces (Section "CD-GCN") against the CPU oracle: the skip-connection step, the LSTM
cell, and a whole layer over a block of timesteps."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from dtdg_synth import WORKLOADS, DynamicGraph, features, glorot_weight
from helpers import assert_close, to_f64
from paper_2109_07893_amd.cdgcn import CdgcnLayer
from dtdg_synth.blocks import make_block

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
WIDTHS = [16, 32, 64, 128]


def randn(shape, seed, dtype=torch.float32, scale=1.0):
    return (torch.randn(shape, generator=torch.Generator().manual_seed(seed)) * scale).to(dtype)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f0", WIDTHS)
@pytest.mark.parametrize("f1", [16, 128])
def test_concat_relu(dtype, f0, f1):
    n = 777
    y0, y1 = randn((n, f0), f0, dtype), randn((n, f1), f1 + 1, dtype)
    out = torch.full((n, f0 + f1), float("nan"), dtype=dtype, device=DEV)
    dg.concat_relu(y0.to(DEV), y1.to(DEV), out)
    want = np.maximum(np.concatenate([to_f64(y0), to_f64(y1)], axis=1), 0.0)
    assert np.array_equal(to_f64(out), want)          # nothing is computed: exact


@pytest.mark.parametrize("dtype,f_in,f_out", [(torch.float32, 16, 32), (torch.float32, 32, 32), (torch.float32, 32, 64),
                                              (torch.float32, 64, 64), (torch.float32, 64, 32), (torch.bfloat16, 32, 32),
                                              (torch.bfloat16, 64, 64), (torch.bfloat16, 32, 64), (torch.bfloat16, 64, 32)])
@pytest.mark.parametrize("n", [1, 33, 4097, 150_001])
def test_transform_concat_relu(dtype, f_in, f_out, n):
    """Y = relu([Y0 | Y0 W]) in one pass against the definition, and against the product followed by the concatenation:
    the left part is a copy under the ReLU (exact), the right part the same product (fp32: same kernel arithmetic,
    bit for bit; bf16: rounded to bf16 once either way, bit for bit as well)."""
    assert dg.transform_concat_relu_supported(torch.empty((1, f_in), dtype=dtype), f_out)
    x = randn((n, f_in), n + f_in, dtype)
    w = (randn((f_in, f_out), 3) / np.sqrt(f_in)).to(dtype)
    out = torch.full((n, f_in + f_out), float("nan"), dtype=dtype, device=DEV)
    dg.transform_concat_relu(x.to(DEV), w.to(DEV), out)
    want = np.maximum(np.concatenate([to_f64(x), oracle.xw(to_f64(x), to_f64(w))], axis=1), 0.0)
    assert np.array_equal(to_f64(out)[:, :f_in], want[:, :f_in])
    assert_close(to_f64(out), want, dtype, f"relu([x | x W]) {f_in}->{f_out} n={n}")
    y1 = torch.empty((n, f_out), dtype=dtype, device=DEV)
    two = torch.empty_like(out)
    dg.feature_transform(x.to(DEV), w.to(DEV), y1)
    dg.concat_relu(x.to(DEV), y1, two)
    assert torch.equal(out.view(torch.uint8), two.view(torch.uint8))


def test_transform_concat_relu_refuses_other_widths():
    assert not dg.transform_concat_relu_supported(torch.empty((1, 128)), 32)
    assert not dg.transform_concat_relu_supported(torch.empty((1, 64), dtype=torch.bfloat16), 128)
    x = torch.zeros((8, 128), device=DEV)
    with pytest.raises(dg.DgnnError):
        dg.transform_concat_relu(x, torch.zeros((128, 32), device=DEV), torch.zeros((8, 160), device=DEV))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("hidden", WIDTHS)
@pytest.mark.parametrize("with_bias", [False, True])
def test_lstm_cell(dtype, hidden, with_bias):
    n = 513
    gx, gh = randn((n, 4 * hidden), hidden, dtype, 2.0), randn((n, 4 * hidden), hidden + 1, dtype, 2.0)
    c = randn((n, hidden), hidden + 2, dtype)
    bias = randn((4 * hidden,), hidden + 3) if with_bias else None
    a = to_f64(gx) + to_f64(gh) + (to_f64(bias)[None, :] if with_bias else 0.0)
    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    ai, af, ag, ao = (a[:, q * hidden:(q + 1) * hidden] for q in range(4))
    c_want = sig(af) * to_f64(c) + sig(ai) * np.tanh(ag)
    h_want = sig(ao) * np.tanh(c_want)
    cd = c.to(DEV)
    h = torch.full((n, hidden), float("nan"), dtype=dtype, device=DEV)
    dg.lstm_cell(gx.to(DEV), gh.to(DEV), bias.to(DEV) if with_bias else None, cd, cd, h)      # state updated in place
    assert_close(to_f64(cd), c_want, dtype, "c")
    assert_close(to_f64(h), h_want, dtype, "h")


@pytest.mark.parametrize("case", ["undirected_f32", "directed_f32", "undirected_bf16"])
def test_cdgcn_layer_over_a_block(case):
    wl = {"undirected_f32": replace(WORKLOADS["c1"], f=32, window=0, name="cd-c1"),
          "directed_f32": replace(WORKLOADS["c3"].scaled(4096, T=5), name="cd-c3"),
          "undirected_bf16": replace(WORKLOADS["c4"].scaled(3000, T=4), f=32, window=0, name="cd-c4")}[case]
    dtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    f, hidden = wl.f, 32
    w = glorot_weight(wl, 0)
    w_x = (randn((2 * f, 4 * hidden), 11) / np.sqrt(2 * f)).to(dtype)
    w_h = (randn((hidden, 4 * hidden), 12) / np.sqrt(hidden)).to(dtype)
    bias = randn((4 * hidden,), 13) * 0.1
    blk = make_block(wl, DEV, gen_device="cpu")
    layer = CdgcnLayer(blk, w.to(DEV), w_x.to(DEV), w_h.to(DEV), bias.to(DEV), hidden)
    layer.load_first()
    got = layer.run()
    torch.cuda.synchronize()
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    h, c = np.zeros((wl.n, hidden)), np.zeros((wl.n, hidden))
    for t in range(1, wl.T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        y = oracle.cdgcn_gcn(rp, ci, to_f64(features(wl, t)), to_f64(w))
        h, c = oracle.lstm_cell(y, h, c, to_f64(w_x), to_f64(w_h), to_f64(bias))
        # every timestep adds stored tensors between the inputs and h_t (Y0, Y1, Y, the two gate halves, c, h)
        assert_close(to_f64(got[t - 1]), h, dtype, f"{case}: h_{t}", stores=7 * t)


@pytest.mark.parametrize("dtype,hidden,f_y", [(torch.float32, 32, 32), (torch.float32, 32, 64), (torch.float32, 16, 16),
                                              (torch.float32, 16, 32), (torch.bfloat16, 32, 32), (torch.bfloat16, 32, 64),
                                              (torch.bfloat16, 64, 64), (torch.bfloat16, 64, 128)])
@pytest.mark.parametrize("n", [1, 31, 32, 33, 4097, 20_011])
@pytest.mark.parametrize("with_bias", [False, True])
def test_fused_lstm_step(dtype, hidden, f_y, n, with_bias):
    assert dg.lstm_step_supported(torch.empty((1, f_y), dtype=dtype), hidden)
    y, h = randn((n, f_y), n + f_y, dtype), randn((n, hidden), n + 1, dtype)
    c = randn((n, hidden), n + 2, dtype)
    w_x = (randn((f_y, 4 * hidden), 5) / np.sqrt(f_y)).to(dtype)
    w_h = (randn((hidden, 4 * hidden), 6) / np.sqrt(hidden)).to(dtype)
    bias = randn((4 * hidden,), 7) if with_bias else None
    h_want, c_want = oracle.lstm_cell(to_f64(y), to_f64(h), to_f64(c), to_f64(w_x), to_f64(w_h),
                                      to_f64(bias) if with_bias else None)
    cd = c.to(DEV)
    hn = torch.full((n, hidden), float("nan"), dtype=dtype, device=DEV)
    dg.lstm_step(y.to(DEV), h.to(DEV), w_x.to(DEV), w_h.to(DEV), bias.to(DEV) if with_bias else None, cd, hn)
    assert_close(to_f64(cd), c_want, dtype, f"fused step: c, n={n}")
    assert_close(to_f64(hn), h_want, dtype, f"fused step: h, n={n}")


@pytest.mark.parametrize("dtype,hidden", [(torch.float32, 16), (torch.float32, 32), (torch.bfloat16, 32)])
def test_fused_lstm_step_against_the_composed_step(dtype, hidden):
    """The same step from the two dense transforms and the cell kernel: both within the storage type's bound of
    each other, over a few steps of carried state.  (hidden = 64 has no composed form: its gate pre-activations are
    256 wide, beyond the dense transform's widths.)"""
    n, f_y = 5000, 2 * hidden
    w_x = (randn((f_y, 4 * hidden), 5) / np.sqrt(f_y)).to(dtype).to(DEV)
    w_h = (randn((hidden, 4 * hidden), 6) / np.sqrt(hidden)).to(dtype).to(DEV)
    bias = (randn((4 * hidden,), 7) * 0.1).to(DEV)
    state = {}
    for fused in (True, False):
        h = torch.zeros((n, hidden), dtype=dtype, device=DEV)
        c = torch.zeros((n, hidden), dtype=dtype, device=DEV)
        for t in range(3):
            y = randn((n, f_y), 100 + t, dtype).to(DEV)
            hn = torch.empty_like(h)
            if fused:
                dg.lstm_step(y, h, w_x, w_h, bias, c, hn)
            else:
                gx = torch.empty((n, 4 * hidden), dtype=dtype, device=DEV)
                gh = torch.empty_like(gx)
                dg.feature_transform(y, w_x, gx)
                dg.feature_transform(h, w_h, gh)
                dg.lstm_cell(gx, gh, bias, c, c, hn)
            h = hn
        state[fused] = (to_f64(h), to_f64(c))
    assert_close(state[True][0], state[False][0], dtype, "fused vs composed: h", stores=9)
    assert_close(state[True][1], state[False][1], dtype, "fused vs composed: c", stores=9)


def test_fused_and_composed_layers_agree():
    wl = replace(WORKLOADS["c3"].scaled(4096, T=5), name="cd-c3")
    f, hidden = wl.f, 32
    w = glorot_weight(wl, 0).to(DEV)
    w_x = (randn((2 * f, 4 * hidden), 11) / np.sqrt(2 * f)).to(DEV)
    w_h = (randn((hidden, 4 * hidden), 12) / np.sqrt(hidden)).to(DEV)
    blk = make_block(wl, DEV, gen_device="cpu")
    outs = []
    for fused in (True, False):
        layer = CdgcnLayer(blk, w, w_x, w_h, None, hidden, fused=fused)
        layer.load_first()
        outs.append(layer.run().clone())
    assert_close(to_f64(outs[0]), to_f64(outs[1]), torch.float32, "fused vs composed layer")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("hidden", [16, 32, 128])
@pytest.mark.parametrize("carried", [False, True])
def test_lstm_cell_backward(dtype, hidden, carried):
    n = 1003
    gx, gh = randn((n, 4 * hidden), 1, dtype), randn((n, 4 * hidden), 2, dtype)
    bias = randn((4 * hidden,), 3) * 0.1
    c_prev, g_h = randn((n, hidden), 4, dtype), randn((n, hidden), 5, dtype)
    dh_c, dc_n = (randn((n, hidden), 6, dtype), randn((n, hidden), 7, dtype)) if carried else (None, None)
    da = torch.full((n, 4 * hidden), float("nan"), dtype=dtype, device=DEV)
    dc = dc_n.to(DEV) if carried else torch.full((n, hidden), float("nan"), dtype=dtype, device=DEV)
    dg.lstm_cell_backward(gx.to(DEV), gh.to(DEV), bias.to(DEV), c_prev.to(DEV), g_h.to(DEV), dh_c.to(DEV) if carried else None,
                          dc if carried else None, da, dc)            # dc_prev written over dc_next
    # the oracle's cell takes x W_x + h W_h + b: feed it the pre-activations through identity weights
    eye = np.eye(4 * hidden)
    dh = to_f64(g_h) + (to_f64(dh_c) if carried else 0.0)
    want = oracle.lstm_cell_backward(to_f64(gx) + to_f64(gh), np.zeros((n, 4 * hidden)), to_f64(c_prev), eye, eye, to_f64(bias),
                                     dh, to_f64(dc_n) if carried else None)
    assert_close(to_f64(da), want[0], dtype, "dL/d(pre-activations)")
    assert_close(to_f64(dc), want[3], dtype, "dL/dc_prev")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f0,f1", [(16, 16), (32, 128), (128, 64)])
def test_concat_relu_backward(dtype, f0, f1):
    n = 601
    dy, y = randn((n, f0 + f1), 1, dtype), randn((n, f0 + f1), 2, dtype)
    d0 = torch.full((n, f0), float("nan"), dtype=dtype, device=DEV)
    d1 = torch.full((n, f1), float("nan"), dtype=dtype, device=DEV)
    dg.concat_relu_backward(dy.to(DEV), y.to(DEV), d0, d1, f0)
    want = to_f64(dy) * (to_f64(y) > 0)
    assert np.array_equal(to_f64(d0), want[:, :f0]) and np.array_equal(to_f64(d1), want[:, f0:])     # a copy under a mask: exact
    d1.fill_(float("nan"))
    dg.concat_relu_backward(dy.to(DEV), y.to(DEV), None, d1, f0)
    assert np.array_equal(to_f64(d1), want[:, f0:])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f,n", [(128, 100_003), (64, 7), (16, 5000), (512, 3001)])
def test_bias_grad(dtype, f, n):
    g = randn((n, f), f + n, dtype)
    db = torch.full((f,), float("nan"), device=DEV)
    ws = torch.empty(dg.bias_grad_workspace(f), dtype=torch.uint8, device=DEV)
    dg.bias_grad(g.to(DEV), db, ws)
    want = to_f64(g).sum(axis=0)
    first = db.clone()
    np.testing.assert_allclose(to_f64(db), want, rtol=1e-5, atol=1e-5 * np.sqrt(n))
    dg.bias_grad(g.to(DEV), db, ws, accumulate=True)
    np.testing.assert_allclose(to_f64(db), 2 * want, rtol=1e-5, atol=2e-5 * np.sqrt(n))
    dg.bias_grad(g.to(DEV), db, ws)
    assert torch.equal(db, first)                     # fixed order of summation


@pytest.mark.parametrize("dtype,hidden,f_y", [(torch.float32, 32, 32), (torch.float32, 32, 64), (torch.bfloat16, 32, 32),
                                              (torch.bfloat16, 32, 64), (torch.float32, 16, 16), (torch.float32, 16, 32)])
@pytest.mark.parametrize("n", [1, 31, 32, 33, 4097, 20_011])
@pytest.mark.parametrize("carried", [False, True])
def test_fused_lstm_step_backward(n, carried, f_y, hidden, dtype):
    assert dg.lstm_step_backward_supported(torch.empty((1, f_y), dtype=dtype), hidden)
    y, h_prev = randn((n, f_y), 1, dtype), randn((n, hidden), 2, dtype)
    w_x, w_h = (randn((f_y, 4 * hidden), 3) / 8).to(dtype), (randn((hidden, 4 * hidden), 4) / 6).to(dtype)
    bias = randn((4 * hidden,), 5) * 0.1
    c_prev, g_h = randn((n, hidden), 6, dtype), randn((n, hidden), 7, dtype)
    dh_c, dc_n = (randn((n, hidden), 8, dtype), randn((n, hidden), 9, dtype)) if carried else (None, None)
    da = torch.full((n, 4 * hidden), float("nan"), dtype=dtype, device=DEV)
    dc = dc_n.to(DEV) if carried else torch.full((n, hidden), float("nan"), dtype=dtype, device=DEV)
    dg.lstm_step_backward(y.to(DEV), h_prev.to(DEV), w_x.to(DEV), w_h.to(DEV), bias.to(DEV), c_prev.to(DEV), g_h.to(DEV),
                          dh_c.to(DEV) if carried else None, dc if carried else None, da, dc)
    dh = to_f64(g_h) + (to_f64(dh_c) if carried else 0.0)
    want = oracle.lstm_cell_backward(to_f64(y), to_f64(h_prev), to_f64(c_prev), to_f64(w_x), to_f64(w_h), to_f64(bias), dh,
                                     to_f64(dc_n) if carried else None)
    assert_close(to_f64(da), want[0], dtype, "dL/d(pre-activations), fused")
    assert_close(to_f64(dc), want[3], dtype, "dL/dc_prev, fused")


@pytest.mark.parametrize("keep,fused", [(False, True), (True, True), (False, False)])
@pytest.mark.parametrize("case", ["undirected_f32", "directed_f32", "undirected_bf16", "undirected_f32_width16"])
def test_cdgcn_training_step(case, keep, fused):
    """Gradients of sum_t <G_t, h_t> with respect to W, W_x, W_h and b over a block, against the oracle's backward
    pass (itself pinned by finite differences); the ReLU mask is taken on fp32 values on the device and fp64 in
    the oracle, which agree except for outputs within rounding of zero (none at these sizes would move a gradient
    beyond the tolerance; the bf16 case has its own bound for dW, see below)."""
    from paper_2109_07893_amd.cdgcn import CdgcnTrainer
    wl = {"undirected_f32": replace(WORKLOADS["c1"], f=32, window=0, name="cd-c1"),
          "directed_f32": replace(WORKLOADS["c3"].scaled(4096, T=5), name="cd-c3"),
          "undirected_bf16": replace(WORKLOADS["c4"].scaled(3000, T=4), f=32, window=0, name="cd-c4"),
          "undirected_f32_width16": replace(WORKLOADS["c1"], window=0, name="cd-c1-16")}[case]      # c1's own width
    dtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    f, hidden, T = wl.f, (16 if case.endswith("width16") else 32), wl.T
    w = glorot_weight(wl, 0)
    w_x = (randn((2 * f, 4 * hidden), 11) / np.sqrt(2 * f)).to(dtype)
    w_h = (randn((hidden, 4 * hidden), 12) / np.sqrt(hidden)).to(dtype)
    bias = randn((4 * hidden,), 13) * 0.1
    g_h = randn((T, wl.n, hidden), 14, dtype)
    blk = make_block(wl, DEV, gen_device="cpu")
    tr = CdgcnTrainer(blk, w.to(DEV), w_x.to(DEV), w_h.to(DEV), bias.to(DEV), hidden, fused=fused, keep_activations=keep)
    tr.load_first()
    for _ in range(2):                                # a second step must not see leftovers of the first
        tr.forward()
        tr.backward(g_h.to(DEV))
    torch.cuda.synchronize()
    # oracle: forward keeping what the backward needs, then backward
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    snaps, ys, hs, cs = [], [], [np.zeros((wl.n, hidden))], [np.zeros((wl.n, hidden))]
    W, WX, WH, Bv = to_f64(w), to_f64(w_x), to_f64(w_h), to_f64(bias)
    for t in range(1, T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        snaps.append((rp, ci))
        ys.append(oracle.cdgcn_gcn(rp, ci, to_f64(features(wl, t)), W))
        h, c = oracle.lstm_cell(ys[-1], hs[-1], cs[-1], WX, WH, Bv)
        hs.append(h); cs.append(c)
        assert_close(to_f64(tr.h_all[t - 1]), h, dtype, f"{case}: h_{t}", stores=7 * t)
    d_w, d_wx, d_wh, d_b = 0.0, 0.0, 0.0, 0.0
    dh, dc = 0.0, None
    for t in range(T, 0, -1):
        _, d_y, dh, dc, a, b, cgrad = oracle.lstm_cell_backward(ys[t - 1], hs[t - 1], cs[t - 1], WX, WH, Bv,
                                                                to_f64(g_h[t - 1]) + dh, dc)
        d_wx, d_wh, d_b = d_wx + a, d_wh + b, d_b + cgrad
        d_w = d_w + oracle.cdgcn_gcn_backward(*snaps[t - 1], to_f64(features(wl, t)), W, d_y)[0]
    bad = []
    for name, got, want in (("dW", tr.dw, d_w), ("dW_x", tr.dw_x, d_wx), ("dW_h", tr.dw_h, d_wh), ("db", tr.db, d_b)):
        want = np.asarray(want)
        err = np.abs(to_f64(got) - want).max()
        # bf16: every gradient is a sum over thousands of vertices of products of values that were each rounded to 8 bits
        # several times on the way; the roundings are independent, so the sums keep two to three digits (measured:
        # 3e-3 of the largest entry).  dW is another matter: Y0 is stored in bf16, so Y1 = Y0 W has the other sign than
        # the oracle's wherever |Y1| is below that rounding, about 3 in 1000 entries, and each such ReLU mask bit
        # changes its term of Y0^T dY1 by 100 %: sqrt(0.003) = 5 % of a sum of terms with random signs
        tol = 2e-4 if dtype == torch.float32 else (8e-2 if name == "dW" else 2e-2)
        if err > tol * np.abs(want).max():
            bad.append(f"{name}: max err {err:.3e} against max |.| {np.abs(want).max():.3e}")
    assert not bad, f"{case}: " + "; ".join(bad)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_add(dtype):
    n, f = 999, 64
    a, b = randn((n, f), 1, dtype), randn((n, f), 2, dtype)
    out = a.to(DEV).clone()
    dg.add(out, b.to(DEV), out)                          # in place
    want = (a.to(torch.float32) + b.to(torch.float32)).to(dtype)
    assert torch.equal(out.cpu(), want)                  # one fp32 sum, rounded once


@pytest.mark.parametrize("case,keep", [("undirected_f32", False), ("directed_f32", False), ("directed_f32", True)])
def test_two_layer_cdgcn_training_step(case, keep):
    """The two-layer CD-GCN the paper trains (Section "CD-GCN"): the second layer's input is the first layer's h_t,
    so its backward pass has to deliver dL/dX_t = A~_t^T (dY0 + dY1 W^T), which becomes the first layer's dL/dh_t.
    Parameter gradients of both layers against the oracle's chain."""
    from dtdg_synth import transpose_coo
    from paper_2109_07893_amd.cdgcn import CdgcnTrainer
    from paper_2109_07893_amd.pipeline import BlockInputs
    wl = {"undirected_f32": replace(WORKLOADS["c1"], f=32, window=0, name="cd-c1"),
          "directed_f32": replace(WORKLOADS["c3"].scaled(4096, T=4), name="cd-c3")}[case]
    f, hidden, T, n = wl.f, 32, wl.T, wl.n
    par = []
    for layer, f_in in enumerate((f, hidden)):
        par.append((randn((f_in, f_in), 20 + layer) / np.sqrt(f_in), randn((2 * f_in, 4 * hidden), 30 + layer) / np.sqrt(2 * f_in),
                    randn((hidden, 4 * hidden), 40 + layer) / np.sqrt(hidden), randn((4 * hidden,), 50 + layer) * 0.1))
    g_h = randn((T, n, hidden), 60)
    blk = make_block(wl, DEV, gen_device="cpu")
    l1 = CdgcnTrainer(blk, *[p.to(DEV) for p in par[0]], hidden, keep_activations=keep)
    blk2 = BlockInputs(n=n, T=T, f=hidden, layers=1, window=0, rowptr1=blk.rowptr1, colidx1=blk.colidx1, deltas=blk.deltas,
                       x=[l1.h_all[t] for t in range(T)], w=[par[1][0].to(DEV)], nnz=list(blk.nnz))
    kw = {}
    if wl.graph != "er":                                  # directed: the transposed first snapshot and lists
        rows = torch.repeat_interleave(torch.arange(n, dtype=torch.int32, device=DEV), (blk.rowptr1[1:] - blk.rowptr1[:-1]).to(torch.int64))
        tr_, tc_ = transpose_coo(rows, blk.colidx1)
        rp_t = torch.zeros(n + 1, dtype=torch.int32, device=DEV)
        rp_t[1:] = torch.cumsum(torch.bincount(tr_.to(torch.int64), minlength=n), 0).to(torch.int32)
        kw = dict(transposed_first=(rp_t, tc_), transposed_deltas=[transpose_coo(ar, ac) + transpose_coo(dr, dc) for ar, ac, dr, dc in blk.deltas])
    l2 = CdgcnTrainer(blk2, *[p.to(DEV) for p in par[1]], hidden, keep_activations=keep, want_dx=True, **kw)
    l1.load_first(); l2.load_first()
    for _ in range(2):
        l1.forward(); l2.forward()
        l2.backward(g_h.to(DEV))
        l1.backward(l2.dx)
    torch.cuda.synchronize()
    # oracle: forward of both layers, then backward
    P = [[to_f64(p) for p in layer] for layer in par]
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    snaps = []
    xs = [[None] * T, [None] * T]
    ys = [[None] * T, [None] * T]
    hs = [[np.zeros((n, hidden))], [np.zeros((n, hidden))]]
    cs = [[np.zeros((n, hidden))], [np.zeros((n, hidden))]]
    for t in range(1, T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(n, rp, ci, *[x.numpy() for x in g.advance()])
        snaps.append((rp, ci))
        x = to_f64(features(wl, t))
        for layer in range(2):
            W, WX, WH, Bv = P[layer]
            xs[layer][t - 1] = x
            ys[layer][t - 1] = oracle.cdgcn_gcn(rp, ci, x, W)
            h, c = oracle.lstm_cell(ys[layer][t - 1], hs[layer][-1], cs[layer][-1], WX, WH, Bv)
            hs[layer].append(h); cs[layer].append(c)
            x = h
    assert_close(to_f64(l2.h_all[T - 1]), hs[1][T], torch.float32, "second layer's h_T")
    grads = [None, None]
    upstream = [to_f64(g_h[t]) for t in range(T)]
    for layer in (1, 0):
        W, WX, WH, Bv = P[layer]
        d_w = d_wx = d_wh = d_b = 0.0
        dh, dc = 0.0, None
        d_x_all = [None] * T
        for t in range(T, 0, -1):
            _, d_y, dh, dc, a, b, cg = oracle.lstm_cell_backward(ys[layer][t - 1], hs[layer][t - 1], cs[layer][t - 1], WX, WH, Bv,
                                                                 upstream[t - 1] + dh, dc)
            d_wx, d_wh, d_b = d_wx + a, d_wh + b, d_b + cg
            dw_t, d_x_all[t - 1] = oracle.cdgcn_gcn_backward(*snaps[t - 1], xs[layer][t - 1], W, d_y)
            d_w = d_w + dw_t
        grads[layer] = (d_w, d_wx, d_wh, d_b)
        upstream = d_x_all
    for layer, tr in enumerate((l1, l2)):
        for name, got, want in zip(("dW", "dW_x", "dW_h", "db"), (tr.dw, tr.dw_x, tr.dw_h, tr.db), grads[layer]):
            err = np.abs(to_f64(got) - want).max()
            assert err <= 3e-4 * np.abs(want).max(), f"{case} layer {layer + 1} {name}: max err {err:.3e} against max |.| {np.abs(want).max():.3e}"
