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
from paper_2109_07893_amd.pipeline import make_block

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


@pytest.mark.parametrize("f_y", [32, 64])
@pytest.mark.parametrize("n", [1, 31, 32, 33, 4097, 20_011])
@pytest.mark.parametrize("with_bias", [False, True])
def test_fused_lstm_step(f_y, n, with_bias):
    hidden = 32
    y, h = randn((n, f_y), n + f_y), randn((n, hidden), n + 1)
    c = randn((n, hidden), n + 2)
    w_x = randn((f_y, 4 * hidden), 5) / np.sqrt(f_y)
    w_h = randn((hidden, 4 * hidden), 6) / np.sqrt(hidden)
    bias = randn((4 * hidden,), 7) if with_bias else None
    h_want, c_want = oracle.lstm_cell(to_f64(y), to_f64(h), to_f64(c), to_f64(w_x), to_f64(w_h),
                                      to_f64(bias) if with_bias else None)
    cd = c.to(DEV)
    hn = torch.full((n, hidden), float("nan"), device=DEV)
    dg.lstm_step(y.to(DEV), h.to(DEV), w_x.to(DEV), w_h.to(DEV), bias.to(DEV) if with_bias else None, cd, hn)
    assert_close(to_f64(cd), c_want, torch.float32, f"fused step: c, n={n}")
    assert_close(to_f64(hn), h_want, torch.float32, f"fused step: h, n={n}")


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
