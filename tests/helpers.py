"""Shared by the GPU parity tests: tolerance form and an oracle run of a whole block."""
import numpy as np
import torch

import oracle
from dtdg_synth import DynamicGraph, features, glorot_weight

RTOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


def assert_close(got, expect, dtype, what="", stores=1):
    """|g - o| <= rtol |o| + rtol rms(o), rtol = 1e-4 for fp32 storage, 2e-2 for bf16 storage.
    (Purely relative error is meaningless next to the zeros ReLU produces.)  The bound is the one for a
    result that was rounded to its storage type once; a bf16 result that has passed through `stores`
    consecutive bf16 tensors carries that many independent roundings and gets sqrt(stores) times the bound."""
    got = np.asarray(got, dtype=np.float64)
    expect = np.asarray(expect, dtype=np.float64)
    assert got.shape == expect.shape, (what, got.shape, expect.shape)
    rtol = RTOL[dtype] * (float(stores) ** 0.5 if dtype == torch.bfloat16 else 1.0)
    rms = float(np.sqrt(np.mean(expect ** 2))) if expect.size else 0.0
    err = np.abs(got - expect)
    bound = rtol * np.abs(expect) + rtol * rms
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} outside tolerance, max err {err.max():.3e}, rms {rms:.3e}"


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_block(wl, T=None, rows=None):
    """Oracle forward pass over a block: yields per t (rowptr, colidx, Z_t) with Z_t the output of
    the last GCN layer (all rows, float64); the M-transform is left to the caller."""
    T = T or wl.T
    g = DynamicGraph(wl)
    rp, ci = (x.numpy() for x in g.csr())
    ws = [to_f64(glorot_weight(wl, layer)) for layer in range(wl.layers)]
    for t in range(1, T + 1):
        if t > 1:
            rp, ci = oracle.delta_apply(wl.n, rp, ci, *[x.numpy() for x in g.advance()])
        cur = to_f64(features(wl, t))
        val = oracle.gcn_values(rp, ci)
        for layer in range(wl.layers):
            cur = oracle.spmm(rp, ci, oracle.xw(cur, ws[layer]), relu=True, val=val)
        yield rp, ci, cur
