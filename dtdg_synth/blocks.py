"""Harness glue: a workload of the seeded generator laid out as the inputs of one block of timesteps on a device (the
first snapshot whole, the difference lists of the later ones, feature frames, weights).  Used by the tests, the
benchmark and the smoke check; the library and its Python package do not depend on it."""
from __future__ import annotations

from typing import Optional

import torch

from . import DynamicGraph, features, glorot_weight


def make_block(wl, device, gen_device=None, pinned: bool = False, T: Optional[int] = None, repeat_features: bool = False,
               progress=None) -> BlockInputs:
    """Generate a workload's block with the seeded generator and place it on `device`.  repeat_features: every
    timestep gets the frame of the first one (one frame in memory; for runs that only count bytes).  progress: called
    with a line of text now and then (a long generation on the host must not look hung)."""
    from paper_2109_07893_amd.pipeline import BlockInputs
    gen_device = torch.device(gen_device if gen_device is not None else device)
    T = T or wl.T
    g = DynamicGraph(wl, device=gen_device)
    rowptr1, colidx1 = (t.to(device) for t in g.csr())
    deltas, pins = [], []
    for t in range(2, T + 1):
        d = g.advance()
        deltas.append(tuple(t.to(device) for t in d))
        if pinned:
            pins.append(tuple(torch.empty(t.shape, dtype=t.dtype, pin_memory=True).copy_(t) for t in d))
        if progress is not None and t % 16 == 0:
            progress(f"snapshot {t} of {T} generated")
    if repeat_features:
        x = [features(wl, 1, device=gen_device).to(device)] * T
    else:
        x = [features(wl, t, device=gen_device).to(device) for t in range(1, T + 1)]
    w = [glorot_weight(wl, layer, device=gen_device).to(device) for layer in range(wl.layers)]
    return BlockInputs(n=wl.n, T=T, f=wl.f, layers=wl.layers, window=wl.window, rowptr1=rowptr1,
                       colidx1=colidx1, deltas=deltas, x=x, w=w, pinned=pins if pinned else None)
