"""GPU parity of the backward entry points (gradient propagation through a block, Section "Gradient
Checkpoint") against the CPU oracle's adjoints, kernel by kernel, on seeded inputs that span several tiles
and a ragged tail."""
import numpy as np
import pytest
import torch

import oracle
import paper_2109_07893_amd as dg
from helpers import assert_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
WIDTHS = [16, 32, 64, 128]


def randn(shape, seed, dtype=torch.float32):
    return torch.randn(shape, generator=torch.Generator().manual_seed(seed)).to(dtype)


# ------------------------------------------------------------------------------- G x_1 M^T
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,w", [(8, 3), (32, 8), (5, 1), (6, 9), (40, 16), (3, 32), (33, 32), (7, 4)])
def test_mproduct_backward_paper_weights(dtype, T, w):
    n, f = 333, 32
    g = randn((T, n, f), T * 100 + w + 7, dtype)
    expect = oracle.mproduct_t(to_f64(g), oracle.m_matrix(T, w))
    gd = g.to(DEV)
    out = torch.full_like(gd, float("nan"))
    dg.mproduct_backward(gd, out, w)
    assert_close(to_f64(out), expect, dtype, f"mproduct_backward T={T} w={w}")
    assert torch.equal(gd.cpu(), g)                                      # input untouched out of place
    dg.mproduct_backward(gd, gd, w)                                      # in place
    torch.cuda.synchronize()
    assert torch.equal(gd, out)


def test_mproduct_backward_explicit_band():
    T, w, n, f = 12, 4, 100, 16
    gen = torch.Generator().manual_seed(5)
    g = torch.randn((T, n, f), generator=gen)
    band = torch.randn((T, w), generator=gen)
    M = np.zeros((T, T))
    for t in range(T):
        for j in range(min(w, t + 1)):
            M[t, t - j] = float(band[t, j])
    out = torch.empty((T, n, f), device=DEV)
    dg.mproduct_backward(g.to(DEV), out, w, m_band=band.to(DEV))
    assert_close(to_f64(out), oracle.mproduct_t(to_f64(g), M), torch.float32, "explicit band, adjoint")


def test_mproduct_backward_is_adjoint_of_forward_on_gpu():
    T, w, n, f = 20, 6, 257, 16
    z, g = randn((T, n, f), 1).to(DEV), randn((T, n, f), 2).to(DEV)
    y, gz = torch.empty_like(z), torch.empty_like(g)
    dg.mproduct(z, y, w)
    dg.mproduct_backward(g, gz, w)
    lhs, rhs = float((gz.double() * z.double()).sum()), float((g.double() * y.double()).sum())
    assert abs(lhs - rhs) <= 1e-5 * (abs(lhs) + abs(rhs) + 1.0)


# ------------------------------------------------------------------------------- ReLU mask
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f", WIDTHS)
@pytest.mark.parametrize("scaled", [False, True])
def test_relu_backward(dtype, f, scaled):
    n = 1237
    g = randn((n, f), 10 + f, dtype)
    z = torch.relu(randn((n, f), 20 + f, dtype))
    z[5, :] = 0.0
    z[7, 0] = -0.0
    scale = (torch.rand(n, generator=torch.Generator().manual_seed(3)) + 0.5) if scaled else None
    expect = oracle.relu_grad(to_f64(g), to_f64(z))
    if scaled:
        expect = expect * to_f64(scale)[:, None]
    gd = g.to(DEV)
    out = torch.full_like(gd, float("nan"))
    dg.relu_backward(gd, z.to(DEV), out, row_scale=scale.to(DEV) if scaled else None)
    assert_close(to_f64(out), expect, dtype, f"relu_backward f={f}")
    if not scaled:
        assert np.array_equal(to_f64(out) != 0, (to_f64(z) > 0) & (to_f64(g) != 0))   # the mask itself is exact
    dg.relu_backward(gd, z.to(DEV), gd, row_scale=scale.to(DEV) if scaled else None)  # in place
    torch.cuda.synchronize()
    assert torch.equal(gd, out)


# ------------------------------------------------------------------------------- X^T G
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f_in", WIDTHS)
@pytest.mark.parametrize("f_out", WIDTHS)
def test_weight_grad_all_widths(dtype, f_in, f_out):
    n = 2000 + 13                                   # several 16-row steps per worker and a ragged last step
    x = randn((n, f_in), f_in * 7 + f_out, dtype)
    g = randn((n, f_out), f_in * 11 + f_out, dtype)
    expect = oracle.weight_grad(to_f64(x), to_f64(g))
    ws = torch.empty(dg.weight_grad_workspace(f_in, f_out), dtype=torch.uint8, device=DEV)
    dw = torch.full((f_in, f_out), float("nan"), device=DEV)
    dg.weight_grad(x.to(DEV), g.to(DEV), dw, ws)
    # inputs are exact in either storage type and products accumulate in fp32: the fp32 bound applies to both
    assert_close(to_f64(dw), expect, torch.float32, f"weight_grad {f_in}x{f_out} {dtype}")
    first = dw.clone()
    dg.weight_grad(x.to(DEV), g.to(DEV), dw, ws, accumulate=True)
    assert_close(to_f64(dw), 2 * expect, torch.float32, "accumulate")
    dg.weight_grad(x.to(DEV), g.to(DEV), dw, ws)
    torch.cuda.synchronize()
    assert torch.equal(dw, first)                    # fixed summation order: bit-identical repeats


@pytest.mark.parametrize("n", [1, 15, 16, 17, 100_003])
def test_weight_grad_row_counts(n):
    x, g = randn((n, 32), n), randn((n, 64), n + 1)
    ws = torch.empty(dg.weight_grad_workspace(32, 64), dtype=torch.uint8, device=DEV)
    dw = torch.empty((32, 64), device=DEV)
    dg.weight_grad(x.to(DEV), g.to(DEV), dw, ws)
    assert_close(to_f64(dw), oracle.weight_grad(to_f64(x), to_f64(g)), torch.float32, f"weight_grad n={n}")


# ------------------------------------------------------------------------------- G W^T
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f_in", WIDTHS)
@pytest.mark.parametrize("f_out", WIDTHS)
def test_input_grad_all_widths(dtype, f_in, f_out):
    n = 1000 + 7
    g = randn((n, f_out), f_in * 13 + f_out, dtype)
    w = (randn((f_in, f_out), f_in * 17 + f_out) / np.sqrt(f_out)).to(dtype)
    expect = oracle.input_grad(to_f64(g), to_f64(w))
    dx = torch.full((n, f_in), float("nan"), dtype=dtype, device=DEV)
    dg.input_grad(g.to(DEV), w.to(DEV), dx)
    assert_close(to_f64(dx), expect, dtype, f"input_grad {f_in}x{f_out}")


# ------------------------------------------------------------------------------- A~^T G through dgnn_spmm
def _transpose_csr(n, rp, ci):
    rows = np.repeat(np.arange(n, dtype=np.int32), np.diff(rp))
    return oracle.csr_from_edges(n, ci, rows)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("prescaled", [False, True])
def test_transposed_aggregation_on_a_directed_graph(dtype, prescaled):
    n, f = 3000, 32
    rng = np.random.default_rng(6)
    m = 40_000
    src = (rng.random(m) ** 2 * n).astype(np.int32)               # skewed sources: long rows and long columns differ
    dst = rng.integers(0, n, m).astype(np.int32)
    rp, ci = oracle.csr_from_edges(n, np.concatenate([src, np.arange(n, dtype=np.int32)]),
                                   np.concatenate([dst, np.arange(n, dtype=np.int32)]))
    rpt, cit = _transpose_csr(n, rp, ci)
    g = randn((n, f), 8, dtype)
    expect = oracle.spmm_t(rp, ci, to_f64(g))
    dinv = torch.empty(n, device=DEV)
    dg.csr_dinv(torch.as_tensor(rp).to(DEV), dinv)                 # of A, not of its transpose
    rpt_d, cit_d = torch.as_tensor(rpt).to(DEV), torch.as_tensor(cit).to(DEV)
    ws = torch.empty(dg.spmm_workspace(n, int(cit.size), f), dtype=torch.uint8, device=DEV)
    gd = g.to(DEV)
    out = torch.full_like(gd, float("nan"))
    if prescaled:
        z_all_positive = torch.ones_like(gd)
        gs = torch.empty_like(gd)
        dg.relu_backward(gd, z_all_positive, gs, row_scale=dinv)
        dg.spmm(rpt_d, cit_d, int(cit.size), dinv, gs, out, ws, flags=dg.DGNN_H_PRESCALED)
    else:
        dg.spmm(rpt_d, cit_d, int(cit.size), dinv, gd, out, ws)
    assert_close(to_f64(out), expect, dtype, "A~^T G")


# ------------------------------------------------------------------------------- M-transform block by block
def _band_matrix(band, T, w):
    M = np.zeros((T, T))
    for t in range(T):
        for j in range(min(w, t + 1)):
            M[t, t - j] = float(band[t, j])
    return M


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,w,cuts", [(20, 6, [7, 13]), (12, 5, [2, 3, 4]), (9, 12, [4]), (40, 16, [16, 17, 39]),
                                       (10, 1, [5]), (33, 32, [1, 32])])
@pytest.mark.parametrize("explicit_band", [False, True])
def test_mproduct_in_blocks_equals_whole_series(dtype, T, w, cuts, explicit_band):
    """Forward with the frames before each block handed over, adjoint with the gradient frames after it: the
    pieces must be the frames of the transform of the whole series."""
    n, f = 130, 16
    z, g = randn((T, n, f), 31 * T + w, dtype), randn((T, n, f), 37 * T + w, dtype)
    if explicit_band:
        band = randn((T, w), 41 * T + w)
        M = _band_matrix(band, T, w)
    else:
        band, M = None, oracle.m_matrix(T, w)
    y_want, gz_want = oracle.mproduct(to_f64(z), M), oracle.mproduct_t(to_f64(g), M)
    zd, gd = z.to(DEV), g.to(DEV)
    y, gz = torch.full_like(zd, float("nan")), torch.full_like(gd, float("nan"))
    bounds = [0] + cuts + [T]
    for a, b in zip(bounds[:-1], bounds[1:]):
        nb = min(w - 1, a)
        na = min(w - 1, T - b)
        fb = band[a:b].contiguous().to(DEV) if explicit_band else None
        bb = band[a:b + na].contiguous().to(DEV) if explicit_band else None
        dg.mproduct_block(zd[a:b], y[a:b], w, a, z_before=zd[a - nb:a] if nb else None, m_band=fb)
        dg.mproduct_backward_block(gd[a:b], gz[a:b], w, a, g_after=gd[b:b + na] if na else None, m_band=bb)
    assert_close(to_f64(y), y_want, dtype, f"blocks forward T={T} w={w}")
    assert_close(to_f64(gz), gz_want, dtype, f"blocks adjoint T={T} w={w}")
    if not explicit_band:     # and bit for bit what the one-call transform gives
        y1, gz1 = torch.empty_like(zd), torch.empty_like(gd)
        dg.mproduct(zd, y1, w)
        dg.mproduct_backward(gd, gz1, w)
        assert_close(to_f64(y), to_f64(y1), dtype, "blocks vs one call")
        assert_close(to_f64(gz), to_f64(gz1), dtype, "blocks vs one call, adjoint")


def test_mproduct_block_argument_checks():
    z = torch.zeros((4, 10, 16), device=DEV)
    with pytest.raises(dg.DgnnError):      # three timesteps before the block, window 3: two frames must come along
        dg.mproduct_block(z, torch.empty_like(z), 3, 3, z_before=z[:1])
    with pytest.raises(dg.DgnnError):      # more gradient frames than the window reaches
        dg.mproduct_backward_block(z, torch.empty_like(z), 3, 0, g_after=torch.zeros((3, 10, 16), device=DEV))
