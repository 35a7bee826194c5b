"""ctypes binding of libdgnn (include/dgnn.h).  Same names as the C entry points, argument
marshalling only: tensors become device pointers, the current torch stream becomes the
hipStream_t, and a non-zero status becomes a DgnnError."""
from __future__ import annotations

import ctypes
import glob
import os
import subprocess
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_CSRC = os.path.join(_HERE, "csrc")
_LIB_PATH = os.path.join(_CSRC, "libdgnn.so")

DGNN_F32, DGNN_BF16 = 0, 1
DGNN_VALIDATE = 1
DGNN_UPDATES_SORTED = 2
DGNN_RELU = 1
DGNN_H_PRESCALED = 2

EXPORTS = (
    "dgnn_strerror", "dgnn_csr_validate", "dgnn_csr_dinv", "dgnn_delta_h2d", "dgnn_delta_rebuild_workspace",
    "dgnn_delta_rebuild", "dgnn_feature_transform", "dgnn_spmm_workspace", "dgnn_spmm", "dgnn_spmm_static_limit",
    "dgnn_spmm_static", "dgnn_mproduct",
    "dgnn_delta_rebuild_weighted", "dgnn_spmm_weighted", "dgnn_csr_combine_workspace", "dgnn_csr_combine", "dgnn_csr_weighted_dinv_workspace", "dgnn_csr_weighted_dinv", "dgnn_concat_relu", "dgnn_transform_concat_relu", "dgnn_lstm_cell", "dgnn_lstm_step", "dgnn_lstm_cell_backward", "dgnn_lstm_step_backward", "dgnn_concat_relu_backward", "dgnn_bias_grad_workspace", "dgnn_bias_grad", "dgnn_add",
    "dgnn_csr_transpose_workspace", "dgnn_csr_transpose", "dgnn_coo_transpose_workspace", "dgnn_coo_transpose",
    "dgnn_mproduct_backward", "dgnn_mproduct_block", "dgnn_mproduct_backward_block", "dgnn_relu_backward", "dgnn_weight_grad_workspace", "dgnn_weight_grad", "dgnn_input_grad",
)


class DgnnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def library_path() -> str:
    return _LIB_PATH


def build_library(verbose: bool = False) -> str:
    """Compile csrc/*.hip for gfx950 into csrc/libdgnn.so with hipcc (cross-compiles without a GPU): one object per
    source, compiled side by side, then one link."""
    from concurrent.futures import ThreadPoolExecutor
    srcs = sorted(glob.glob(os.path.join(_CSRC, "*.hip")))
    objdir = os.path.join(_CSRC, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(_ROOT, "include"), "-I", _CSRC]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        return obj, subprocess.run(["hipcc", "-c"] + flags + ["-o", obj, src], capture_output=True, text=True)

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        results = list(pool.map(compile_one, srcs))
    for obj, res in results:
        if verbose or res.returncode != 0:
            print(res.stdout)
            print(res.stderr)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed compiling {obj}")
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", _LIB_PATH] + [o for o, _ in results],
                         capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking libdgnn.so")
    return _LIB_PATH


_lib = None
_vp, _i64, _i32, _u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32
_sz = ctypes.c_size_t


def load_library():
    """Load the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(or paper_2109_07893_amd.build_library()) first; there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.dgnn_strerror.restype = ctypes.c_char_p
    lib.dgnn_strerror.argtypes = [ctypes.c_int]
    lib.dgnn_csr_dinv.argtypes = [_i64, _vp, _vp, _vp]
    lib.dgnn_delta_h2d.argtypes = [_vp, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp]
    lib.dgnn_delta_rebuild_workspace.argtypes = [_i64, _i64, _i64, _i64, ctypes.POINTER(_sz)]
    lib.dgnn_delta_rebuild.argtypes = [_i64, _vp, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _i64,
                                       _vp, _vp, _i64, ctypes.POINTER(_i64), _vp, _vp, _sz, _u32, _vp, _vp]
    lib.dgnn_feature_transform.argtypes = [_vp, _i64, _i32, _vp, _i32, _vp, _vp, ctypes.c_int, _vp]
    lib.dgnn_spmm_workspace.argtypes = [_i64, _i64, _i32, ctypes.POINTER(_sz)]
    lib.dgnn_spmm.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _i32, _vp, ctypes.c_int, _u32, _vp, _sz, _vp]
    lib.dgnn_spmm_static_limit.argtypes = [ctypes.POINTER(_sz)]
    lib.dgnn_spmm_static.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _i32, _vp, ctypes.c_int, _u32, _vp]
    lib.dgnn_mproduct.argtypes = [_vp, _vp, _i64, _i64, _i32, _i32, _vp, ctypes.c_int, _vp]
    lib.dgnn_mproduct_backward.argtypes = [_vp, _vp, _i64, _i64, _i32, _i32, _vp, ctypes.c_int, _vp]
    lib.dgnn_delta_rebuild_weighted.argtypes = [_i64, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _i64,
                                                _vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, ctypes.POINTER(_i64),
                                                _vp, _sz, _u32, _vp, _vp]
    lib.dgnn_spmm_weighted.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _i32, _vp, ctypes.c_int, _u32, _vp, _sz, _vp]
    lib.dgnn_csr_validate.argtypes = [_i64, _vp, _vp, _i64, ctypes.c_int, _vp, _vp]
    lib.dgnn_csr_combine_workspace.argtypes = [_i64, ctypes.POINTER(_sz)]
    lib.dgnn_csr_combine.argtypes = [_i64, _vp, _vp, _vp, _i64, _vp, _vp, _i64, ctypes.c_float, _vp, _vp, _i64, ctypes.c_float,
                                     ctypes.c_float, _vp, _vp, _vp, _i64, _vp, _vp, _sz, _vp]
    lib.dgnn_csr_weighted_dinv_workspace.argtypes = [_i64, ctypes.POINTER(_sz)]
    lib.dgnn_csr_weighted_dinv.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.dgnn_csr_transpose_workspace.argtypes = [_i64, _i64, ctypes.c_int, ctypes.POINTER(_sz)]
    lib.dgnn_csr_transpose.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.dgnn_coo_transpose_workspace.argtypes = [_i64, _i64, ctypes.POINTER(_sz)]
    lib.dgnn_coo_transpose.argtypes = [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.dgnn_concat_relu.argtypes = [_vp, _i32, _vp, _i32, _vp, _i64, ctypes.c_int, _vp]
    lib.dgnn_transform_concat_relu.argtypes = [_vp, _i64, _i32, _vp, _i32, _vp, ctypes.c_int, _vp]
    lib.dgnn_lstm_cell.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, ctypes.c_int, _vp]
    lib.dgnn_lstm_cell_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, ctypes.c_int, _vp]
    lib.dgnn_lstm_step_backward.argtypes = [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, ctypes.c_int, _vp]
    lib.dgnn_concat_relu_backward.argtypes = [_vp, _vp, _vp, _i32, _vp, _i32, _i64, ctypes.c_int, _vp]
    lib.dgnn_bias_grad_workspace.argtypes = [_i32, ctypes.POINTER(_sz)]
    lib.dgnn_bias_grad.argtypes = [_vp, _i64, _i32, _vp, ctypes.c_int, ctypes.c_int, _vp, _sz, _vp]
    lib.dgnn_add.argtypes = [_vp, _vp, _vp, _i64, _i32, ctypes.c_int, _vp]
    lib.dgnn_lstm_step.argtypes = [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i32, ctypes.c_int, _vp]
    lib.dgnn_mproduct_block.argtypes = [_vp, _vp, _i64, _i64, _i32, _i32, _vp, _i64, _vp, _i64, ctypes.c_int, _vp]
    lib.dgnn_mproduct_backward_block.argtypes = [_vp, _vp, _i64, _i64, _i32, _i32, _vp, _i64, _vp, _i64, ctypes.c_int, _vp]
    lib.dgnn_relu_backward.argtypes = [_vp, _vp, _vp, _vp, _i64, _i32, ctypes.c_int, _vp]
    lib.dgnn_weight_grad_workspace.argtypes = [_i32, _i32, ctypes.POINTER(_sz)]
    lib.dgnn_weight_grad.argtypes = [_vp, _vp, _i64, _i32, _i32, _vp, _i32, ctypes.c_int, _vp, _sz, _vp]
    lib.dgnn_input_grad.argtypes = [_vp, _i64, _i32, _vp, _i32, _vp, _vp, ctypes.c_int, _vp]
    for name in EXPORTS:
        if name != "dgnn_strerror":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().dgnn_strerror(int(code)).decode()


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise DgnnError(rc, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "dgnn takes contiguous tensors"
    return t.data_ptr() if t.numel() > 0 else None


def _stream(t: torch.Tensor) -> Optional[int]:
    return torch.cuda.current_stream(t.device).cuda_stream if t.is_cuda else None


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DGNN_F32
    if t.dtype == torch.bfloat16:
        return DGNN_BF16
    raise TypeError(f"dgnn feature tensors are float32 or bfloat16, not {t.dtype}")


def _need(t: torch.Tensor, dtype, name: str) -> None:
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")


def csr_dinv(rowptr: torch.Tensor, dinv: torch.Tensor) -> None:
    _need(rowptr, torch.int32, "rowptr"); _need(dinv, torch.float32, "dinv")
    n = rowptr.numel() - 1
    _check(load_library().dgnn_csr_dinv(n, _ptr(rowptr), _ptr(dinv), _stream(rowptr)), "dgnn_csr_dinv")


def delta_h2d(h_add_row, h_add_col, h_del_row, h_del_col, d_add_row, d_add_col, d_del_row, d_del_col) -> None:
    """Pinned-host index lists -> device staging, asynchronously on the current stream."""
    for t in (h_add_row, h_add_col, h_del_row, h_del_col):
        _need(t, torch.int32, "difference list")
        if t.numel() and not t.is_pinned():
            raise ValueError("host difference lists must live in pinned memory")
    n_add, n_del = h_add_row.numel(), h_del_row.numel()
    assert d_add_row.numel() >= n_add and d_add_col.numel() >= n_add
    assert d_del_row.numel() >= n_del and d_del_col.numel() >= n_del
    _check(load_library().dgnn_delta_h2d(_ptr(h_add_row), _ptr(h_add_col), n_add, _ptr(h_del_row), _ptr(h_del_col),
                                         n_del, _ptr(d_add_row), _ptr(d_add_col), _ptr(d_del_row), _ptr(d_del_col),
                                         _stream(d_add_row)), "dgnn_delta_h2d")


def delta_rebuild_workspace(n: int, nnz_prev: int, n_add: int, n_del: int) -> int:
    out = _sz(0)
    _check(load_library().dgnn_delta_rebuild_workspace(n, nnz_prev, n_add, n_del, ctypes.byref(out)),
           "dgnn_delta_rebuild_workspace")
    return int(out.value)


def delta_rebuild(rowptr_prev, colidx_prev, nnz_prev: int, add_row, add_col, n_add: int, del_row, del_col, n_del: int,
                  rowptr_next, colidx_next, dinv_next, ws, flags: int = 0, d_status=None) -> int:
    """A_next = (A_prev minus deleted) plus added; returns nnz of A_next."""
    for t, name in ((rowptr_prev, "rowptr_prev"), (colidx_prev, "colidx_prev"), (rowptr_next, "rowptr_next"),
                    (colidx_next, "colidx_next")):
        _need(t, torch.int32, name)
    n = rowptr_prev.numel() - 1
    if rowptr_next.numel() < n + 1:
        raise DgnnError(-3, "dgnn_delta_rebuild (rowptr_next)")
    nnz_next = _i64(0)
    rc = load_library().dgnn_delta_rebuild(
        n, _ptr(rowptr_prev), _ptr(colidx_prev), nnz_prev, _ptr(add_row), _ptr(add_col), n_add,
        _ptr(del_row), _ptr(del_col), n_del, _ptr(rowptr_next), _ptr(colidx_next), colidx_next.numel(),
        ctypes.byref(nnz_next), _ptr(dinv_next), _ptr(ws), ws.numel() * ws.element_size(), flags,
        _ptr(d_status), _stream(rowptr_prev))
    _check(rc, "dgnn_delta_rebuild")
    return int(nnz_next.value)


def feature_transform(x: torch.Tensor, w: torch.Tensor, h: torch.Tensor, row_scale: Optional[torch.Tensor] = None) -> None:
    """H = X W, or diag(row_scale) X W."""
    dt = _dtype_code(x)
    if w.dtype != x.dtype or h.dtype != x.dtype:
        raise TypeError("x, w, h must share one dtype")
    n, f_in = x.shape
    f_out = w.shape[1]
    if w.shape[0] != f_in or tuple(h.shape) != (n, f_out):
        raise ValueError("shape mismatch in feature_transform")
    if row_scale is not None:
        _need(row_scale, torch.float32, "row_scale")
        if row_scale.numel() != n:
            raise ValueError("row_scale must have one entry per row")
    _check(load_library().dgnn_feature_transform(_ptr(x), n, f_in, _ptr(w), f_out, _ptr(row_scale), _ptr(h), dt,
                                                 _stream(x)), "dgnn_feature_transform")


def spmm_workspace(n: int, nnz: int, f: int) -> int:
    out = _sz(0)
    _check(load_library().dgnn_spmm_workspace(n, nnz, f, ctypes.byref(out)), "dgnn_spmm_workspace")
    return int(out.value)


def spmm(rowptr, colidx, nnz: int, dinv, h: torch.Tensor, z: torch.Tensor, ws, flags: int = 0) -> None:
    """Z = sigma?(A~ H)."""
    _need(rowptr, torch.int32, "rowptr"); _need(colidx, torch.int32, "colidx")
    dt = _dtype_code(h)
    n, f = h.shape
    if rowptr.numel() != n + 1 or tuple(z.shape) != (n, f) or z.dtype != h.dtype or colidx.numel() < nnz:
        raise ValueError("shape mismatch in spmm")
    _check(load_library().dgnn_spmm(n, nnz, _ptr(rowptr), _ptr(colidx), _ptr(dinv), _ptr(h), f, _ptr(z), dt, flags,
                                    _ptr(ws), ws.numel() * ws.element_size(), _stream(h)), "dgnn_spmm")


def spmm_static_limit() -> int:
    out = _sz(0)
    _check(load_library().dgnn_spmm_static_limit(ctypes.byref(out)), "dgnn_spmm_static_limit")
    return int(out.value)


def spmm_static(rowptr, colidx, nnz: int, dinv, h: torch.Tensor, z: torch.Tensor, flags: int = 0) -> None:
    """Z = sigma?(A~ H) without a workspace argument (scratch inside the library; nothing is allocated)."""
    _need(rowptr, torch.int32, "rowptr"); _need(colidx, torch.int32, "colidx")
    dt = _dtype_code(h)
    n, f = h.shape
    if rowptr.numel() != n + 1 or tuple(z.shape) != (n, f) or z.dtype != h.dtype or colidx.numel() < nnz:
        raise ValueError("shape mismatch in spmm_static")
    _check(load_library().dgnn_spmm_static(n, nnz, _ptr(rowptr), _ptr(colidx), _ptr(dinv), _ptr(h), f, _ptr(z), dt, flags,
                                           _stream(h)), "dgnn_spmm_static")


def mproduct(z: torch.Tensor, y: torch.Tensor, w: int, m_band: Optional[torch.Tensor] = None) -> None:
    """Y = Z x_1 M over tensors [T, n, f]; y may be z itself."""
    dt = _dtype_code(z)
    T, n, f = z.shape
    if tuple(y.shape) != (T, n, f) or y.dtype != z.dtype:
        raise ValueError("shape mismatch in mproduct")
    if m_band is not None:
        _need(m_band, torch.float32, "m_band")
        if m_band.numel() != T * w:
            raise ValueError("m_band must be [T, w]")
    _check(load_library().dgnn_mproduct(_ptr(z), _ptr(y), T, n, f, w, _ptr(m_band), dt, _stream(z)), "dgnn_mproduct")


def delta_rebuild_weighted(rowptr_prev, colidx_prev, val_prev, nnz_prev: int, add, dele, upd,
                           rowptr_next, colidx_next, val_next, ws, flags: int = 0, d_status=None) -> int:
    """Snapshots with values: add = (row, col, val), dele = (row, col), upd = (row, col, val) device tensors
    (or None); returns nnz of A_next.  flags may hold DGNN_UPDATES_SORTED (upd sorted by (row, col): the merge consumes it)."""
    n = rowptr_prev.numel() - 1
    ar, ac, av = add if add is not None else (None, None, None)
    dr, dc = dele if dele is not None else (None, None)
    ur, uc, uv = upd if upd is not None else (None, None, None)
    cnt = lambda t: 0 if t is None else int(t.numel())
    for t in (val_prev, val_next, av, uv):
        if t is not None:
            _need(t, torch.float32, "values")
    nnz_next = _i64(0)
    rc = load_library().dgnn_delta_rebuild_weighted(
        n, _ptr(rowptr_prev), _ptr(colidx_prev), _ptr(val_prev), nnz_prev, _ptr(ar), _ptr(ac), _ptr(av), cnt(ar),
        _ptr(dr), _ptr(dc), cnt(dr), _ptr(ur), _ptr(uc), _ptr(uv), cnt(ur), _ptr(rowptr_next), _ptr(colidx_next),
        _ptr(val_next), min(colidx_next.numel(), val_next.numel()), ctypes.byref(nnz_next), _ptr(ws),
        ws.numel() * ws.element_size(), flags, _ptr(d_status), _stream(rowptr_prev))
    _check(rc, "dgnn_delta_rebuild_weighted")
    return int(nnz_next.value)


def spmm_weighted(rowptr, colidx, val, nnz: int, h: torch.Tensor, z: torch.Tensor, ws, flags: int = 0,
                  dinv: Optional[torch.Tensor] = None) -> None:
    """Z = sigma?(V H) with one explicit value per stored entry; with dinv (and DGNN_H_PRESCALED) the
    sym-normalised weighted matrix."""
    _need(rowptr, torch.int32, "rowptr"); _need(colidx, torch.int32, "colidx"); _need(val, torch.float32, "val")
    dt = _dtype_code(h)
    n, f = h.shape
    if rowptr.numel() != n + 1 or tuple(z.shape) != (n, f) or z.dtype != h.dtype or colidx.numel() < nnz or val.numel() < nnz:
        raise ValueError("shape mismatch in spmm_weighted")
    _check(load_library().dgnn_spmm_weighted(n, nnz, _ptr(rowptr), _ptr(colidx), _ptr(val), _ptr(dinv), _ptr(h), f, _ptr(z),
                                             dt, flags, _ptr(ws), ws.numel() * ws.element_size(), _stream(h)),
           "dgnn_spmm_weighted")


def csr_validate(rowptr: torch.Tensor, colidx: torch.Tensor, nnz: int, status: torch.Tensor, require_diagonal: bool = True) -> None:
    """status[0] <- 0 if (rowptr, colidx) is a canonical snapshot, else the smallest DGNN_BAD_* code found."""
    _need(rowptr, torch.int32, "rowptr"); _need(colidx, torch.int32, "colidx"); _need(status, torch.int32, "status")
    if colidx.numel() < nnz:
        raise ValueError("colidx shorter than nnz")
    _check(load_library().dgnn_csr_validate(rowptr.numel() - 1, _ptr(rowptr), _ptr(colidx), nnz, int(require_diagonal),
                                            _ptr(status), _stream(rowptr)), "dgnn_csr_validate")


def csr_combine_workspace(nnz_s: int) -> int:
    out = _sz(0)
    _check(load_library().dgnn_csr_combine_workspace(nnz_s, ctypes.byref(out)), "dgnn_csr_combine_workspace")
    return int(out.value)


def csr_combine(s, a_in, alpha: float, a_out, beta: float, out, ws: torch.Tensor, diag_value: float = 0.0,
                status: Optional[torch.Tensor] = None) -> None:
    """C = S + alpha * A_in + beta * A_out.  s = (rowptr, colidx, val or None, nnz or an upper bound of it); a_in,
    a_out = (rowptr, colidx, nnz) or None; out = (rowptr, colidx, val) with capacity = colidx.numel().  Enqueue-only:
    the number of stored entries of C is left on the device, in out[0][n]."""
    rp_s, ci_s, val_s, nnz_s = s
    rp_c, ci_c, val_c = out
    n = rp_s.numel() - 1
    _need(rp_s, torch.int32, "rowptr_s"); _need(ci_s, torch.int32, "colidx_s")
    _need(rp_c, torch.int32, "rowptr_c"); _need(ci_c, torch.int32, "colidx_c"); _need(val_c, torch.float32, "val_c")
    if val_s is not None:
        _need(val_s, torch.float32, "val_s")
    if status is not None:
        _need(status, torch.int32, "status")
    if rp_c.numel() != n + 1 or val_c.numel() < ci_c.numel() or ci_s.numel() < nnz_s or (val_s is not None and val_s.numel() < nnz_s):
        raise ValueError("shape mismatch in csr_combine")
    args = []
    for op, name in ((a_in, "a_in"), (a_out, "a_out")):
        if op is None:
            args.append((None, None, 0))
            continue
        rp, ci, nnz = op
        _need(rp, torch.int32, name + " rowptr"); _need(ci, torch.int32, name + " colidx")
        if rp.numel() != n + 1 or ci.numel() < nnz:
            raise ValueError(f"shape mismatch in csr_combine ({name})")
        args.append((rp, ci, nnz))
    (rp_a, ci_a, nnz_a), (rp_o, ci_o, nnz_o) = args
    _check(load_library().dgnn_csr_combine(n, _ptr(rp_s), _ptr(ci_s), _ptr(val_s), nnz_s, _ptr(rp_a), _ptr(ci_a), nnz_a,
                                           float(alpha), _ptr(rp_o), _ptr(ci_o), nnz_o, float(beta), float(diag_value),
                                           _ptr(rp_c), _ptr(ci_c), _ptr(val_c), ci_c.numel(), _ptr(status), _ptr(ws),
                                           ws.numel() * ws.element_size(), _stream(rp_s)), "dgnn_csr_combine")


def csr_transpose(rowptr: torch.Tensor, colidx: torch.Tensor, nnz: int, val: Optional[torch.Tensor] = None):
    """(rowptr_t, colidx_t[, val_t]) of the transposed snapshot, in new tensors (the workspace is allocated here too:
    input formatting, once per block)."""
    _need(rowptr, torch.int32, "rowptr"); _need(colidx, torch.int32, "colidx")
    n = rowptr.numel() - 1
    if colidx.numel() < nnz or (val is not None and (val.numel() < nnz or val.dtype != torch.float32)):
        raise ValueError("shape mismatch in csr_transpose")
    lib = load_library()
    need = _sz(0)
    _check(lib.dgnn_csr_transpose_workspace(n, nnz, 0 if val is None else 1, ctypes.byref(need)), "dgnn_csr_transpose_workspace")
    dev = rowptr.device
    ws = torch.empty(need.value, dtype=torch.uint8, device=dev)
    rowptr_t = torch.empty(n + 1, dtype=torch.int32, device=dev)
    colidx_t = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    val_t = None if val is None else torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)
    _check(lib.dgnn_csr_transpose(n, nnz, _ptr(rowptr), _ptr(colidx), _ptr(val), _ptr(rowptr_t), _ptr(colidx_t), _ptr(val_t),
                                  _ptr(ws), need.value, _stream(rowptr)), "dgnn_csr_transpose")
    out = (rowptr_t, colidx_t[:nnz]) + (() if val is None else (val_t[:nnz],))
    return out


def coo_transpose(n: int, row: torch.Tensor, col: torch.Tensor):
    """(row_t, col_t): the pairs (col, row) sorted ascending, in new tensors (a difference list of the transposed series)."""
    _need(row, torch.int32, "row"); _need(col, torch.int32, "col")
    m = int(row.numel())
    if col.numel() != m:
        raise ValueError("shape mismatch in coo_transpose")
    lib = load_library()
    need = _sz(0)
    _check(lib.dgnn_coo_transpose_workspace(n, m, ctypes.byref(need)), "dgnn_coo_transpose_workspace")
    dev = row.device
    ws = torch.empty(need.value, dtype=torch.uint8, device=dev)
    row_t, col_t = torch.empty(m, dtype=torch.int32, device=dev), torch.empty(m, dtype=torch.int32, device=dev)
    _check(lib.dgnn_coo_transpose(n, m, _ptr(row), _ptr(col), _ptr(row_t), _ptr(col_t), _ptr(ws), need.value, _stream(row) if row.is_cuda else None),
           "dgnn_coo_transpose")
    return row_t, col_t


def csr_weighted_dinv_workspace(nnz: int) -> int:
    out = _sz(0)
    _check(load_library().dgnn_csr_weighted_dinv_workspace(nnz, ctypes.byref(out)), "dgnn_csr_weighted_dinv_workspace")
    return int(out.value)


def csr_weighted_dinv(rowptr: torch.Tensor, val: torch.Tensor, nnz: int, dinv: torch.Tensor, ws: torch.Tensor) -> None:
    """dinv[u] = (sum of the values of row u)^(-1/2)."""
    _need(rowptr, torch.int32, "rowptr"); _need(val, torch.float32, "val"); _need(dinv, torch.float32, "dinv")
    n = rowptr.numel() - 1
    if dinv.numel() != n or val.numel() < nnz:
        raise ValueError("shape mismatch in csr_weighted_dinv")
    _check(load_library().dgnn_csr_weighted_dinv(n, nnz, _ptr(rowptr), _ptr(val), _ptr(dinv), _ptr(ws),
                                                 ws.numel() * ws.element_size(), _stream(rowptr)), "dgnn_csr_weighted_dinv")


def concat_relu(y0: torch.Tensor, y1: torch.Tensor, out: torch.Tensor) -> None:
    """out = relu([y0 | y1]) row by row."""
    dt = _dtype_code(y0)
    n, f0 = y0.shape
    f1 = y1.shape[1]
    if y1.shape[0] != n or tuple(out.shape) != (n, f0 + f1) or y1.dtype != y0.dtype or out.dtype != y0.dtype:
        raise ValueError("shape mismatch in concat_relu")
    _check(load_library().dgnn_concat_relu(_ptr(y0), f0, _ptr(y1), f1, _ptr(out), n, dt, _stream(y0)), "dgnn_concat_relu")


def transform_concat_relu_supported(x: torch.Tensor, f_out: int) -> bool:
    f_in = x.shape[1]
    if x.dtype == torch.float32:
        return f_in in (16, 32, 64) and f_out in (32, 64)
    return x.dtype == torch.bfloat16 and f_in in (32, 64) and f_out in (32, 64) and f_in + f_out <= 128


def transform_concat_relu(x: torch.Tensor, w: torch.Tensor, out: torch.Tensor) -> None:
    """out = relu([x | x W]) in one pass (the CD-GCN layer's Y from Y0)."""
    dt = _dtype_code(x)
    n, f_in = x.shape
    f_out = w.shape[1]
    if w.dtype != x.dtype or out.dtype != x.dtype or w.shape[0] != f_in or tuple(out.shape) != (n, f_in + f_out):
        raise ValueError("shape or dtype mismatch in transform_concat_relu")
    if not (x.is_contiguous() and w.is_contiguous() and out.is_contiguous()):
        raise ValueError("transform_concat_relu needs contiguous tensors")
    _check(load_library().dgnn_transform_concat_relu(_ptr(x), n, f_in, _ptr(w), f_out, _ptr(out), dt, _stream(x)),
           "dgnn_transform_concat_relu")


def lstm_cell(gates_x, gates_h, bias, c_prev, c_next, h_next) -> None:
    """One LSTM step from the two halves of the gate pre-activations (gate order: input, forget, cell, output)."""
    dt = _dtype_code(gates_x)
    n, hidden = c_prev.shape
    for t in (gates_x, gates_h):
        if tuple(t.shape) != (n, 4 * hidden) or t.dtype != gates_x.dtype:
            raise ValueError("gate pre-activations must be [n, 4 * hidden]")
    for t in (c_prev, c_next, h_next):
        if tuple(t.shape) != (n, hidden) or t.dtype != gates_x.dtype:
            raise ValueError("state tensors must be [n, hidden]")
    if bias is not None:
        _need(bias, torch.float32, "bias")
        if bias.numel() != 4 * hidden:
            raise ValueError("bias must have 4 * hidden entries")
    _check(load_library().dgnn_lstm_cell(_ptr(gates_x), _ptr(gates_h), _ptr(bias), _ptr(c_prev), _ptr(c_next), _ptr(h_next),
                                         n, hidden, dt, _stream(gates_x)), "dgnn_lstm_cell")


def lstm_cell_backward(gates_x, gates_h, bias, c_prev, dh_a, dh_b, dc_next, da, dc_prev) -> None:
    """Gradient of one LSTM step with respect to the gate pre-activations (da) and the old cell state (dc_prev)."""
    dt = _dtype_code(gates_x)
    n, hidden = c_prev.shape
    for t in (gates_x, gates_h, da):
        if tuple(t.shape) != (n, 4 * hidden) or t.dtype != gates_x.dtype:
            raise ValueError("gate tensors must be [n, 4 * hidden]")
    for t in (c_prev, dh_a, dh_b, dc_next, dc_prev):
        if t is not None and (tuple(t.shape) != (n, hidden) or t.dtype != gates_x.dtype):
            raise ValueError("state tensors must be [n, hidden]")
    if bias is not None:
        _need(bias, torch.float32, "bias")
    _check(load_library().dgnn_lstm_cell_backward(_ptr(gates_x), _ptr(gates_h), _ptr(bias), _ptr(c_prev), _ptr(dh_a), _ptr(dh_b),
                                                  _ptr(dc_next), _ptr(da), _ptr(dc_prev), n, hidden, dt, _stream(gates_x)),
           "dgnn_lstm_cell_backward")


def lstm_step_backward_supported(y: torch.Tensor, hidden: int) -> bool:
    widths = {torch.float32: (16, 32), torch.bfloat16: (32,)}.get(y.dtype, ())
    return hidden in widths and y.shape[1] in (hidden, 2 * hidden)


def lstm_step_backward(y, h_prev, w_x, w_h, bias, c_prev, dh_a, dh_b, dc_next, da, dc_prev) -> None:
    """lstm_cell_backward with the gate pre-activations recomputed on chip from Y, h_prev and the weights."""
    n, f_y = y.shape
    hidden = c_prev.shape[1]
    if tuple(w_x.shape) != (f_y, 4 * hidden) or tuple(w_h.shape) != (hidden, 4 * hidden) or tuple(da.shape) != (n, 4 * hidden):
        raise ValueError("shape mismatch in lstm_step_backward")
    for t in (h_prev, c_prev, dh_a, dh_b, dc_next, dc_prev):
        if t is not None and (tuple(t.shape) != (n, hidden) or t.dtype != y.dtype):
            raise ValueError("state tensors must be [n, hidden]")
    if bias is not None:
        _need(bias, torch.float32, "bias")
    _check(load_library().dgnn_lstm_step_backward(_ptr(y), f_y, _ptr(h_prev), _ptr(w_x), _ptr(w_h), _ptr(bias), _ptr(c_prev),
                                                  _ptr(dh_a), _ptr(dh_b), _ptr(dc_next), _ptr(da), _ptr(dc_prev), n, hidden,
                                                  _dtype_code(y), _stream(y)), "dgnn_lstm_step_backward")


def concat_relu_backward(dy: torch.Tensor, y: torch.Tensor, d0: Optional[torch.Tensor], d1: torch.Tensor, f0: int) -> None:
    """d0 o d1 = dy where y > 0 (the adjoint of concat_relu); d0 may be None."""
    dt = _dtype_code(dy)
    n, ftot = dy.shape
    f1 = ftot - f0
    if tuple(y.shape) != (n, ftot) or tuple(d1.shape) != (n, f1) or y.dtype != dy.dtype or d1.dtype != dy.dtype or \
            (d0 is not None and (tuple(d0.shape) != (n, f0) or d0.dtype != dy.dtype)):
        raise ValueError("shape mismatch in concat_relu_backward")
    _check(load_library().dgnn_concat_relu_backward(_ptr(dy), _ptr(y), _ptr(d0), f0, _ptr(d1), f1, n, dt, _stream(dy)),
           "dgnn_concat_relu_backward")


def bias_grad_workspace(f: int) -> int:
    out = _sz(0)
    _check(load_library().dgnn_bias_grad_workspace(f, ctypes.byref(out)), "dgnn_bias_grad_workspace")
    return int(out.value)


def bias_grad(g: torch.Tensor, db: torch.Tensor, ws: torch.Tensor, accumulate: bool = False) -> None:
    """db (+)= column sums of g."""
    dt = _dtype_code(g)
    n, f = g.shape
    _need(db, torch.float32, "db")
    if db.numel() != f:
        raise ValueError("db must have one entry per column of g")
    _check(load_library().dgnn_bias_grad(_ptr(g), n, f, _ptr(db), int(accumulate), dt, _ptr(ws), ws.numel() * ws.element_size(),
                                         _stream(g)), "dgnn_bias_grad")


def add(a: torch.Tensor, b: torch.Tensor, out: torch.Tensor) -> None:
    """out = a + b (out may be a or b)."""
    dt = _dtype_code(a)
    n, f = a.shape
    if tuple(b.shape) != (n, f) or tuple(out.shape) != (n, f) or b.dtype != a.dtype or out.dtype != a.dtype:
        raise ValueError("shape mismatch in add")
    _check(load_library().dgnn_add(_ptr(a), _ptr(b), _ptr(out), n, f, dt, _stream(a)), "dgnn_add")


def lstm_step_supported(y: torch.Tensor, hidden: int) -> bool:
    widths = (16, 32) if y.dtype == torch.float32 else (32, 64) if y.dtype == torch.bfloat16 else ()
    return hidden in widths and y.shape[1] in (hidden, 2 * hidden)


def lstm_step(y, h_prev, w_x, w_h, bias, c, h_next) -> None:
    """One LSTM step with the gate pre-activations kept on chip; c is updated in place."""
    dt = _dtype_code(y)
    n, f_y = y.shape
    hidden = c.shape[1]
    if (tuple(h_prev.shape) != (n, hidden) or tuple(h_next.shape) != (n, hidden) or tuple(w_x.shape) != (f_y, 4 * hidden)
            or tuple(w_h.shape) != (hidden, 4 * hidden)):
        raise ValueError("shape mismatch in lstm_step")
    if bias is not None:
        _need(bias, torch.float32, "bias")
    _check(load_library().dgnn_lstm_step(_ptr(y), f_y, _ptr(h_prev), _ptr(w_x), _ptr(w_h), _ptr(bias), _ptr(c), _ptr(h_next),
                                         n, hidden, dt, _stream(y)), "dgnn_lstm_step")


def mproduct_backward(g_y: torch.Tensor, g_z: torch.Tensor, w: int, m_band: Optional[torch.Tensor] = None) -> None:
    """G_Z = G_Y x_1 M^T over tensors [T, n, f]; g_z may be g_y itself."""
    dt = _dtype_code(g_y)
    T, n, f = g_y.shape
    if tuple(g_z.shape) != (T, n, f) or g_z.dtype != g_y.dtype:
        raise ValueError("shape mismatch in mproduct_backward")
    if m_band is not None:
        _need(m_band, torch.float32, "m_band")
        if m_band.numel() != T * w:
            raise ValueError("m_band must be [T, w]")
    _check(load_library().dgnn_mproduct_backward(_ptr(g_y), _ptr(g_z), T, n, f, w, _ptr(m_band), dt, _stream(g_y)),
           "dgnn_mproduct_backward")


def _mproduct_block(fn, name, src, dst, w, t0, halo, m_band):
    dt = _dtype_code(src)
    T, n, f = src.shape
    if tuple(dst.shape) != (T, n, f) or dst.dtype != src.dtype:
        raise ValueError(f"shape mismatch in {name}")
    n_halo = 0
    if halo is not None and halo.numel() > 0:
        if halo.dtype != src.dtype or tuple(halo.shape[1:]) != (n, f):
            raise ValueError("hand-over frames must have the block's frame shape and dtype")
        n_halo = halo.shape[0]
    if m_band is not None:
        _need(m_band, torch.float32, "m_band")
    _check(fn(_ptr(src), _ptr(dst), T, n, f, w, _ptr(m_band), t0, _ptr(halo) if n_halo else None, n_halo, dt,
              _stream(src)), name)


def mproduct_block(z, y, w: int, t0: int, z_before: Optional[torch.Tensor] = None, m_band=None) -> None:
    """The M-transform of timesteps t0+1 .. t0+T of a longer series; z_before = the min(w-1, t0) frames before."""
    _mproduct_block(load_library().dgnn_mproduct_block, "dgnn_mproduct_block", z, y, w, t0, z_before, m_band)


def mproduct_backward_block(g_y, g_z, w: int, t0: int, g_after: Optional[torch.Tensor] = None, m_band=None) -> None:
    """Its adjoint for one block; g_after = upstream gradient of the (up to w-1) timesteps after the block."""
    _mproduct_block(load_library().dgnn_mproduct_backward_block, "dgnn_mproduct_backward_block", g_y, g_z, w, t0,
                    g_after, m_band)


def relu_backward(g: torch.Tensor, z: torch.Tensor, out: torch.Tensor, row_scale: Optional[torch.Tensor] = None) -> None:
    """out = row_scale * (z > 0 ? g : 0); out may be g itself."""
    dt = _dtype_code(g)
    n, f = g.shape
    if tuple(z.shape) != (n, f) or tuple(out.shape) != (n, f) or z.dtype != g.dtype or out.dtype != g.dtype:
        raise ValueError("shape mismatch in relu_backward")
    if row_scale is not None:
        _need(row_scale, torch.float32, "row_scale")
        if row_scale.numel() != n:
            raise ValueError("row_scale must have one entry per row")
    _check(load_library().dgnn_relu_backward(_ptr(g), _ptr(z), _ptr(row_scale), _ptr(out), n, f, dt, _stream(g)),
           "dgnn_relu_backward")


def weight_grad_workspace(f_in: int, f_out: int) -> int:
    out = _sz(0)
    _check(load_library().dgnn_weight_grad_workspace(f_in, f_out, ctypes.byref(out)), "dgnn_weight_grad_workspace")
    return int(out.value)


def weight_grad(x: torch.Tensor, g: torch.Tensor, dw: torch.Tensor, ws: torch.Tensor, accumulate: bool = False) -> None:
    """dw = X^T G (or dw += X^T G); dw is float32 whatever the storage type of x and g."""
    dt = _dtype_code(x)
    n, f_in = x.shape
    f_out = g.shape[1]
    _need(dw, torch.float32, "dw")
    if g.dtype != x.dtype or g.shape[0] != n or tuple(dw.shape) != (f_in, f_out):
        raise ValueError("shape mismatch in weight_grad")
    _check(load_library().dgnn_weight_grad(_ptr(x), _ptr(g), n, f_in, f_out, _ptr(dw), int(bool(accumulate)), dt,
                                           _ptr(ws), ws.numel() * ws.element_size(), _stream(x)), "dgnn_weight_grad")


def input_grad(g: torch.Tensor, w: torch.Tensor, dx: torch.Tensor, row_scale: Optional[torch.Tensor] = None) -> None:
    """dX = G W^T with w in its forward layout [f_in, f_out]."""
    dt = _dtype_code(g)
    n, f_out = g.shape
    f_in = w.shape[0]
    if w.dtype != g.dtype or dx.dtype != g.dtype or w.shape[1] != f_out or tuple(dx.shape) != (n, f_in):
        raise ValueError("shape mismatch in input_grad")
    if row_scale is not None:
        _need(row_scale, torch.float32, "row_scale")
    _check(load_library().dgnn_input_grad(_ptr(g), n, f_out, _ptr(w), f_in, _ptr(row_scale), _ptr(dx), dt, _stream(g)),
           "dgnn_input_grad")


# codes a device-side validation can leave in d_status (include/dgnn.h)
DGNN_BAD_INDEX_RANGE, DGNN_BAD_DELTA_ORDER, DGNN_BAD_DIAGONAL = 1, 2, 3
DGNN_BAD_DEL_ABSENT, DGNN_BAD_ADD_PRESENT, DGNN_BAD_EMPTY_ROW = 4, 5, 6
