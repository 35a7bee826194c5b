"""Seeded synthetic discrete-time dynamic graphs (DTDGs) and feature frames.

This module only makes *inputs*: snapshot edge sets E_1..E_T over a fixed vertex
set (Section "Discrete Time Dynamic Graphs"), the per-step graph difference of
consecutive snapshots (the two "extra edge" sets of Section "Graph-difference
Based Input Transfer"), feature frames X_t and GCN weights W.  It holds none of
the method's arithmetic (no normalisation, no aggregation, no temporal mixing)
and is the only code shared by the CPU oracle's tests and the GPU path's tests.

Everything is a pure function of (seed, purpose, timestep, index) through one
counter-based integer hash, written with wrap-around int64 tensor ops only, so
the same graph comes out on a CPU tensor and on a GPU tensor.  Real-valued
outputs (features, weights) use library log/cos and are therefore generated once
on one device and copied to whoever needs them.

The shapes stand in for the paper's workloads: uniform random snapshots like the
weak-scaling generator of Section "Scaling Study" (N vertices, N*f random
pairs), and R-MAT power-law snapshots for the skew of the real graphs of
Table 1, with small per-step churn, which is the regime the graph-difference
argument addresses.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import torch

__all__ = [
    "Workload", "WORKLOADS", "DynamicGraph", "mix64", "rand_bits", "rand_below",
    "stream_base", "features", "glorot_weight", "keys_to_coo", "keys_to_csr", "transpose_coo", "gradient", "SmoothedGraph",
]

_M64 = (1 << 64) - 1
MASK32 = (1 << 32) - 1


def _s64(c: int) -> int:
    """Python int -> the signed 64-bit value with the same low 64 bits."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """SplitMix64 output function (Steele, Lea, Flood 2014) on int64 tensors, mod 2^64."""
    x = x + _GOLDEN
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _mix64_int(v: int) -> int:
    v = (v + 0x9E3779B97F4A7C15) & _M64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _M64
    return v ^ (v >> 31)


def stream_base(seed: int, purpose: int, t: int = 0, sub: int = 0) -> int:
    """Key of an independent random stream, as a signed 64-bit Python int."""
    v = _mix64_int(seed & _M64)
    v = _mix64_int(v ^ ((purpose * 0xD6E8FEB86659FD93) & _M64))
    v = _mix64_int(v ^ ((t * 0xA0761D6478BD642F) & _M64))
    v = _mix64_int(v ^ ((sub * 0xE7037ED1A0B428DB) & _M64))
    return _s64(v)


def rand_bits(base: int, idx: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits per index (as int64), stream `base`."""
    return mix64(mix64(idx * _GOLDEN + base))


def rand_below(base: int, idx: torch.Tensor, m: int) -> torch.Tensor:
    """Integers in [0, m), m < 2^32, from the top 31 bits of the hash."""
    assert 0 < m < (1 << 32)
    return (_lsr(rand_bits(base, idx), 33) * m) >> 31


# purposes of the random streams
_P_ER, _P_RMAT, _P_PERM, _P_DEL, _P_ADD_U, _P_ADD_V, _P_FEAT, _P_W, _P_GRAD = range(1, 10)


@dataclass(frozen=True)
class Workload:
    """One seeded synthetic DTDG configuration."""
    name: str
    n: int                      # vertices N
    T: int                      # snapshots
    graph: str                  # "er" (undirected uniform) | "rmat" (directed power law)
    avg_deg: float = 0.0        # er: off-diagonal nonzeros per row (2 * undirected edges / N)
    n_draws: int = 0            # rmat: directed draws before de-duplication
    del_frac: float = 0.0       # fraction of off-diagonal edges deleted per step
    add_frac: float = 0.0       # fraction (of the same base) added per step
    f: int = 32                 # feature width F = F'
    dtype: str = "f32"          # storage type of X, W, H, Z: "f32" | "bf16"
    layers: int = 1             # GCN layers per snapshot
    window: int = 0             # M-product window w (0: no M-product)
    seed: int = 0x210907893
    scramble: bool = True       # rmat: relabel vertices by a seeded bijection
    rmat: Tuple[float, float, float, float] = (0.57, 0.19, 0.19, 0.05)

    def scaled(self, n: int, T: Optional[int] = None, **kw) -> "Workload":
        """Same recipe at another vertex count (edge count scales with n)."""
        r = n / self.n
        return replace(self, n=n, T=T or self.T,
                       n_draws=int(round(self.n_draws * r)), name=f"{self.name}@{n}", **kw)


_SEED0 = 0x210907893
WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1", n=1000, T=8, graph="er", avg_deg=10, del_frac=0.05, add_frac=0.05,
                   f=16, layers=1, window=3, seed=_SEED0 + 1),
    "c2": Workload("c2", n=1_000_000, T=32, graph="er", avg_deg=16, del_frac=0.02, add_frac=0.02,
                   f=64, layers=2, window=8, seed=_SEED0 + 2),
    "c3": Workload("c3", n=1 << 23, T=16, graph="rmat", n_draws=1 << 27, del_frac=0.01,
                   add_frac=0.01, f=32, layers=1, window=0, seed=_SEED0 + 3),
    "c4": Workload("c4", n=2_000_000, T=128, graph="er", avg_deg=12, del_frac=0.002,
                   add_frac=0.003, f=128, dtype="bf16", layers=1, window=16, seed=_SEED0 + 4),
    "c5": Workload("c5", n=1 << 24, T=8, graph="rmat", n_draws=1 << 28, del_frac=0.03,
                   add_frac=0.03, f=32, layers=1, window=0, seed=_SEED0 + 5),
}


def _first_k_unique(vals: torch.Tensor, k: int) -> torch.Tensor:
    """The first k distinct values of `vals`, in order of first appearance."""
    if vals.numel() == 0 or k <= 0:
        return vals[:0]
    sv, order = torch.sort(vals, stable=True)
    first = torch.ones_like(sv, dtype=torch.bool)
    first[1:] = sv[1:] != sv[:-1]
    pos = torch.sort(order[first]).values[:k]
    return vals[pos]


def _member(sorted_keys: torch.Tensor, q: torch.Tensor) -> torch.Tensor:
    if sorted_keys.numel() == 0:
        return torch.zeros_like(q, dtype=torch.bool)
    p = torch.searchsorted(sorted_keys, q).clamp_(max=sorted_keys.numel() - 1)
    return sorted_keys[p] == q


def keys_to_coo(keys: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """64-bit keys (row << 32 | col) -> int32 row, int32 col."""
    return (keys >> 32).to(torch.int32), (keys & MASK32).to(torch.int32)


def transpose_coo(row: torch.Tensor, col: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """The same entries with rows and columns exchanged, sorted by their new (row, col): the form in which
    a difference list (or a snapshot) of the transposed dynamic graph is handed over.  Input formatting
    only."""
    keys = torch.sort((col.to(torch.int64) << 32) | row.to(torch.int64)).values
    return keys_to_coo(keys)


def keys_to_csr(keys: torch.Tensor, n: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Sorted unique keys -> (rowptr int32[n+1], colidx int32[nnz]); input formatting only,
    used to hand the first snapshot of a block over whole."""
    rows = keys >> 32
    bounds = torch.arange(n + 1, dtype=torch.int64, device=keys.device)
    rowptr = torch.searchsorted(rows, bounds).to(torch.int32)
    return rowptr, (keys & MASK32).to(torch.int32)


class DynamicGraph:
    """State machine over snapshots: `keys` is E_t as sorted unique int64 keys
    (row << 32 | col), diagonal included; `advance()` moves to E_{t+1} and returns the
    graph difference as sorted COO (added edges, deleted edges)."""

    def __init__(self, wl: Workload, device: str | torch.device = "cpu", chunk: int = 1 << 24):
        self.wl = wl
        self.device = torch.device(device)
        self.chunk = chunk
        self.t = 1
        n = wl.n
        assert 0 < n < (1 << 31)
        self._diag = torch.arange(n, dtype=torch.int64, device=self.device) * ((1 << 32) + 1)
        if wl.graph == "er":
            self._upper = self._er_upper()
            self.keys = self._directed_from_upper(self._upper)
        elif wl.graph == "rmat":
            self._upper = None
            off = self._rmat_offdiag()
            self.keys = torch.sort(torch.cat([off, self._diag])).values
        else:
            raise ValueError(wl.graph)

    # ---------------------------------------------------------------- first snapshot
    def _pair_key_upper(self, u: torch.Tensor, v: torch.Tensor) -> torch.Tensor:
        lo, hi = torch.minimum(u, v), torch.maximum(u, v)
        return (lo << 32) | hi

    def _er_upper(self) -> torch.Tensor:
        wl = self.wl
        m = int(round(wl.n * wl.avg_deg / 2))
        got = torch.empty(0, dtype=torch.int64, device=self.device)
        rnd = 0
        while got.numel() < m:
            k = m + m // 4 + 64
            idx = torch.arange(k, dtype=torch.int64, device=self.device)
            u = rand_below(stream_base(wl.seed, _P_ER, 0, 2 * rnd), idx, wl.n)
            v = rand_below(stream_base(wl.seed, _P_ER, 0, 2 * rnd + 1), idx, wl.n)
            cand = self._pair_key_upper(u, v)[u != v]
            got = _first_k_unique(torch.cat([got, cand]), m)
            rnd += 1
        return torch.sort(got).values

    def _directed_from_upper(self, upper: torch.Tensor) -> torch.Tensor:
        lo, hi = upper >> 32, upper & MASK32
        return torch.sort(torch.cat([upper, (hi << 32) | lo, self._diag])).values

    def _perm(self, x: torch.Tensor) -> torch.Tensor:
        """Seeded bijection on [0, 2^k), k = log2 N: odd multiply-add and xor-shift rounds."""
        wl = self.wl
        k = wl.n.bit_length() - 1
        mask = wl.n - 1
        s = max(1, k // 2)
        for r in range(2):
            a = (_mix64_int(stream_base(wl.seed, _P_PERM, r, 0) & _M64) | 1) & mask
            b = _mix64_int(stream_base(wl.seed, _P_PERM, r, 1) & _M64) & mask
            x = (x * a + b) & mask
            x = x ^ (x >> s)
        return x

    def _rmat_pairs(self, base_t: int, start: int, count: int) -> Tuple[torch.Tensor, torch.Tensor]:
        wl = self.wl
        k = wl.n.bit_length() - 1
        assert (1 << k) == wl.n, "R-MAT needs a power-of-two vertex count"
        a, b, c, _ = wl.rmat
        ta, tb, tc = int(a * 65536), int((a + b) * 65536), int((a + b + c) * 65536)
        idx = torch.arange(start, start + count, dtype=torch.int64, device=self.device)
        u = torch.zeros_like(idx)
        v = torch.zeros_like(idx)
        bits = None
        for lvl in range(k):
            if lvl % 4 == 0:
                bits = rand_bits(stream_base(wl.seed, _P_RMAT, base_t, lvl // 4), idx)
            r = _lsr(bits, 16 * (lvl % 4)) & 0xFFFF
            rowbit = (r >= tb).to(torch.int64)                       # quadrants c, d
            colbit = (((r >= ta) & (r < tb)) | (r >= tc)).to(torch.int64)   # quadrants b, d
            u = (u << 1) | rowbit
            v = (v << 1) | colbit
        if wl.scramble:
            u, v = self._perm(u), self._perm(v)
        return u, v

    def _rmat_offdiag(self) -> torch.Tensor:
        wl = self.wl
        parts = []
        for start in range(0, wl.n_draws, self.chunk):
            cnt = min(self.chunk, wl.n_draws - start)
            u, v = self._rmat_pairs(0, start, cnt)
            key = ((u << 32) | v)[u != v]
            parts.append(torch.unique(key))
        return torch.unique(torch.cat(parts)) if parts else self._diag[:0]

    # ---------------------------------------------------------------- one step of churn
    def _pick_indices(self, m: int, k: int, base_purpose: int) -> torch.Tensor:
        """k distinct positions in [0, m), uniformly."""
        wl = self.wl
        k = min(k, m)
        got = torch.empty(0, dtype=torch.int64, device=self.device)
        rnd = 0
        while got.numel() < k:
            kk = k + k // 4 + 64
            idx = torch.arange(kk, dtype=torch.int64, device=self.device)
            cand = rand_below(stream_base(wl.seed, base_purpose, self.t, rnd), idx, m)
            got = _first_k_unique(torch.cat([got, cand]), k)
            rnd += 1
        return got

    def advance(self):
        """E_t -> E_{t+1}.  Returns (add_row, add_col, del_row, del_col), int32, each list
        sorted by (row, col) and duplicate-free; added edges are absent from E_t, deleted
        edges are present in E_t, the diagonal is never touched."""
        wl = self.wl
        dev = self.device
        if wl.graph == "er":
            base = self._upper
            m = base.numel()
            n_del = int(round(wl.del_frac * m))
            n_add = int(round(wl.add_frac * m))
            del_pos = self._pick_indices(m, n_del, _P_DEL)
            keep = torch.ones(m, dtype=torch.bool, device=dev)
            keep[del_pos] = False
            del_u = base[del_pos]
            add_u = torch.empty(0, dtype=torch.int64, device=dev)
            rnd = 0
            while add_u.numel() < n_add:
                kk = n_add + n_add // 4 + 64
                idx = torch.arange(kk, dtype=torch.int64, device=dev)
                u = rand_below(stream_base(wl.seed, _P_ADD_U, self.t, rnd), idx, wl.n)
                v = rand_below(stream_base(wl.seed, _P_ADD_V, self.t, rnd), idx, wl.n)
                cand = self._pair_key_upper(u, v)[u != v]
                cand = cand[~_member(base, cand)]
                add_u = _first_k_unique(torch.cat([add_u, cand]), n_add)
                rnd += 1
            self._upper = torch.sort(torch.cat([base[keep], add_u])).values
            self.keys = self._directed_from_upper(self._upper)

            def both(x):
                lo, hi = x >> 32, x & MASK32
                return torch.sort(torch.cat([x, (hi << 32) | lo])).values
            add_k, del_k = both(add_u), both(del_u)
        else:
            keys = self.keys
            offmask = (keys >> 32) != (keys & MASK32)
            off = keys[offmask]
            m = off.numel()
            n_del = int(round(wl.del_frac * m))
            n_add = int(round(wl.add_frac * m))
            # deletions: uniform over stored off-diagonal entries (so proportional to row degree)
            del_pos = self._pick_indices(m, n_del, _P_DEL)
            keep = torch.ones(m, dtype=torch.bool, device=dev)
            keep[del_pos] = False
            del_k = torch.sort(off[del_pos]).values
            # additions: source of one random stored entry, destination of another
            add_k = torch.empty(0, dtype=torch.int64, device=dev)
            rnd = 0
            while add_k.numel() < n_add and m > 0:
                kk = n_add + n_add // 4 + 64
                idx = torch.arange(kk, dtype=torch.int64, device=dev)
                i1 = rand_below(stream_base(wl.seed, _P_ADD_U, self.t, rnd), idx, m)
                i2 = rand_below(stream_base(wl.seed, _P_ADD_V, self.t, rnd), idx, m)
                u, v = off[i1] >> 32, off[i2] & MASK32
                cand = ((u << 32) | v)[u != v]
                cand = cand[~_member(keys, cand)]
                add_k = _first_k_unique(torch.cat([add_k, cand]), n_add)
                rnd += 1
            add_k = torch.sort(add_k).values
            self.keys = torch.sort(torch.cat([off[keep], add_k, self._diag])).values
        self.t += 1
        ar, ac = keys_to_coo(add_k)
        dr, dc = keys_to_coo(del_k)
        return ar, ac, dr, dc

    # ---------------------------------------------------------------- views
    def csr(self) -> Tuple[torch.Tensor, torch.Tensor]:
        return keys_to_csr(self.keys, self.wl.n)

    @property
    def nnz(self) -> int:
        return int(self.keys.numel())


def _normal(base: int, start: int, count: int, device) -> torch.Tensor:
    """count N(0,1) draws by Box-Muller from the hashed counter, float32."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    h = rand_bits(base, idx)
    u1 = ((_lsr(h, 40) & 0xFFFFFF).to(torch.float64) + 1.0) / 16777216.0     # (0, 1]
    u2 = ((_lsr(h, 16) & 0xFFFFFF).to(torch.float64)) / 16777216.0           # [0, 1)
    z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
    return z.to(torch.float32)


class SmoothedGraph:
    """The smoothed series of a dynamic graph (Section "Smoothening the Input Graphs"), prepared the way that
    section describes it, as pre-processing: snapshot t of the smoothed series is the sum of the raw snapshots
    of the last `life` timesteps, S_t = sum_{i = max(1, t-life+1)}^{t} A_i, so a stored entry carries the number
    of those snapshots that hold the edge (mode "edge_life"), or that number divided by min(life, t), which is
    what the M-transform of the adjacency tensor gives (mode "mproduct").

    `keys` / `vals` are S_t as sorted unique int64 keys and float32 values; `advance()` moves to S_{t+1} and
    returns the weighted graph difference in the form the weighted rebuild takes:
        (add_row, add_col, add_val), (del_row, del_col), (upd_row, upd_col, upd_val)
    each sorted by (row, col).  Input formatting: the method's arithmetic is not here."""

    def __init__(self, wl: Workload, life: int, mode: str = "edge_life", device="cpu"):
        assert life >= 1 and mode in ("edge_life", "mproduct")
        self.raw = DynamicGraph(wl, device=device)
        self.life, self.mode = life, mode
        self.window = [self.raw.keys]
        self.t = 1
        self.keys, self.vals = self._sum()

    def _sum(self):
        keys, counts = torch.unique(torch.cat(self.window), return_counts=True)      # sorted
        vals = counts.to(torch.float32)
        if self.mode == "mproduct":
            vals = vals / float(min(self.life, self.t))
        return keys, vals

    def csr(self):
        rp, ci = keys_to_csr(self.keys, self.raw.wl.n)
        return rp, ci, self.vals

    def advance(self):
        self.raw.advance()
        self.t += 1
        self.window.append(self.raw.keys)
        if len(self.window) > self.life:
            self.window.pop(0)
        old_k, old_v = self.keys, self.vals
        self.keys, self.vals = self._sum()
        in_old = _member(old_k, self.keys)
        in_new = _member(self.keys, old_k)
        add_k, add_v = self.keys[~in_old], self.vals[~in_old]
        del_k = old_k[~in_new]
        stay_new, stay_old = self.vals[in_old], old_v[in_new]          # same keys, same order
        changed = stay_new != stay_old
        upd_k, upd_v = self.keys[in_old][changed], stay_new[changed]
        return (keys_to_coo(add_k) + (add_v,), keys_to_coo(del_k), keys_to_coo(upd_k) + (upd_v,))


def features(wl: Workload, t: int, device="cpu", chunk_rows: int = 1 << 20) -> torch.Tensor:
    """Frame X_t, N x F, entries N(0,1); float32, or rounded to bfloat16 for bf16 workloads."""
    out = torch.empty((wl.n, wl.f), dtype=torch.float32, device=device)
    base = stream_base(wl.seed, _P_FEAT, t, 0)
    for r0 in range(0, wl.n, chunk_rows):
        r1 = min(wl.n, r0 + chunk_rows)
        out[r0:r1] = _normal(base, r0 * wl.f, (r1 - r0) * wl.f, device).view(r1 - r0, wl.f)
    return out.to(torch.bfloat16) if wl.dtype == "bf16" else out


def gradient(wl: Workload, t: int, device="cpu", chunk_rows: int = 1 << 20) -> torch.Tensor:
    """Frame t of a stand-in upstream gradient dL/dY, N x F, entries N(0,1) (what a loss layer above the
    block would send down); float32, or rounded to bfloat16 for bf16 workloads."""
    out = torch.empty((wl.n, wl.f), dtype=torch.float32, device=device)
    base = stream_base(wl.seed, _P_GRAD, t, 0)
    for r0 in range(0, wl.n, chunk_rows):
        r1 = min(wl.n, r0 + chunk_rows)
        out[r0:r1] = _normal(base, r0 * wl.f, (r1 - r0) * wl.f, device).view(r1 - r0, wl.f)
    return out.to(torch.bfloat16) if wl.dtype == "bf16" else out


def glorot_weight(wl: Workload, layer: int, device="cpu", t: int = 0) -> torch.Tensor:
    """W (F x F'), Glorot-uniform U(-a, a), a = sqrt(6 / (F + F')); `t` selects a per-timestep
    weight for models that evolve W over time."""
    f = wl.f
    a = math.sqrt(6.0 / (f + f))
    idx = torch.arange(f * f, dtype=torch.int64, device=device)
    h = rand_bits(stream_base(wl.seed, _P_W, t, layer), idx)
    u = (_lsr(h, 11).to(torch.float64)) / float(1 << 53)
    w = ((2.0 * u - 1.0) * a).to(torch.float32).view(f, f)
    return w.to(torch.bfloat16) if wl.dtype == "bf16" else w
