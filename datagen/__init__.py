"""Seeded synthetic inputs shaped like the paper's workloads (Section 4: click-through-rate
logistic regression on ~45 M x 1 M one-hot data, plus dense / SVM stand-ins).

This module serves BOTH the CPU oracle and the HIP library and therefore contains none of the
solver's arithmetic: it only fabricates matrices and labels.  Every random draw is a pure function
of (seed, purpose, index) through a 64-bit integer mixer written with wrapping int64 tensor
arithmetic, so the same code gives the same bits on the CPU and on the GPU for all integer outputs
(sparsity patterns, categories).  Real-valued outputs (values, labels) are produced once and the
same arrays are handed to both sides.

The public Criteo click logs that the paper trains on are not available here; `onehot_fields`
is a stand-in that takes only their shape (n rows, 1 M hashed columns, 39 one-hot fields, 25.6 %
positive rate).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

__all__ = [
    "Problem", "uniform_sparse_logistic", "dense_ridge", "zipf_sparse_svm", "onehot_fields",
    "csr_to_csc", "config", "CONFIG_SEED",
]

CONFIG_SEED = 180306333  # master seed; config k uses CONFIG_SEED + k

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 stores for the same bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(z: int) -> int:
    z = (z + _GOLD) & _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_base(seed: int, *purpose: int) -> int:
    """Fold (seed, purpose ids...) into one 64-bit stream constant (host side, python ints)."""
    h = _mix_py(seed & _M64)
    for p in purpose:
        h = _mix_py(h ^ ((p * _GOLD) & _M64))
    return h


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    return (z >> k) & ((1 << (64 - k)) - 1)


def hash64(base: int, idx: torch.Tensor) -> torch.Tensor:
    """64-bit mix of (base, idx); idx is an int64 tensor; arithmetic wraps mod 2^64."""
    z = idx * _s64(_GOLD) + _s64(base)
    z = z + _s64(_GOLD)
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def u32(base: int, idx: torch.Tensor) -> torch.Tensor:
    """Uniform integer in [0, 2^32) as int64."""
    return _lsr(hash64(base, idx), 32)


def uniform01(base: int, idx: torch.Tensor) -> torch.Tensor:
    """Uniform double in (0, 1)."""
    return (_lsr(hash64(base, idx), 11).to(torch.float64) + 0.5) * (2.0 ** -53)


def normal(base: int, idx: torch.Tensor) -> torch.Tensor:
    """Standard normal double (Box-Muller on two decorrelated streams)."""
    u1 = uniform01(_mix_py(base ^ 0x1111), idx)
    u2 = uniform01(_mix_py(base ^ 0x2222), idx)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)


def _arange(n: int, device) -> torch.Tensor:
    return torch.arange(n, dtype=torch.int64, device=device)


def cdf_table_u32(pmf: np.ndarray, device) -> torch.Tensor:
    """Integer CDF thresholds scaled to 2^32 (built once on the host in fp64).  A uniform 32-bit
    integer u falls in category searchsorted(table, u, right=True)."""
    c = np.cumsum(np.asarray(pmf, dtype=np.float64))
    c = c / c[-1]
    t = np.floor(c * 4294967296.0).astype(np.int64)
    t[-1] = 1 << 32
    return torch.from_numpy(t).to(device)


def zipf_pmf(ncat: int, s: float) -> np.ndarray:
    r = np.arange(1, ncat + 1, dtype=np.float64)
    p = r ** (-s)
    return p / p.sum()


def sample_table(table: torch.Tensor, base: int, idx: torch.Tensor) -> torch.Tensor:
    c = torch.searchsorted(table, u32(base, idx), right=True)
    return torch.clamp(c, max=table.numel() - 1)


@dataclass
class Problem:
    """A generated problem.  Sparse layouts: ptr int64[m+1], idx int32[nnz], val fp32[nnz].
    Dense: val fp32 holding the matrix in the stated order.  y fp32[n]."""
    name: str
    layout: str            # "csr" | "csc" | "dense_colmajor"
    n: int
    d: int
    ptr: Optional[torch.Tensor]
    idx: Optional[torch.Tensor]
    val: torch.Tensor
    y: torch.Tensor
    loss: str              # "ridge" | "logistic" | "hinge"
    lam: float
    epochs: int
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        # (val = None: pattern-only data, every stored value is 1)
        return int(self.val.numel()) if self.val is not None else int(self.idx.numel())

    def to(self, device) -> "Problem":
        mv = lambda t: None if t is None else t.to(device)
        return Problem(self.name, self.layout, self.n, self.d, mv(self.ptr), mv(self.idx),
                       mv(self.val), mv(self.y), self.loss, self.lam, self.epochs, dict(self.meta))


def csr_to_csc(n: int, d: int, ptr, idx, val):
    """Transpose a CSR triple into CSC (rows ascending inside each column)."""
    device = idx.device
    counts = (ptr[1:] - ptr[:-1])
    rows = torch.repeat_interleave(_arange(n, device), counts)
    order = torch.sort(idx.to(torch.int64), stable=True).indices
    cidx = rows[order].to(torch.int32)
    cval = val[order]
    cptr = torch.zeros(d + 1, dtype=torch.int64, device=device)
    cptr[1:] = torch.cumsum(torch.bincount(idx.to(torch.int64), minlength=d), 0)
    return cptr, cidx, cval


def _distinct_draws(n: int, k: int, base_seed: int, draw, device) -> torch.Tensor:
    """n rows of k distinct categories: draw, then redraw in-row duplicates until none remain
    (integer rejection).  Returns int64 [n, k], ascending inside each row."""
    slot = _arange(n * k, device).view(n, k)
    cols = draw(stream_base(base_seed, 0), slot)
    rnd = 0
    while True:
        cols, _ = torch.sort(cols, dim=1)
        dup = torch.zeros_like(cols, dtype=torch.bool)
        dup[:, 1:] = cols[:, 1:] == cols[:, :-1]
        if not bool(dup.any()):
            return cols
        rnd += 1
        cols[dup] = draw(stream_base(base_seed, rnd), slot[dup])
        if rnd > 10000:
            raise RuntimeError("duplicate rejection did not terminate")


def uniform_sparse_logistic(n=10_000, d=1_000, k=20, seed=CONFIG_SEED + 1, lam=1e-3,
                            epochs=10, device="cpu") -> Problem:
    """Config 1: every row has k distinct columns, uniform; values 1.0;
    y = sign(x.w* + 0.1 N(0,1)), w* ~ N(0,1).  Stored CSC (primal SCD)."""
    draw = lambda base, slot: u32(base, slot) % d
    cols = _distinct_draws(n, k, stream_base(seed, 10), draw, device)
    wstar = normal(stream_base(seed, 20), _arange(d, device))
    margin = wstar[cols].sum(dim=1) + 0.1 * normal(stream_base(seed, 21), _arange(n, device))
    y = torch.where(margin >= 0, 1.0, -1.0).to(torch.float32)
    ptr = _arange(n + 1, device) * k
    idx = cols.reshape(-1).to(torch.int32)
    val = torch.ones(n * k, dtype=torch.float32, device=device)
    cptr, cidx, cval = csr_to_csc(n, d, ptr, idx, val)
    return Problem("uniform_sparse_logistic", "csc", n, d, cptr, cidx, cval, y, "logistic", lam,
                   epochs, {"csr": (ptr, idx, val), "wstar": wstar})


def dense_ridge(n=400_000, d=2_000, seed=CONFIG_SEED + 2, lam=1e-4, epochs=20,
                device="cpu", row_block=50_000) -> Problem:
    """Config 2: dense N(0,1) entries, every row scaled to unit L2 norm;
    y = x.w* + 0.01 N(0,1), w* ~ N(0, 1/d).  Stored column-major (fp32[d][n])."""
    wstar = normal(stream_base(seed, 20), _arange(d, device)) / math.sqrt(d)
    A = torch.empty((d, n), dtype=torch.float32, device=device)  # column-major n x d
    y = torch.empty(n, dtype=torch.float32, device=device)
    base = stream_base(seed, 10)
    for r0 in range(0, n, row_block):
        r1 = min(n, r0 + row_block)
        e = _arange((r1 - r0) * d, device) + r0 * d
        X = normal(base, e).view(r1 - r0, d)
        X = X / torch.linalg.norm(X, dim=1, keepdim=True)
        Xf = X.to(torch.float32)
        A[:, r0:r1] = Xf.t()
        noise = normal(stream_base(seed, 21), _arange(r1 - r0, device) + r0)
        y[r0:r1] = (Xf.to(torch.float64) @ wstar + 0.01 * noise).to(torch.float32)
    return Problem("dense_ridge", "dense_colmajor", n, d, None, None, A.reshape(-1), y, "ridge", lam,
                   epochs, {"wstar": wstar})


def zipf_sparse_svm(n=1_000_000, d=100_000, k=50, s=1.1, seed=CONFIG_SEED + 3, lam=1e-5,
                    epochs=30, flip=0.05, device="cpu") -> Problem:
    """Config 3: k distinct columns per row with Zipf(s) popularity (column = rank), values
    |N(0,1)| with rows scaled to unit L2 norm; labels from a planted sparse w* (1 % nonzero),
    a fraction `flip` of them flipped.  Stored CSR (dual SCD)."""
    table = cdf_table_u32(zipf_pmf(d, s), device)
    draw = lambda base, slot: sample_table(table, base, slot)
    cols = _distinct_draws(n, k, stream_base(seed, 10), draw, device)
    vals = normal(stream_base(seed, 11), _arange(n * k, device)).abs().view(n, k)
    vals = vals / torch.linalg.norm(vals, dim=1, keepdim=True)
    nz = max(1, d // 100)
    support = torch.sort(u32(stream_base(seed, 20), _arange(d, device)), stable=True).indices[:nz]
    wstar = torch.zeros(d, dtype=torch.float64, device=device)
    wstar[support] = normal(stream_base(seed, 21), _arange(nz, device))
    margin = (vals * wstar[cols]).sum(dim=1)
    coin = uniform01(stream_base(seed, 22), _arange(n, device)) < 0.5
    y = torch.where(margin > 0, 1.0, torch.where(margin < 0, -1.0, torch.where(coin, 1.0, -1.0)))
    flipm = uniform01(stream_base(seed, 23), _arange(n, device)) < flip
    y = torch.where(flipm, -y, y).to(torch.float32)
    ptr = _arange(n + 1, device) * k
    return Problem("zipf_sparse_svm", "csr", n, d, ptr, cols.reshape(-1).to(torch.int32),
                   vals.reshape(-1).to(torch.float32), y, "hinge", lam, epochs, {"wstar": wstar})


# ---- 39-field one-hot generator (configs 4 and 5) ----------------------------------------------
N_NUMERIC = 13
N_CATEG = 26
NUM_BINS = 64


def field_layout(d: int):
    """Column range [start, start+size) of every field: 13 numeric fields of 64 bins first,
    then 26 categorical fields sharing the remaining columns (the first few one larger)."""
    sizes = [NUM_BINS] * N_NUMERIC
    rest = d - NUM_BINS * N_NUMERIC
    if rest < N_CATEG:
        raise ValueError("d too small for the 39-field layout")
    q, r = divmod(rest, N_CATEG)
    sizes += [q + 1 if f < r else q for f in range(N_CATEG)]
    starts = np.concatenate([[0], np.cumsum(sizes)])[:-1]
    return [int(s) for s in starts], sizes


def _numeric_bin_pmf(f: int) -> np.ndarray:
    """pmf of bin = clamp(floor(4 log2(1+z)), 0, 63) for a log-normal count z = exp(mu + sigma N)."""
    mu, sigma = 0.5 + 0.25 * f, 2.0
    edges = 2.0 ** (np.arange(0, NUM_BINS + 1) / 4.0) - 1.0   # z-range of bin b is [edges[b], edges[b+1])
    cdf = np.array([0.0 if e <= 0 else 0.5 * (1 + math.erf((math.log(e) - mu) / (sigma * math.sqrt(2))))
                    for e in edges])
    cdf[-1] = 1.0
    p = np.diff(cdf)
    return np.maximum(p, 1e-12)


def onehot_categories(n: int, d: int, seed: int, f: int, device, row0: int = 0, nrows: Optional[int] = None,
                      rows: Optional[torch.Tensor] = None):
    """Category (column offset inside field f) of rows [row0, row0+nrows), or of the given int64
    row numbers: int64."""
    starts, sizes = field_layout(d)
    nrows = n - row0 if nrows is None else nrows
    pmf = _numeric_bin_pmf(f) if f < N_NUMERIC else zipf_pmf(sizes[f], 1.2)
    table = cdf_table_u32(pmf, device)
    which = _arange(nrows, device) + row0 if rows is None else rows.to(device=device, dtype=torch.int64)
    return sample_table(table, stream_base(seed, 100 + f), which)


def onehot_fields(n=45_840_617, d=1_000_000, seed=CONFIG_SEED + 4, lam=1e-6, epochs=100,
                  pos_rate=0.256, device="cpu", want_csr=False, name="onehot_fields", pattern_only=False) -> Problem:
    """Configs 4/5: exactly 39 nonzeros (1.0) per row, one per field; categorical fields are
    Zipf(1.2) over disjoint column ranges, numeric fields fall into 64 log-spaced bins.
    w*_j ~ N(0, 1/39); y ~ Bernoulli(sigmoid(x.w* + b)) mapped to +-1 with b set by bisection so
    that the mean probability over the first 10^6 rows is `pos_rate`.  Stored CSC with rows
    ascending inside each column; field f occupies idx[f*n:(f+1)*n]."""
    starts, sizes = field_layout(d)
    nf = N_NUMERIC + N_CATEG
    wstar = normal(stream_base(seed, 20), _arange(d, device)) / math.sqrt(nf)
    ptr = torch.zeros(d + 1, dtype=torch.int64, device=device)
    idx = torch.empty(n * nf, dtype=torch.int32, device=device)
    margin = torch.zeros(n, dtype=torch.float64, device=device)
    csr_cols = torch.empty((n, nf), dtype=torch.int32, device=device) if want_csr else None
    for f in range(nf):
        cat = onehot_categories(n, d, seed, f, device)
        margin += wstar[cat + starts[f]]
        if want_csr:
            csr_cols[:, f] = (cat + starts[f]).to(torch.int32)
        order = torch.sort(cat, stable=True).indices
        idx[f * n:(f + 1) * n] = order.to(torch.int32)
        ptr[starts[f] + 1: starts[f] + sizes[f] + 1] = torch.bincount(cat, minlength=sizes[f])
        del cat, order
    ptr = torch.cumsum(ptr, 0)
    ms = margin[: min(n, 1_000_000)]
    lo, hi = -30.0, 30.0
    for _ in range(80):
        b = 0.5 * (lo + hi)
        if float(torch.sigmoid(ms + b).mean()) < pos_rate:
            lo = b
        else:
            hi = b
    b = 0.5 * (lo + hi)
    u = uniform01(stream_base(seed, 21), _arange(n, device))
    y = torch.where(u < torch.sigmoid(margin + b), 1.0, -1.0).to(torch.float32)
    # pattern_only: no value array at all (val = None stands for "every stored value is 1")
    val = None if pattern_only else torch.ones(n * nf, dtype=torch.float32, device=device)
    meta = {"wstar": wstar, "bias": b, "field_starts": starts, "field_sizes": sizes}
    if want_csr:
        meta["csr"] = (_arange(n + 1, device) * nf, csr_cols.reshape(-1),
                       torch.ones(n * nf, dtype=torch.float32, device=device))
    return Problem(name, "csc", n, d, ptr, idx, val, y, "logistic", lam, epochs, meta)


def config(k: int, device="cpu", scale: float = 1.0, **kw) -> Problem:
    """The five benchmark configurations; `scale` < 1 shrinks the row count (tests)."""
    s = lambda x: max(1, int(round(x * scale)))
    if k == 1:
        return uniform_sparse_logistic(n=s(10_000), device=device, **kw)
    if k == 2:
        return dense_ridge(n=s(400_000), device=device, **kw)
    if k == 3:
        return zipf_sparse_svm(n=s(1_000_000), device=device, **kw)
    if k == 4:
        return onehot_fields(n=s(45_840_617), device=device, **kw)
    if k == 5:
        return onehot_fields(n=s(200_000_000), seed=CONFIG_SEED + 5, lam=1e-7, epochs=5,
                             device=device, name="onehot_fields_streamed", **kw)
    raise ValueError("config index must be 1..5")
