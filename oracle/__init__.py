"""CPU oracle for the SCD local solver (arXiv 1803.06333, Section 3.1) -- TEST INFRASTRUCTURE.

Thin ctypes/numpy access to `snap_oracle.c` (built by `oracle/build.py`) plus a small driver that
runs epochs the way the paper's solver does (Section 3.1-3.2: a fresh permutation per pass, every
coordinate once).  Nothing here may be imported by the product package; only `tests/`, the smoke
check and the benchmark's CPU-baseline leg use it.  It shares no code with the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

from .build import build as build_oracle, LIB_PATH

RIDGE, LOGISTIC, HINGE = 0, 1, 2
LOSS_ID = {"ridge": RIDGE, "logistic": LOGISTIC, "hinge": HINGE}

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build_oracle()
        L = C.CDLL(LIB_PATH)
        L.oracle_key.restype = C.c_uint32
        L.oracle_key.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.oracle_perm.restype = C.c_int
        L.oracle_primal_objective.restype = C.c_double
        L.oracle_hinge_dual_objective.restype = C.c_double
        L.oracle_logistic_dual_objective.restype = C.c_double
        L.oracle_primal_gap_fenchel.restype = C.c_double
        L.oracle_primal_gap_gradient.restype = C.c_double
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def key(seed: int, chunk: int, c: int) -> int:
    return int(lib().oracle_key(C.c_uint64(seed), C.c_uint32(chunk), C.c_uint32(c)))


def permutation(seed: int, m: int, chunk: int = 0, want_keys: bool = False):
    """perm[k] = the coordinate (relative to the chunk start) visited k-th."""
    perm = np.empty(m, dtype=np.uint32)
    keys = np.empty(m, dtype=np.uint32) if want_keys else None
    rc = lib().oracle_perm(C.c_uint64(seed), C.c_uint32(chunk), C.c_uint32(m), _p(keys), _p(perm))
    if rc != 0:
        raise MemoryError("oracle_perm")
    return (perm, keys) if want_keys else perm


@dataclass
class Matrix:
    """layout: 'csr' | 'csc' | 'dense_colmajor' of the n x d example matrix X."""
    layout: str
    n: int
    d: int
    ptr: Optional[np.ndarray]
    idx: Optional[np.ndarray]
    val: np.ndarray

    @staticmethod
    def from_problem(p) -> "Matrix":
        """From a datagen.Problem (tensors are moved to host numpy)."""
        g = lambda t: None if t is None else t.detach().cpu().numpy()
        # (a problem without a value array is pattern-only data: every stored value is 1)
        val = _f32(g(p.val)) if p.val is not None else np.ones(int(p.idx.numel()), dtype=np.float32)
        return Matrix(p.layout, p.n, p.d,
                      None if p.ptr is None else _i64(g(p.ptr)),
                      None if p.idx is None else _i32(g(p.idx)), val)

    # products --------------------------------------------------------------------------------
    def matvec(self, x: np.ndarray) -> np.ndarray:
        """X x  (length n)."""
        x = _f64(x)
        out = np.empty(self.n, dtype=np.float64)
        if self.layout == "csr":
            lib().oracle_compressed_matvec(C.c_int64(self.n), C.c_int64(self.n), _p(self.ptr), _p(self.idx),
                                           _p(self.val), _p(x), C.c_int(0), _p(out))
        elif self.layout == "csc":
            lib().oracle_compressed_matvec(C.c_int64(self.d), C.c_int64(self.n), _p(self.ptr), _p(self.idx),
                                           _p(self.val), _p(x), C.c_int(1), _p(out))
        else:
            lib().oracle_dense_matvec(C.c_int64(self.n), C.c_int64(self.d), _p(self.val), _p(x), C.c_int(0), _p(out))
        return out

    def rmatvec(self, u: np.ndarray) -> np.ndarray:
        """X^T u  (length d)."""
        u = _f64(u)
        out = np.empty(self.d, dtype=np.float64)
        if self.layout == "csr":
            lib().oracle_compressed_matvec(C.c_int64(self.n), C.c_int64(self.d), _p(self.ptr), _p(self.idx),
                                           _p(self.val), _p(u), C.c_int(1), _p(out))
        elif self.layout == "csc":
            lib().oracle_compressed_matvec(C.c_int64(self.d), C.c_int64(self.d), _p(self.ptr), _p(self.idx),
                                           _p(self.val), _p(u), C.c_int(0), _p(out))
        else:
            lib().oracle_dense_matvec(C.c_int64(self.n), C.c_int64(self.d), _p(self.val), _p(u), C.c_int(1), _p(out))
        return out

    def to_dense(self) -> np.ndarray:
        X = np.zeros((self.n, self.d), dtype=np.float64)
        if self.layout == "dense_colmajor":
            return self.val.reshape(self.d, self.n).T.astype(np.float64)
        major = self.n if self.layout == "csr" else self.d
        for s in range(major):
            for k in range(self.ptr[s], self.ptr[s + 1]):
                if self.layout == "csr":
                    X[s, self.idx[k]] += self.val[k]
                else:
                    X[self.idx[k], s] += self.val[k]
        return X


class Solver:
    """Sequential SCD on one problem.  form: 'primal' (CSC / dense, ridge or logistic) or 'dual'
    (CSR, hinge or logistic).  State starts at zero (Algorithm 1's starting point); the logistic dual
    at alpha = 1/2."""

    GROUP_ORDER_CHUNK = 0xFFFFFFFF     # chunk id under which the order of the chunks is drawn

    def __init__(self, A: Matrix, y, loss: str, lam: float, chunk_bounds: Optional[Sequence[int]] = None,
                 shuffle_chunks: bool = False, lam1: float = 0.0):
        self.A, self.y, self.loss, self.lam, self.lam1 = A, _f32(y), LOSS_ID[loss], float(lam), float(lam1)
        if lam1 != 0.0 and A.layout == "csr":
            raise ValueError("the l1 term belongs to the primal forms")
        if A.layout == "csr":
            if loss == "ridge":
                raise ValueError("dual form is implemented for the hinge and logistic losses")
            self.form, self.m, self.vlen = "dual", A.n, A.d
        else:
            if loss == "hinge":
                raise ValueError("hinge loss is solved in the dual form (CSR)")
            self.form, self.m, self.vlen = "primal", A.d, A.n
        self.x = np.zeros(self.m, dtype=np.float64)      # w (primal) or alpha (dual)
        self.v = np.zeros(self.vlen, dtype=np.float64)   # shared vector
        if self.form == "dual" and loss == "logistic":
            # the entropy term needs alpha inside (0,1): start at 1/2, v = X^T (y o alpha)
            self.x[:] = 0.5
            self.v = A.rmatvec(self.y.astype(np.float64) * self.x)
        # streaming: coordinates are visited chunk by chunk, permuted inside each chunk
        self.bounds = [0, self.m] if chunk_bounds is None else list(chunk_bounds)
        # shuffle_chunks: the chunks themselves are visited in a seeded random order (their keys under
        # the reserved chunk id, sorted), not 0, 1, 2, ...
        self.shuffle_chunks = shuffle_chunks
        self.last_perm = None

    def epoch(self, seed: int, chunks: Optional[Sequence[int]] = None):
        """One pass over all chunks, or (Section 3.2, processing only part of the data in a round) over
        the given chunks only, in the given order."""
        L = lib()
        n = C.c_int64(self.A.n)
        perms = []
        nch = len(self.bounds) - 1
        order = permutation(seed, nch, chunk=self.GROUP_ORDER_CHUNK) if self.shuffle_chunks else range(nch)
        if chunks is not None:
            order = list(chunks)
            assert len(set(order)) == len(order) and all(0 <= int(c) < nch for c in order)
        for ch in order:
            ch = int(ch)
            c0, c1 = self.bounds[ch], self.bounds[ch + 1]
            perm = permutation(seed, c1 - c0, chunk=ch)
            perms.append(perm.astype(np.int64) + c0)
            tail = (_p(perm), C.c_int64(c0), C.c_int64(c1 - c0), _p(self.x), _p(self.v))
            if self.form == "dual":
                fn = L.oracle_epoch_dual_hinge if self.loss == HINGE else L.oracle_epoch_dual_logistic
                fn(n, _p(self.A.ptr), _p(self.A.idx), _p(self.A.val), _p(self.y), C.c_double(self.lam), *tail)
            elif self.A.layout == "csc":
                L.oracle_epoch_primal_sparse(C.c_int(self.loss), n, _p(self.A.ptr), _p(self.A.idx), _p(self.A.val),
                                             _p(self.y), C.c_double(self.lam), C.c_double(self.lam1), *tail)
            else:
                L.oracle_epoch_primal_dense(C.c_int(self.loss), n, _p(self.A.val), _p(self.y), C.c_double(self.lam),
                                            C.c_double(self.lam1), *tail)
        self.last_perm = np.concatenate(perms) if perms else np.zeros(0, dtype=np.int64)

    def visit(self, order):
        """Sequential updates of the listed coordinates (absolute numbers), one after the other in the
        order given -- a pass in an order that the caller fixes instead of a seeded permutation."""
        L = lib()
        n = C.c_int64(self.A.n)
        perm = np.ascontiguousarray(order, dtype=np.uint32)
        tail = (_p(perm), C.c_int64(0), C.c_int64(perm.size), _p(self.x), _p(self.v))
        if self.form == "dual":
            fn = L.oracle_epoch_dual_hinge if self.loss == HINGE else L.oracle_epoch_dual_logistic
            fn(n, _p(self.A.ptr), _p(self.A.idx), _p(self.A.val), _p(self.y), C.c_double(self.lam), *tail)
        elif self.A.layout == "csc":
            L.oracle_epoch_primal_sparse(C.c_int(self.loss), n, _p(self.A.ptr), _p(self.A.idx), _p(self.A.val),
                                         _p(self.y), C.c_double(self.lam), C.c_double(self.lam1), *tail)
        else:
            L.oracle_epoch_primal_dense(C.c_int(self.loss), n, _p(self.A.val), _p(self.y), C.c_double(self.lam),
                                        C.c_double(self.lam1), *tail)
        self.last_perm = perm.astype(np.int64)

    # model ----------------------------------------------------------------------------------
    def weights(self) -> np.ndarray:
        return self.x.copy() if self.form == "primal" else self.v / (self.lam * self.A.n)

    def shared_from_model(self) -> np.ndarray:
        """v recomputed from the model by the definition v = A alpha."""
        if self.form == "primal":
            return self.A.matvec(self.x)
        return self.A.rmatvec(self.y.astype(np.float64) * self.x)

    # objectives -----------------------------------------------------------------------------
    def primal(self) -> float:
        if self.form == "primal":
            return primal_objective(self.loss, self.v, self.y, self.x, self.lam, self.lam1)
        return self.primal_dual()[0]

    def primal_dual(self):
        assert self.form == "dual"
        w = self.weights()
        xw = self.A.matvec(w)
        P, D = C.c_double(), C.c_double()
        fn = lib().oracle_hinge_primal_dual if self.loss == HINGE else lib().oracle_logistic_primal_dual
        fn(C.c_int64(self.A.n), C.c_int64(self.A.d), _p(self.x), _p(self.v), _p(xw), _p(self.y),
           C.c_double(self.lam), C.byref(P), C.byref(D))
        return P.value, D.value

    def dual(self) -> float:
        assert self.form == "dual"
        fn = lib().oracle_hinge_dual_objective if self.loss == HINGE else lib().oracle_logistic_dual_objective
        return float(fn(C.c_int64(self.A.n), C.c_int64(self.A.d), _p(self.x), _p(self.v), C.c_double(self.lam)))

    def gap(self, form: str = "gradient") -> float:
        if self.form == "dual":
            P, D = self.primal_dual()
            return P - D
        if self.lam1 != 0.0:
            form = "fenchel"              # the gradient form needs a differentiable regulariser
        return primal_gap(self.A, self.loss, self.v, self.y, self.x, self.lam, form, self.lam1)

    def chunk_gaps(self) -> np.ndarray:
        """Share of every chunk in the duality gap at the current state: the sum of its coordinates'
        shares (primal_gap_shares, dual_gap_shares)."""
        if self.form == "primal":
            share = primal_gap_shares(self.A, self.loss, self.v, self.y, self.x, self.lam, self.lam1)
        else:
            share = dual_gap_shares(self.A, self.loss, self.x, self.v, self.y, self.lam)
        return np.array([share[self.bounds[c]:self.bounds[c + 1]].sum() for c in range(len(self.bounds) - 1)])

    def predict(self, X: Matrix) -> np.ndarray:
        return X.matvec(self.weights())


def primal_objective(loss: int, z, y, w, lam: float, lam1: float = 0.0) -> float:
    z, w, y = _f64(z), _f64(w), _f32(y)
    return float(lib().oracle_primal_objective(C.c_int(loss), C.c_int64(z.size), C.c_int64(w.size), _p(z), _p(y),
                                               _p(w), C.c_double(lam), C.c_double(lam1)))


def primal_gap(A: Matrix, loss: int, v, y, w, lam: float, form: str = "gradient", lam1: float = 0.0) -> float:
    v, w, y = _f64(v), _f64(w), _f32(y)
    u = np.empty(A.n, dtype=np.float64)
    lib().oracle_primal_dual_candidate(C.c_int(loss), C.c_int64(A.n), _p(v), _p(y), _p(u))
    xtu = A.rmatvec(u)
    if form == "gradient":
        return float(lib().oracle_primal_gap_gradient(C.c_int64(A.d), _p(w), _p(xtu), C.c_double(lam)))
    return float(lib().oracle_primal_gap_fenchel(C.c_int(loss), C.c_int64(A.n), C.c_int64(A.d), _p(v), _p(y),
                                                 _p(w), _p(u), _p(xtu), C.c_double(lam), C.c_double(lam1)))


def primal_gap_shares(A: Matrix, loss: int, v, y, w, lam: float, lam1: float = 0.0) -> np.ndarray:
    """The duality gap of eq. (1) coordinate by coordinate (the importance measure of the scheme that
    Section 3.2 cites for choosing what to process).  With the dual candidate u = grad f(v) the loss part
    of the Fenchel gap vanishes (f(v) + f*(u) = <u, v>) and what is left is a sum over the coordinates,
        share_j = g_j(w_j) + g_j*(-z_j) + w_j z_j,   z_j = a_j . u,
    each term non-negative by the Fenchel-Young inequality and zero exactly when w_j minimises the
    objective along coordinate j's direction for this u.  Here g_j(w) = (lam/2) w^2 + lam1 |w| and
    g_j*(t) = max(|t| - lam1, 0)^2 / (2 lam)."""
    v, w, y = _f64(v), _f64(w), _f32(y)
    u = np.empty(A.n, dtype=np.float64)
    lib().oracle_primal_dual_candidate(C.c_int(loss), C.c_int64(A.n), _p(v), _p(y), _p(u))
    z = A.rmatvec(u)
    gstar = np.maximum(np.abs(z) - lam1, 0.0) ** 2 / (2.0 * lam)
    return 0.5 * lam * w * w + lam1 * np.abs(w) + gstar + w * z


def dual_gap_shares(A: Matrix, loss: int, alpha, v, y, lam: float) -> np.ndarray:
    """The gap P(w(alpha)) - D(alpha) of the dual forms example by example.  With w = v / (lam n) the
    regulariser's part is lam ||w||^2 = (1/n) sum_i alpha_i m_i, m_i = y_i x_i . w, so
        P - D = (1/n) sum_i [ l(m_i) + l*(-alpha_i) + alpha_i m_i ],
    each bracket non-negative by the Fenchel-Young inequality.  Hinge: l(m) = max(0, 1 - m),
    l*(-a) = -a on [0, 1]; logistic: l(m) = log(1 + exp(-m)), l*(-a) = a ln a + (1 - a) ln(1 - a)."""
    alpha, v, y = _f64(alpha), _f64(v), _f32(y).astype(np.float64)
    n = A.n
    m = y * A.matvec(v / (lam * n))
    if loss == HINGE:
        term = np.maximum(0.0, 1.0 - m) - alpha
    else:
        with np.errstate(divide="ignore", invalid="ignore"):
            ent = np.where(alpha > 0, alpha * np.log(alpha), 0.0) + np.where(alpha < 1, (1 - alpha) * np.log1p(-alpha), 0.0)
        term = np.logaddexp(0.0, -m) + ent
    return (term + alpha * m) / n


def select_chunks(shares, keep: int):
    """The `keep` chunks with the largest shares, largest first; equal shares in index order."""
    order = sorted(range(len(shares)), key=lambda c: (-float(shares[c]), c))
    return order[:keep]


def solve_selected(s: "Solver", seed0: int, max_passes: int, gap_tol: float, refresh_every: int, keep: int):
    """Gap-based selection of the chunks to process (Section 3.2): every `refresh_every`-th pass visits
    all chunks and is followed by an evaluation of the chunks' gap shares (their sum is the gap: the
    stopping test); the passes in between visit only the `keep` chunks whose shares were largest.
    Returns (passes done, chunk visits, last gap)."""
    visits, gap, p = 0, float("inf"), 0
    chosen = list(range(len(s.bounds) - 1))
    while p < max_passes:
        full = p % refresh_every == 0
        s.epoch(seed0 + p, None if full else chosen)
        visits += (len(s.bounds) - 1) if full else len(chosen)
        p += 1
        if full:
            shares = s.chunk_gaps()
            gap = float(shares.sum())
            if gap <= gap_tol:
                break
            chosen = select_chunks(shares, keep)
    return p, visits, gap


def solve(A: Matrix, y, loss: str, lam: float, epochs: int, seed0: int = 0, tol: Optional[float] = None,
          chunk_bounds=None, shuffle_chunks: bool = False, lam1: float = 0.0) -> Solver:
    """Run `epochs` passes with permutation seeds seed0, seed0+1, ...; stop early when the gap
    falls below tol * max(1, |P|)."""
    s = Solver(A, y, loss, lam, chunk_bounds, shuffle_chunks, lam1)
    for e in range(epochs):
        s.epoch(seed0 + e)
        if tol is not None and (e % 5 == 4 or e == epochs - 1):
            if s.gap() <= tol * max(1.0, abs(s.primal())):
                break
    return s
