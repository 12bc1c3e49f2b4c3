"""ctypes binding of libsnap (include/snap.h).  Argument marshalling only: every step of the
solver runs in the HIP library.  Matrices and labels may be torch tensors (CPU, pinned or on the
GPU) or numpy arrays; their memory space is passed along as the header describes."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

try:  # torch is only used to recognise tensors and read their pointers
    import torch
except Exception:  # pragma: no cover
    torch = None

from .build import LIB_PATH

CSR, CSC, DENSE_ROWMAJOR, DENSE_COLMAJOR = 0, 1, 2, 3
RIDGE, LOGISTIC, HINGE = 0, 1, 2
FORM_AUTO, PRIMAL, DUAL = 0, 1, 2
MEM_HOST, MEM_HOST_PINNED, MEM_DEVICE = 0, 1, 2
LAYOUTS = {"csr": CSR, "csc": CSC, "dense_rowmajor": DENSE_ROWMAJOR, "dense_colmajor": DENSE_COLMAJOR}
LOSSES = {"ridge": RIDGE, "logistic": LOGISTIC, "hinge": HINGE}

EXPORTS = ["snap_create", "snap_epoch", "snap_objective", "snap_duality_gap", "snap_predict", "snap_get_model",
           "snap_set_model", "snap_get_shared", "snap_recompute_shared", "snap_get_perm", "snap_get_epoch_stats",
           "snap_get_dims", "snap_get_chunks", "snap_get_stream_bytes", "snap_solve", "snap_perm_key", "snap_block_order",
           "snap_epoch_chunks", "snap_chunk_gaps", "snap_solve_selected", "snap_get_bytes_copied", "snap_last_error",
           "snap_destroy", "snap_predict_static", "snap_stream_probe"]


class SnapMatrix(C.Structure):
    _fields_ = [("layout", C.c_int), ("mem", C.c_int), ("n_rows", C.c_int64), ("n_cols", C.c_int64),
                ("nnz", C.c_int64), ("ptr", C.c_void_p), ("idx", C.c_void_p), ("val", C.c_void_p)]


class SnapOptions(C.Structure):
    _fields_ = [("form", C.c_int), ("device_budget_bytes", C.c_size_t), ("chunk_bytes", C.c_size_t),
                ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p), ("refresh_v_every", C.c_int),
                ("profile", C.c_int), ("adaptive", C.c_int), ("damping", C.c_float),
                ("max_inflight_nnz", C.c_int64), ("group_bounds", C.c_void_p), ("n_groups", C.c_int64),
                ("lambda1", C.c_double), ("dense_tiles", C.c_int), ("auto_groups", C.c_int), ("host_keys", C.c_int)]


class SnapEpochStats(C.Structure):
    _fields_ = [("epoch_ms", C.c_float), ("scd_ms", C.c_float), ("perm_ms", C.c_float), ("copy_ms", C.c_float),
                ("n_chunks", C.c_int64), ("n_small", C.c_int64), ("n_large", C.c_int64), ("n_items", C.c_int64),
                ("inflight_nnz", C.c_int64), ("damping", C.c_float), ("rejected", C.c_int),
                ("large_ms", C.c_float), ("small_ms", C.c_float), ("nnz_large", C.c_int64), ("nnz_small", C.c_int64),
                ("row_map_bytes", C.c_int), ("unit_values", C.c_int), ("byte_map_groups", C.c_int)]


class SnapError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libsnap error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load_library():
    """Load the built HIP library; there is no fallback path."""
    global _lib
    if _lib is None:
        path = LIB_PATH
        if not os.path.exists(path):
            raise ImportError("libsnap.so is not built (%s); run `python -m paper_1803_06333_amd.build` or "
                              "__graft_entry__.build()" % LIB_PATH)
        L = C.CDLL(path)
        L.snap_last_error.restype = C.c_char_p
        L.snap_destroy.restype = None
        L.snap_destroy.argtypes = [C.c_void_p]
        L.snap_create.argtypes = [C.POINTER(SnapMatrix), C.c_void_p, C.c_int, C.c_double, C.POINTER(SnapOptions),
                                  C.POINTER(C.c_void_p)]
        L.snap_epoch.argtypes = [C.c_void_p, C.c_uint64]
        L.snap_objective.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.snap_duality_gap.argtypes = [C.c_void_p, C.POINTER(C.c_double)]
        L.snap_predict.argtypes = [C.c_void_p, C.POINTER(SnapMatrix), C.c_void_p]
        L.snap_predict_static.argtypes = [C.c_void_p, C.POINTER(SnapMatrix), C.c_void_p]
        L.snap_get_model.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.snap_set_model.argtypes = [C.c_void_p, C.c_void_p]
        L.snap_get_shared.argtypes = [C.c_void_p, C.c_void_p]
        L.snap_recompute_shared.argtypes = [C.c_void_p]
        L.snap_get_perm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.snap_get_epoch_stats.argtypes = [C.c_void_p, C.POINTER(SnapEpochStats)]
        L.snap_get_dims.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.snap_get_chunks.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.c_void_p]
        L.snap_solve.argtypes = [C.c_void_p, C.c_uint64, C.c_int64, C.c_double, C.c_int64, C.POINTER(C.c_int64),
                                 C.POINTER(C.c_double)]
        L.snap_epoch_chunks.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int64]
        L.snap_chunk_gaps.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        L.snap_solve_selected.argtypes = [C.c_void_p, C.c_uint64, C.c_int64, C.c_double, C.c_int64, C.c_int64,
                                          C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        L.snap_get_bytes_copied.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.snap_perm_key.restype = C.c_uint32
        L.snap_perm_key.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.snap_block_order.argtypes = [C.c_uint64, C.c_int64, C.c_void_p]
        L.snap_stream_probe.argtypes = [C.c_int, C.c_int64, C.c_int, C.c_void_p, C.POINTER(C.c_double)]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise SnapError(rc, load_library().snap_last_error().decode())


def _describe(a, dtype_np, dtype_name):
    """(pointer, mem space, keepalive object) of a tensor / array, which must already have the
    right dtype and be contiguous."""
    if a is None:
        return None, None, None
    if torch is not None and isinstance(a, torch.Tensor):
        if str(a.dtype) != "torch." + dtype_name or not a.is_contiguous():
            raise TypeError("expected a contiguous %s tensor, got %s" % (dtype_name, a.dtype))
        mem = MEM_DEVICE if a.is_cuda else (MEM_HOST_PINNED if a.is_pinned() else MEM_HOST)
        return a.data_ptr(), mem, a
    a = np.ascontiguousarray(a, dtype=dtype_np)
    return a.ctypes.data, MEM_HOST, a


def make_matrix(layout: str, n_rows: int, n_cols: int, ptr, idx, val):
    """snap_matrix for the given arrays; returns (struct, keepalive)."""
    pp, m1, k1 = _describe(ptr, np.int64, "int64")
    pi, m2, k2 = _describe(idx, np.int32, "int32")
    pv, m3, k3 = _describe(val, np.float32, "float32")
    mems = {m for m in (m1, m2, m3) if m is not None}
    if MEM_DEVICE in mems and len(mems) > 1:
        raise ValueError("matrix arrays must live in one memory space")
    mem = MEM_DEVICE if MEM_DEVICE in mems else (MEM_HOST_PINNED if mems == {MEM_HOST_PINNED} else MEM_HOST)
    count_of = lambda k: int(k.numel() if hasattr(k, "numel") else k.size)
    nnz = count_of(k3) if k3 is not None else count_of(k2)       # (val = None: pattern-only data, snap_create only)
    sm = SnapMatrix(LAYOUTS[layout], mem, n_rows, n_cols, nnz, pp, pi, pv)
    return sm, (k1, k2, k3)


def perm_key(seed: int, chunk: int, c: int) -> int:
    """Key of coordinate c of a chunk under the seed (host function of the library)."""
    return int(load_library().snap_perm_key(seed, chunk, c))


def block_order(seed: int, n_blocks: int) -> list:
    """Visiting order of the groups / tiles of an epoch with this seed (host function of the library)."""
    out = np.empty(max(n_blocks, 1), dtype=np.int64)
    _check(load_library().snap_block_order(seed, n_blocks, out.ctypes.data))
    return out[:n_blocks].tolist()


def stream_probe(kind: int, rows: int, passes: int = 40) -> float:
    """snap_stream_probe: microseconds per pass of a bare streaming kernel (0 read, 1 copy, 2 the row pass's mix)."""
    us = C.c_double()
    _check(load_library().snap_stream_probe(kind, rows, passes, None, C.byref(us)))
    return us.value


class Solver:
    """Thin handle wrapper: snap_create ... snap_destroy."""

    def __init__(self, layout: str, n_rows: int, n_cols: int, ptr, idx, val, y, loss: str, lam: float,
                 form: int = FORM_AUTO, device_budget_bytes: int = 0, chunk_bytes: int = 0, compute_stream: int = 0,
                 copy_stream: int = 0, refresh_v_every: int = 0, profile: bool = False, adaptive=None,
                 damping: float = 0.0, max_inflight_nnz: int = 0, group_bounds=None, lam1: float = 0.0,
                 dense_tiles=None, auto_groups=None, host_keys: bool = False):
        self._lib = load_library()
        self._h = C.c_void_p()
        if torch is not None and isinstance(val, torch.Tensor) and val.is_cuda:
            torch.cuda.synchronize(val.device)       # the library reads the tensors on its own stream
        sm, self._keep = make_matrix(layout, n_rows, n_cols, ptr, idx, val)
        py, my, ky = _describe(y, np.float32, "float32")
        if (my == MEM_DEVICE) != (sm.mem == MEM_DEVICE):
            raise ValueError("labels must live in the memory space of the matrix")
        opt = SnapOptions()
        opt.form, opt.device_budget_bytes, opt.chunk_bytes = form, device_budget_bytes, chunk_bytes
        opt.compute_stream, opt.copy_stream = compute_stream or None, copy_stream or None
        opt.refresh_v_every, opt.profile = refresh_v_every, int(profile)
        opt.adaptive = 0 if adaptive is None else (1 if adaptive else 2)
        opt.damping, opt.max_inflight_nnz, opt.lambda1 = damping, max_inflight_nnz, lam1
        opt.dense_tiles = 0 if dense_tiles is None else (1 if dense_tiles else 2)
        opt.auto_groups = 0 if auto_groups is None else (1 if auto_groups else 2)
        opt.host_keys = int(bool(host_keys))
        if group_bounds is not None:
            gb = np.ascontiguousarray(group_bounds, dtype=np.int64)
            opt.group_bounds, opt.n_groups = gb.ctypes.data, gb.size - 1
        self._keep_stream = (self._keep, ky)
        _check(self._lib.snap_create(C.byref(sm), py, LOSSES[loss], lam, C.byref(opt), C.byref(self._h)))
        m, vl = C.c_int64(), C.c_int64()
        _check(self._lib.snap_get_dims(self._h, C.byref(m), C.byref(vl)))
        self.n_coords, self.shared_len, self.n_rows, self.n_cols = m.value, vl.value, n_rows, n_cols
        if device_budget_bytes == 0:
            self._keep = self._keep_stream = None     # resident mode copied everything

    @classmethod
    def from_problem(cls, p, **kw) -> "Solver":
        """From a datagen.Problem."""
        return cls(p.layout, p.n, p.d, p.ptr, p.idx, p.val, p.y, p.loss, p.lam, **kw)

    def close(self):
        if self._h:
            self._lib.snap_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def epoch(self, perm_seed: int):
        _check(self._lib.snap_epoch(self._h, C.c_uint64(perm_seed)))

    def objective(self, want_dual: bool = False):
        P, D = C.c_double(), C.c_double()
        _check(self._lib.snap_objective(self._h, C.byref(P), C.byref(D) if want_dual else None))
        return (P.value, D.value) if want_dual else P.value

    def duality_gap(self) -> float:
        G = C.c_double()
        _check(self._lib.snap_duality_gap(self._h, C.byref(G)))
        return G.value

    def predict(self, layout: str, n_rows: int, ptr, idx, val):
        sm, keep = make_matrix(layout, n_rows, self.n_cols, ptr, idx, val)
        if sm.mem == MEM_DEVICE:
            torch.cuda.synchronize(keep[2].device)   # the library reads the tensors on its own stream
            out = torch.empty(n_rows, dtype=torch.float32, device=keep[2].device)
            _check(self._lib.snap_predict(self._h, C.byref(sm), out.data_ptr()))
            return out
        out = np.empty(n_rows, dtype=np.float32)
        _check(self._lib.snap_predict(self._h, C.byref(sm), out.ctypes.data))
        return out

    def predict_static(self, layout: str, n_rows: int, ptr, idx, val, out):
        """snap_predict_static: device tensors in, a caller-allocated device tensor out, nothing allocated."""
        sm, keep = make_matrix(layout, n_rows, self.n_cols, ptr, idx, val)
        if torch is not None and isinstance(out, torch.Tensor) and out.is_cuda:
            torch.cuda.synchronize(out.device)       # the library reads and writes the tensors on its own stream
        if str(out.dtype) != "torch.float32" or not out.is_contiguous() or out.numel() < n_rows:
            raise TypeError("out must be a contiguous float32 tensor with n_rows entries")
        _check(self._lib.snap_predict_static(self._h, C.byref(sm), out.data_ptr()))
        return out

    def model(self):
        """(w [n_cols], coordinate vector [n_coords]) as numpy arrays."""
        w = np.empty(self.n_cols, dtype=np.float32)
        x = np.empty(self.n_coords, dtype=np.float32)
        _check(self._lib.snap_get_model(self._h, w.ctypes.data, x.ctypes.data))
        return w, x

    def set_model(self, x):
        x = np.ascontiguousarray(x, dtype=np.float32)
        if x.size != self.n_coords:
            raise ValueError("coordinate vector has the wrong length")
        _check(self._lib.snap_set_model(self._h, x.ctypes.data))

    def shared(self) -> np.ndarray:
        v = np.empty(self.shared_len, dtype=np.float32)
        _check(self._lib.snap_get_shared(self._h, v.ctypes.data))
        return v

    def recompute_shared(self):
        _check(self._lib.snap_recompute_shared(self._h))

    def perm(self, want_keys: bool = False):
        p = np.empty(self.n_coords, dtype=np.uint32)
        k = np.empty(self.n_coords, dtype=np.uint32) if want_keys else None
        _check(self._lib.snap_get_perm(self._h, p.ctypes.data, k.ctypes.data if want_keys else None))
        return (p, k) if want_keys else p

    def chunk_bounds(self) -> list:
        n = C.c_int64()
        _check(self._lib.snap_get_chunks(self._h, C.byref(n), None))
        b = np.empty(n.value + 1, dtype=np.int64)
        _check(self._lib.snap_get_chunks(self._h, C.byref(n), b.ctypes.data))
        return b.tolist()

    def solve(self, seed0: int, max_epochs: int, gap_tol: float, check_every: int = 5):
        """Epochs with seeds seed0, seed0 + 1, ... until the duality gap is at most gap_tol: (epochs run, gap)."""
        e, g = C.c_int64(), C.c_double()
        _check(self._lib.snap_solve(self._h, seed0, max_epochs, gap_tol, check_every, C.byref(e), C.byref(g)))
        return e.value, g.value

    def epoch_chunks(self, perm_seed: int, chunks) -> None:
        """One pass over the listed chunks only, in that order."""
        c = np.ascontiguousarray(chunks, dtype=np.int64)
        _check(self._lib.snap_epoch_chunks(self._h, perm_seed, c.ctypes.data, c.size))

    def chunk_gaps(self) -> np.ndarray:
        """Share of every chunk in the duality gap at the current state."""
        out = np.empty(len(self.chunk_bounds()) - 1, dtype=np.float64)
        _check(self._lib.snap_chunk_gaps(self._h, out.ctypes.data, None))
        return out

    def solve_selected(self, seed0: int, max_passes: int, gap_tol: float, refresh_every: int, keep: int):
        """Passes that visit all chunks every refresh_every-th time and otherwise the `keep` chunks with
        the largest gap shares: (passes, chunk visits, last gap)."""
        p, v, g = C.c_int64(), C.c_int64(), C.c_double()
        _check(self._lib.snap_solve_selected(self._h, seed0, max_passes, gap_tol, refresh_every, keep, C.byref(p),
                                             C.byref(v), C.byref(g)))
        return p.value, v.value, g.value

    def bytes_copied(self) -> int:
        """Bytes of chunk copies from host memory enqueued since creation."""
        b = C.c_int64()
        _check(self._lib.snap_get_bytes_copied(self._h, C.byref(b)))
        return b.value

    def stream_bytes(self) -> int:
        """Bytes copied from host memory by one pass over the data (0: resident)."""
        b = C.c_int64()
        _check(self._lib.snap_get_stream_bytes(self._h, C.byref(b)))
        return b.value

    def epoch_stats(self) -> dict:
        s = SnapEpochStats()
        _check(self._lib.snap_get_epoch_stats(self._h, C.byref(s)))
        return {f: getattr(s, f) for f, _ in SnapEpochStats._fields_}
