"""The C-ABI library loads and exports every symbol include/snap.h declares (no GPU needed)."""
import os
import re

import paper_1803_06333_amd as snap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    if not os.path.exists(snap.binding.LIB_PATH):
        from paper_1803_06333_amd.build import build
        build()
    lib = snap.load_library()
    header = open(os.path.join(ROOT, "include", "snap.h")).read()
    declared = set(re.findall(r"\b(snap_[a-z_]+)\s*\(", header))
    declared -= {"snap_matrix", "snap_options", "snap_handle", "snap_epoch_stats"}
    assert declared == set(snap.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_sizes_match_header_layout():
    import ctypes as C
    assert C.sizeof(snap.binding.SnapMatrix) == 4 + 4 + 3 * 8 + 3 * 8
    assert C.sizeof(snap.binding.SnapOptions) == 8 + 8 + 8 + 8 + 8 + 4 + 4 + 4 + 4 + 8 + 8 + 8 + 8 + 8 + 8
    assert C.sizeof(snap.binding.SnapEpochStats) == 16 + 32 + 8 + 4 + 4 + 4 + 4 + 8 + 8 + 4 + 4 + 4 + 4   # (the last 4: padding)


def test_create_without_a_gpu_reports_an_error_instead_of_crashing():
    """Host logic: argument checks come first; with no device the HIP failure is a return code."""
    import numpy as np
    import pytest
    import torch
    ptr = np.array([0, 1, 2], dtype=np.int64)
    idx = np.array([0, 1], dtype=np.int32)
    val = np.ones(2, dtype=np.float32)
    y = np.array([1.0, -1.0], dtype=np.float32)
    with pytest.raises(snap.SnapError) as e:                       # checked before any device call
        snap.Solver("csc", 2, 2, ptr, idx, val, y, "hinge", 0.1)
    assert e.value.code == -2
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 2, 2, ptr, idx, val, y, "ridge", 0.0)
    assert e.value.code == -1
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csr", 2, 2, ptr, idx, val, y, "ridge", 0.1)   # ridge needs the primal form, CSR gives the dual
    assert e.value.code == -2
    if not torch.cuda.is_available():
        with pytest.raises(snap.SnapError) as e:
            snap.Solver("csc", 2, 2, ptr, idx, val, y, "ridge", 0.1)
        assert e.value.code in (-4, -3)


def test_host_side_epoch_order_matches_the_known_answers_and_the_oracle():
    """The library's own key generator and block order, called on the host (no device), against the
    fixture written from the oracle and against the oracle directly: the two implement the same
    counter-based generator separately."""
    import numpy as np
    import oracle
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "perm_known_answers.txt")) if l[0] != "#"]
    n_checked = 0
    for kind, seed, chunk, m, *vals in rows:
        if kind != "keys":
            continue
        got = [snap.perm_key(int(seed), int(chunk), c) for c in range(16)]
        assert got == [int(v) for v in vals]
        n_checked += 1
    assert n_checked >= 4
    rng = np.random.default_rng(0)
    for seed, chunk in [(0, 0), (7, 3), (2 ** 64 - 1, 2 ** 32 - 1), (180306333, 12345)]:
        for c in [0, 1, 63, 64, 4095, 2 ** 31, 2 ** 32 - 1] + rng.integers(0, 2 ** 32, 20).tolist():
            assert snap.perm_key(seed, chunk, int(c)) == oracle.lib().oracle_key(seed, chunk, int(c))
    for seed, nb in [(0, 1), (5, 2), (42, 39), (9, 1000), (2 ** 63, 4097)]:
        want = oracle.permutation(seed, nb, chunk=oracle.Solver.GROUP_ORDER_CHUNK)
        assert snap.block_order(seed, nb) == want.tolist()
    assert snap.block_order(3, 0) == []
