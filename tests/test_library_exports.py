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
    assert C.sizeof(snap.binding.SnapOptions) == 8 + 8 + 8 + 8 + 8 + 4 + 4 + 4 + 4 + 8 + 8 + 8
    assert C.sizeof(snap.binding.SnapEpochStats) == 16 + 32 + 8 + 4 + 4 + 4 + 4 + 8 + 8
