"""The C-ABI library loads and exports every function include/freeride.h declares (no compute calls here)."""
import ctypes
import os
import re

import paper_2409_06941_amd as fr

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "freeride.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(fr_[a-z0-9_]+)\s*\(", text))
    return {n for n in names if not n.endswith("_fn")}


def test_every_declared_function_is_exported_and_bound():
    declared = _declared_functions()
    assert len(declared) >= 30
    L = ctypes.CDLL(fr.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(L, name), "library does not export %s" % name
    assert declared == set(fr.binding.SIGNATURES), declared ^ set(fr.binding.SIGNATURES)


def test_struct_sizes_match_the_header_layout():
    # natural alignment, as a C compiler lays the header's structs out
    assert ctypes.sizeof(fr.fr_config) == 4 + 4 + 32 + 8 * 4 + 4 * 4
    assert ctypes.sizeof(fr.fr_step) == 8 + 8 + 4 * 4 + 4 + 4
    assert ctypes.sizeof(fr.fr_event) == 6 * 4 + 4 * 8
    assert ctypes.sizeof(fr.fr_progress) == 8 + 12 * 8
    assert ctypes.sizeof(fr.fr_stage_op) == 8 + 3 * 8
