"""The C-ABI library loads and exports every function include/freeride.h declares (no compute calls here)."""
import ctypes
import os
import re
import subprocess

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


STRUCTS = ["fr_config", "fr_step", "fr_task_ops", "fr_task_profile", "fr_progress", "fr_event", "fr_pagerank_desc", "fr_pagerank_info_t", "fr_sgd_desc", "fr_sgd_info_t",
           "fr_load_desc", "fr_stage_desc", "fr_stage_op", "fr_epoch_result"]


def test_struct_sizes_match_the_header_layout(tmp_path):
    # the C compiler's view of the header against the ctypes structures of the binding
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "freeride.h"\nint main(void) {\n' +
                   "".join('  printf("%s %%zu\\n", sizeof(%s));\n' % (n, n) for n in STRUCTS) + "  return 0;\n}\n")
    exe = tmp_path / "sizes"
    include = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-std=c11", "-I", include, str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    sizes = dict((line.split()[0], int(line.split()[1])) for line in out.splitlines())
    for n in STRUCTS:
        assert ctypes.sizeof(getattr(fr.binding, n)) == sizes[n], n
    assert sizes["fr_config"] == 4 + 4 + 32 + 8 * 4 + 4 * 6 + 8
    assert sizes["fr_progress"] == 8 + 14 * 8
    assert sizes["fr_step"] == 64
