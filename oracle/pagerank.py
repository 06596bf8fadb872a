"""ctypes front end of the fp64 PageRank oracle (oracle/pagerank.c).  Test infrastructure only."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pagerank.c")
_LIB = os.path.join(_HERE, "liboracle_pagerank.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pagerank.c with gcc into a shared library beside it; returns its path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.oracle_pagerank_fp64.argtypes = [ctypes.c_int64, i32p, i32p, i32p, ctypes.c_double, ctypes.c_int,
                                           ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
        L.oracle_pagerank_fp64.restype = ctypes.c_int
        _lib = L
    return _lib


def pagerank(row_ptr, col, out_degree, damping: float, iterations: int, n_threads: int = 0, return_threads=False):
    """Ranks after exactly `iterations` Jacobi power iterations, fp64, dangling mass spread uniformly.

    row_ptr / col: in-edge CSR (int32; col holds the sources of each row's in-edges); out_degree: int32 per vertex.
    """
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    out_degree = np.ascontiguousarray(out_degree, dtype=np.int32)
    V = row_ptr.shape[0] - 1
    if out_degree.shape[0] != V or int(row_ptr[-1]) != col.shape[0]:
        raise ValueError("inconsistent CSR")
    out = np.empty(V, dtype=np.float64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    colp = col.ctypes.data_as(i32p) if col.size else ctypes.cast(None, i32p)
    used = _load().oracle_pagerank_fp64(V, row_ptr.ctypes.data_as(i32p), colp, out_degree.ctypes.data_as(i32p),
                                        float(damping), int(iterations), int(n_threads),
                                        out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if used < 0:
        raise RuntimeError("oracle_pagerank_fp64 failed: %d" % used)
    return (out, used) if return_threads else out
