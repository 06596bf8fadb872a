"""ctypes front end of the fp64 PageRank oracle (oracle/pagerank.c) and of its fp32, timed sibling
(oracle/pagerank_f32.c).  Test infrastructure only."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pagerank.c")
_SRC32 = os.path.join(_HERE, "pagerank_f32.c")
_LIB = os.path.join(_HERE, "liboracle_pagerank.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pagerank.c and pagerank_f32.c with gcc into a shared library beside them; returns its path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC32))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, _SRC32])
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
        L.oracle_pagerank_fp32.argtypes = [ctypes.c_int64, i32p, i32p, i32p, ctypes.c_float, ctypes.c_int,
                                           ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
        L.oracle_pagerank_fp32.restype = ctypes.c_int
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


def pagerank_f32(row_ptr, col, out_degree, damping: float, iterations: int, n_threads: int = 0, return_threads=False):
    """The same iteration with fp32 ranks and row sums, rows dealt to threads: the timed CPU baseline."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    out_degree = np.ascontiguousarray(out_degree, dtype=np.int32)
    V = row_ptr.shape[0] - 1
    if out_degree.shape[0] != V or int(row_ptr[-1]) != col.shape[0]:
        raise ValueError("inconsistent CSR")
    out = np.empty(V, dtype=np.float32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    colp = col.ctypes.data_as(i32p) if col.size else ctypes.cast(None, i32p)
    used = _load().oracle_pagerank_fp32(V, row_ptr.ctypes.data_as(i32p), colp, out_degree.ctypes.data_as(i32p),
                                        float(damping), int(iterations), int(n_threads),
                                        out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if used < 0:
        raise RuntimeError("oracle_pagerank_fp32 failed: %d" % used)
    return (out, used) if return_threads else out
