"""Compile-and-load helper for the input generators' C file (gcc, OpenMP)."""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "graphgen.c")
_LIB = os.path.join(_HERE, "libgraphgen.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile graphgen.c into libgraphgen.so next to it; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = build()
        L = ctypes.CDLL(path)
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.wl_rmat_edges.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_double,
                                    ctypes.c_double, ctypes.c_uint64, ctypes.c_int, i32p, i32p]
        L.wl_rmat_edges.restype = ctypes.c_int
        L.wl_fixed_outdeg_edges.argtypes = [ctypes.c_int64, ctypes.c_int, ctypes.c_uint64, i32p, i32p]
        L.wl_fixed_outdeg_edges.restype = ctypes.c_int
        L.wl_build_in_csr.argtypes = [ctypes.c_int64, ctypes.c_int64, i32p, i32p, i32p, i32p, i32p]
        L.wl_build_in_csr.restype = ctypes.c_int
        L.wl_fnv1a.argtypes = [ctypes.c_void_p, ctypes.c_int64]
        L.wl_fnv1a.restype = ctypes.c_uint64
        _lib = L
    return _lib
