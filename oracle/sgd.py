"""ctypes front end of the Graph SGD oracle (oracle/sgd.c).  Test infrastructure only."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sgd.c")
_LIB = os.path.join(_HERE, "liboracle_sgd.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile sgd.c with gcc (no floating-point contraction) into a shared library beside it; returns its path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i32p, f32p, f64p = (ctypes.POINTER(t) for t in (ctypes.c_int32, ctypes.c_float, ctypes.c_double))
        L.oracle_sgd_order.argtypes = [ctypes.c_int64, ctypes.c_int64, i32p, i32p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)]
        i64p = ctypes.POINTER(ctypes.c_int64)
        L.oracle_sgd_blocks.argtypes = [ctypes.c_int64, ctypes.c_int64, i32p, i32p, ctypes.c_int32, i64p, i64p]
        L.oracle_sgd_blocks.restype = ctypes.c_int
        L.oracle_sgd_fp64.argtypes = [ctypes.c_int64, ctypes.c_int64, i32p, i32p, f32p, ctypes.c_int32, ctypes.c_double,
                                      ctypes.c_double, ctypes.c_int32, ctypes.c_int32, f64p, f64p]
        L.oracle_sgd_fp32_ordered.argtypes = [ctypes.c_int64, ctypes.c_int64, i32p, i32p, f32p, ctypes.c_int32,
                                              ctypes.c_float, ctypes.c_float, ctypes.c_int32, ctypes.c_int32, f32p, f32p]
        for f in (L.oracle_sgd_order, L.oracle_sgd_fp64, L.oracle_sgd_fp32_ordered):
            f.restype = ctypes.c_int
        _lib = L
    return _lib


def _csr(row_ptr, item, rating, n_items):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    item = np.ascontiguousarray(item, dtype=np.int32)
    rating = np.ascontiguousarray(rating, dtype=np.float32)
    if int(row_ptr[-1]) != item.shape[0] or item.shape != rating.shape:
        raise ValueError("inconsistent CSR")
    if item.size and (item.min() < 0 or item.max() >= n_items):
        raise ValueError("item out of range")
    return row_ptr, item, rating


def _ptr(a, t):
    return a.ctypes.data_as(ctypes.POINTER(t)) if a.size else ctypes.cast(None, ctypes.POINTER(t))


def order(row_ptr, item, n_items: int, blocks: int):
    """Indices of the ratings in the order one iteration visits them (stratified: see sgd.c)."""
    row_ptr, item, _ = _csr(row_ptr, item, np.zeros(len(item), np.float32), n_items)
    out = np.empty(item.shape[0], dtype=np.int64)
    rc = _load().oracle_sgd_order(row_ptr.shape[0] - 1, n_items, _ptr(row_ptr, ctypes.c_int32), _ptr(item, ctypes.c_int32),
                                  blocks, _ptr(out, ctypes.c_int64))
    if rc != 0:
        raise RuntimeError("oracle_sgd_order failed: %d" % rc)
    return out


def blocks(row_ptr, item, n_items: int, n_blocks: int):
    """First ids of the user blocks and of the item blocks (n_blocks + 1 entries each)."""
    row_ptr, item, _ = _csr(row_ptr, item, np.zeros(len(item), np.float32), n_items)
    us, is_ = np.empty(n_blocks + 1, np.int64), np.empty(n_blocks + 1, np.int64)
    rc = _load().oracle_sgd_blocks(row_ptr.shape[0] - 1, n_items, _ptr(row_ptr, ctypes.c_int32), _ptr(item, ctypes.c_int32),
                                   n_blocks, _ptr(us, ctypes.c_int64), _ptr(is_, ctypes.c_int64))
    if rc != 0:
        raise RuntimeError("oracle_sgd_blocks failed: %d" % rc)
    return us, is_


def sgd(row_ptr, item, rating, P0, Q0, gamma: float, lam: float, iterations: int, blocks: int, ordered_fp32: bool = False):
    """Factors (P, Q) after `iterations` passes over the ratings.

    row_ptr / item / rating: ratings as CSR by user (items ascending and distinct inside a row).  P0 [U, F], Q0 [I, F].
    ordered_fp32=False: the textbook formulas in fp64.  True: the same steps in fp32 with every rounding fixed
    (gamma and lam are rounded to fp32 first), for bit-wise comparison with an fp32 implementation.
    """
    U, F = P0.shape
    I = Q0.shape[0]
    row_ptr, item, rating = _csr(row_ptr, item, rating, I)
    if row_ptr.shape[0] != U + 1 or Q0.shape[1] != F:
        raise ValueError("shapes")
    L = _load()
    if ordered_fp32:
        P, Q = (np.array(x, dtype=np.float32, order="C", copy=True) for x in (P0, Q0))
        rc = L.oracle_sgd_fp32_ordered(U, I, _ptr(row_ptr, ctypes.c_int32), _ptr(item, ctypes.c_int32),
                                       _ptr(rating, ctypes.c_float), F, np.float32(gamma), np.float32(lam), iterations, blocks,
                                       _ptr(P, ctypes.c_float), _ptr(Q, ctypes.c_float))
    else:
        P, Q = (np.array(x, dtype=np.float64, order="C", copy=True) for x in (P0, Q0))
        rc = L.oracle_sgd_fp64(U, I, _ptr(row_ptr, ctypes.c_int32), _ptr(item, ctypes.c_int32), _ptr(rating, ctypes.c_float),
                               F, float(gamma), float(lam), iterations, blocks, _ptr(P, ctypes.c_double), _ptr(Q, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("oracle sgd failed: %d" % rc)
    return P, Q


def rmse(row_ptr, item, rating, P, Q) -> float:
    """Root mean squared error of the predictions <p_u, q_i> over all ratings (fp64)."""
    row_ptr = np.asarray(row_ptr)
    users = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
    pred = np.einsum("ef,ef->e", np.asarray(P, np.float64)[users], np.asarray(Q, np.float64)[np.asarray(item)])
    return float(np.sqrt(np.mean((np.asarray(rating, np.float64) - pred) ** 2))) if len(item) else 0.0
