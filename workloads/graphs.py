"""Seeded synthetic graphs as in-edge CSR (int32), for both the oracle's and the GPU path's tests.

Input construction only: no PageRank arithmetic and no schedule logic lives here.
The graphs stand in for the public social graph the paper runs PageRank on
(Section 6.1.4); the recipes follow the benchmark configurations' wording.
"""
import ctypes
from dataclasses import dataclass

import numpy as np

from . import _native


@dataclass
class Csr:
    """In-edge CSR: row v lists the sources of v's in-edges (ascending, duplicates kept)."""
    n_vertices: int
    n_edges: int
    row_ptr: np.ndarray      # int32 [V + 1]
    col: np.ndarray          # int32 [E]
    out_degree: np.ndarray   # int32 [V], edges leaving each vertex, with multiplicity

    def fingerprint(self) -> int:
        L = _native.lib()
        h = 0
        for arr in (self.row_ptr, self.col, self.out_degree):
            a = np.ascontiguousarray(arr)
            h ^= L.wl_fnv1a(a.ctypes.data_as(ctypes.c_void_p), a.nbytes)
            h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
        return h


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def rmat_edges(scale: int, n_edges: int, seed: int, a=0.57, b=0.19, c=0.19, permute=True):
    """R-MAT edge list (src, dst) over 2**scale vertices; one 24-bit counter-based draw per level."""
    src = np.empty(n_edges, dtype=np.int32)
    dst = np.empty(n_edges, dtype=np.int32)
    rc = _native.lib().wl_rmat_edges(scale, n_edges, a, b, c, seed, 1 if permute else 0, _p(src), _p(dst))
    if rc != 0:
        raise ValueError("wl_rmat_edges: bad arguments")
    return src, dst


def fixed_outdeg_edges(n_vertices: int, degree: int, seed: int):
    """Every vertex emits exactly `degree` edges to independent uniform destinations."""
    src = np.empty(n_vertices * degree, dtype=np.int32)
    dst = np.empty(n_vertices * degree, dtype=np.int32)
    rc = _native.lib().wl_fixed_outdeg_edges(n_vertices, degree, seed, _p(src), _p(dst))
    if rc != 0:
        raise ValueError("wl_fixed_outdeg_edges: bad arguments")
    return src, dst


def csr_from_edges(n_vertices: int, src, dst) -> Csr:
    """In-edge CSR of edges u -> v, sources ascending inside a row; multi-edges and self-loops kept."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    if src.shape != dst.shape or src.ndim != 1:
        raise ValueError("src and dst must be 1-D and of equal length")
    n_edges = int(src.shape[0])
    row_ptr = np.empty(n_vertices + 1, dtype=np.int32)
    col = np.empty(max(n_edges, 1), dtype=np.int32)[:n_edges]
    out_degree = np.empty(max(n_vertices, 1), dtype=np.int32)[:n_vertices]
    rc = _native.lib().wl_build_in_csr(n_vertices, n_edges, _p(src), _p(dst), _p(row_ptr), _p(col), _p(out_degree))
    if rc == -1:
        raise ValueError("wl_build_in_csr: bad arguments or endpoint out of range")
    if rc != 0:
        raise MemoryError("wl_build_in_csr: allocation failed")
    return Csr(n_vertices, n_edges, row_ptr, col, out_degree)


def rmat_csr(scale: int, n_edges: int, seed: int, a=0.57, b=0.19, c=0.19, permute=True) -> Csr:
    src, dst = rmat_edges(scale, n_edges, seed, a, b, c, permute)
    return csr_from_edges(1 << scale, src, dst)


def fixed_outdeg_csr(n_vertices: int, degree: int, seed: int) -> Csr:
    src, dst = fixed_outdeg_edges(n_vertices, degree, seed)
    return csr_from_edges(n_vertices, src, dst)


# Small structured graphs with known PageRank closed forms (used as pins).

def ring_csr(n: int) -> Csr:
    """Directed ring v -> v + 1 (mod n)."""
    src = np.arange(n, dtype=np.int32)
    return csr_from_edges(n, src, (src + 1) % n)


def star_csr(n_leaves: int, kind: str) -> Csr:
    """Star on n_leaves + 1 vertices, centre 0. kind: 'both' (centre <-> leaf), 'in' (leaf -> centre),
    'out' (centre -> leaf)."""
    leaves = np.arange(1, n_leaves + 1, dtype=np.int32)
    zeros = np.zeros(n_leaves, dtype=np.int32)
    if kind == "both":
        src, dst = np.concatenate([zeros, leaves]), np.concatenate([leaves, zeros])
    elif kind == "in":
        src, dst = leaves, zeros
    elif kind == "out":
        src, dst = zeros, leaves
    else:
        raise ValueError(kind)
    return csr_from_edges(n_leaves + 1, src, dst)
