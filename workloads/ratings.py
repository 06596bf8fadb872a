"""Seeded synthetic rating graphs (CSR by user) for the Graph SGD side task, for both the oracle's and the GPU path's tests.

Input construction only: no SGD arithmetic lives here.  The paper runs Graph SGD on a public social graph (Section
6.1.4) whose edges carry no ratings of their own; these graphs stand in for it: the edge structure is the same R-MAT
recipe the PageRank inputs use (users = items = 2**scale vertices, duplicates removed), and the ratings come from
planted low-rank factors plus noise, so that a factorization has something to find.
"""
from dataclasses import dataclass

import numpy as np

from . import graphs


@dataclass
class Ratings:
    n_users: int
    n_items: int
    n_ratings: int
    row_ptr: np.ndarray      # int32 [U + 1]
    item: np.ndarray         # int32 [E], ascending and distinct inside a row
    rating: np.ndarray       # float32 [E]


def rmat_ratings(scale: int, n_edges: int, seed: int, rank: int = 4, noise: float = 0.1) -> Ratings:
    """R-MAT edges over 2**scale users x 2**scale items (duplicates dropped), rating = 3 + <a_u, b_i> + noise."""
    n = 1 << scale
    src, dst = graphs.rmat_edges(scale, n_edges, seed)
    key = np.unique((src.astype(np.int64) << 32) | dst.astype(np.int64))      # sorted by user, then item
    users = (key >> 32).astype(np.int64)
    item = (key & 0xFFFFFFFF).astype(np.int32)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(row_ptr, users + 1, 1)
    row_ptr = np.cumsum(row_ptr).astype(np.int32)
    rng = np.random.default_rng(seed + 0x5eed)
    a = rng.standard_normal((n, rank)) / np.sqrt(rank)
    b = rng.standard_normal((n, rank)) / np.sqrt(rank)
    rating = 3.0 + np.einsum("ef,ef->e", a[users], b[item]) + noise * rng.standard_normal(len(item))
    return Ratings(n, n, len(item), row_ptr, item, rating.astype(np.float32))


def initial_factors(n_users: int, n_items: int, F: int, seed: int):
    """Small uniform starting factors (fp32), the same for every implementation under test."""
    rng = np.random.default_rng(seed + 0xfac)
    s = 1.0 / np.sqrt(F)
    P = rng.uniform(0.0, s, (n_users, F)).astype(np.float32)
    Q = rng.uniform(0.0, s, (n_items, F)).astype(np.float32)
    return P, Q
