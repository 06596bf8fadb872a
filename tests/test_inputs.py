"""Checks of the seeded input generators (structure only)."""
import numpy as np
import pytest

from workloads import graphs, configs


def _check_csr(g):
    assert g.row_ptr[0] == 0 and g.row_ptr[-1] == g.n_edges
    assert np.all(np.diff(g.row_ptr) >= 0)
    assert int(g.out_degree.sum()) == g.n_edges
    assert g.col.min(initial=0) >= 0 and g.col.max(initial=0) < g.n_vertices
    # sources ascending inside each row
    d = np.diff(g.col.astype(np.int64))
    row_starts = g.row_ptr[1:-1]
    row_starts = row_starts[(row_starts > 0) & (row_starts < g.n_edges)]
    mask = np.ones(max(g.n_edges - 1, 0), dtype=bool)
    mask[row_starts - 1] = False
    assert np.all(d[mask] >= 0)
    assert np.array_equal(np.bincount(g.col, minlength=g.n_vertices), g.out_degree)


def test_rmat_csr_structure_and_reproducibility():
    g = graphs.rmat_csr(14, 1 << 18, seed=0)
    assert g.n_vertices == 1 << 14 and g.n_edges == 1 << 18
    _check_csr(g)
    assert graphs.rmat_csr(14, 1 << 18, seed=0).fingerprint() == g.fingerprint()
    assert graphs.rmat_csr(14, 1 << 18, seed=1).fingerprint() != g.fingerprint()


def test_rmat_quadrant_probabilities():
    # unpermuted: the top source bit is 0 with probability a + b, the top destination bit with a + c
    n = 1 << 18
    src, dst = graphs.rmat_edges(14, n, seed=3, permute=False)
    for arr, prob in ((src, 0.76), (dst, 0.76)):
        frac = np.mean(arr < (1 << 13))
        assert abs(frac - prob) < 4 * np.sqrt(prob * (1 - prob) / n)
    both_low = np.mean((src < (1 << 13)) & (dst < (1 << 13)))
    assert abs(both_low - 0.57) < 4 * np.sqrt(0.57 * 0.43 / n)


def test_relabel_is_a_bijection():
    n = 1 << 16
    s0, d0 = graphs.rmat_edges(10, n, seed=11, permute=False)
    s1, d1 = graphs.rmat_edges(10, n, seed=11, permute=True)
    m = {}
    for a, b in zip(np.concatenate([s0, d0]).tolist(), np.concatenate([s1, d1]).tolist()):
        assert m.setdefault(a, b) == b
    assert len(set(m.values())) == len(m)


def test_fixed_outdeg_graph():
    g = graphs.fixed_outdeg_csr(1 << 12, 32, seed=3)
    _check_csr(g)
    assert np.all(g.out_degree == 32)
    indeg = np.diff(g.row_ptr)
    assert abs(indeg.mean() - 32) < 1e-9 and 20 < indeg.var() < 45     # ~Poisson(32)


def test_csr_builder_keeps_multi_edges_and_self_loops():
    src = np.array([2, 0, 2, 2, 1, 1], dtype=np.int32)
    dst = np.array([1, 1, 1, 2, 0, 0], dtype=np.int32)
    g = graphs.csr_from_edges(4, src, dst)
    assert g.row_ptr.tolist() == [0, 2, 5, 6, 6]
    assert g.col.tolist() == [1, 1, 0, 2, 2, 2]
    assert g.out_degree.tolist() == [1, 2, 3, 0]
    with pytest.raises(ValueError):
        graphs.csr_from_edges(2, src, dst)


def test_config_table_matches_the_stated_workloads():
    c = configs.by_name("cfg1")
    assert (c.schedule, c.p, c.m, c.stage, c.vertices, c.edges, c.iterations, c.seed) == ("1f1b", 4, 8, 2, 1 << 14, 1 << 18, 30, 0)
    c = configs.by_name("cfg2")
    assert (c.vertices, c.edges, c.iterations, c.seed, c.load.hidden, c.load.ffn, c.load.tokens) == (1 << 22, 1 << 26, 50, 1, 4096, 16384, 2048)
    c = configs.by_name("cfg4")
    assert c.graph == "fixed_outdeg" and c.edges // c.vertices == 32 and c.cu_count == 64
    assert configs.by_name("cfg5").schedule == "gpipe"
