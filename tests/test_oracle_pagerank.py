"""Pins for the fp64 PageRank oracle: closed forms, invariants, dense brute force, a dense eigen-solver.

Each pin is chosen so that a plausible slip in the oracle (dropped dangling term, damping applied to the wrong
term, out-degree vs in-degree, transposed CSR, off-by-one iteration count) fails at least one of them.
"""
import numpy as np
import pytest

from oracle.pagerank import pagerank
from workloads import graphs

D = 0.85


def test_ring_is_uniform_at_every_iteration():
    g = graphs.ring_csr(64)
    for k in (0, 1, 7, 30):
        r = pagerank(g.row_ptr, g.col, g.out_degree, D, k)
        assert np.all(r == 1.0 / 64)        # exact: base + d * (1/V) stays 1/V up to one rounding; check tight
        assert abs(r.sum() - 1.0) < 1e-14


def _geometric(c_star, ratio, c0, k):
    return c_star + (ratio ** k) * (c0 - c_star)


@pytest.mark.parametrize("n", [1, 7, 100])
@pytest.mark.parametrize("k", [1, 2, 5, 30])
def test_bidirectional_star_closed_form(n, k):
    # centre c, each leaf (1 - c) / n, no dangling vertex:
    #   c' = (1 - d)/V + d * (sum of leaves) = (1 - d)/V + d (1 - c)  =>  c_k - c* = (-d)^k (c_0 - c*)
    V = n + 1
    g = graphs.star_csr(n, "both")
    r = pagerank(g.row_ptr, g.col, g.out_degree, D, k)
    c_star = ((1 - D) / V + D) / (1 + D)
    c = _geometric(c_star, -D, 1.0 / V, k)
    assert r[0] == pytest.approx(c, abs=1e-14)
    assert np.allclose(r[1:], (1 - c) / n, atol=1e-14, rtol=0)


@pytest.mark.parametrize("n", [1, 7, 100])
@pytest.mark.parametrize("k", [1, 2, 5, 30])
def test_in_star_closed_form_exercises_dangling_term(n, k):
    # leaves -> centre, the centre has no out-edge: D_k = c_k,
    #   c' = (1 - d)/V + d c/V + d (1 - c) = (1 - d)/V + d - (d n / V) c
    V = n + 1
    g = graphs.star_csr(n, "in")
    r = pagerank(g.row_ptr, g.col, g.out_degree, D, k)
    q = D * n / V
    c_star = ((1 - D) / V + D) / (1 + q)
    c = _geometric(c_star, -q, 1.0 / V, k)
    assert r[0] == pytest.approx(c, abs=1e-14)
    assert np.allclose(r[1:], (1 - c) / n, atol=1e-14, rtol=0)


@pytest.mark.parametrize("n", [1, 7, 100])
@pytest.mark.parametrize("k", [1, 2, 5, 30])
def test_out_star_closed_form(n, k):
    # centre -> leaves, all leaves dangling: D_k = 1 - c_k, the centre has no in-edge,
    #   c' = (1 - d)/V + d (1 - c)/V = 1/V - (d/V) c   =>   c* = 1 / (V + d)
    V = n + 1
    g = graphs.star_csr(n, "out")
    r = pagerank(g.row_ptr, g.col, g.out_degree, D, k)
    c_star = 1.0 / (V + D)
    c = _geometric(c_star, -D / V, 1.0 / V, k)
    assert r[0] == pytest.approx(c, abs=1e-14)
    assert np.allclose(r[1:], (1 - c) / n, atol=1e-14, rtol=0)


def test_hand_evaluated_values_for_seven_leaf_stars():
    # hand-evaluated from the closed forms above with d = 0.85, n = 7, k = 30 (and k = 1, 2)
    g = graphs.star_csr(7, "both")
    assert pagerank(g.row_ptr, g.col, g.out_degree, D, 1)[0] == pytest.approx(0.7625, abs=1e-15)
    assert pagerank(g.row_ptr, g.col, g.out_degree, D, 2)[0] == pytest.approx(0.220625, abs=1e-15)
    assert pagerank(g.row_ptr, g.col, g.out_degree, D, 30)[0] == pytest.approx(0.46696507608558, abs=1e-13)
    g = graphs.star_csr(7, "in")
    assert pagerank(g.row_ptr, g.col, g.out_degree, D, 1)[0] == pytest.approx(0.77578125, abs=1e-15)
    g = graphs.star_csr(7, "out")
    assert pagerank(g.row_ptr, g.col, g.out_degree, D, 30)[0] == pytest.approx(1 / 8.85, abs=1e-14)


def _dense_google(V, src, dst, d):
    """Column-stochastic Google matrix built entry by entry in pure Python (independent of any CSR code)."""
    outdeg = [0] * V
    for u in src:
        outdeg[u] += 1
    G = [[(1.0 - d) / V for _ in range(V)] for _ in range(V)]
    for u, v in zip(src, dst):
        G[v][u] += d / outdeg[u]
    for u in range(V):
        if outdeg[u] == 0:
            for v in range(V):
                G[v][u] += d / V
    return G


def _dense_power(G, V, k):
    r = [1.0 / V] * V
    for _ in range(k):
        r = [sum(G[v][u] * r[u] for u in range(V)) for v in range(V)]
    return r


def test_brute_force_dense_google_matrix_on_8_vertex_graphs():
    rng = np.random.default_rng(12345)
    for trial in range(300):
        V = 8
        E = int(rng.integers(0, 40))
        src = rng.integers(0, V, size=E).astype(np.int32)      # multi-edges, self-loops, isolated vertices occur
        dst = rng.integers(0, V, size=E).astype(np.int32)
        if trial % 5 == 0 and E:
            src[: E // 2] = src[0]                               # force a hub and several dangling vertices
        g = graphs.csr_from_edges(V, src, dst)
        k = int(rng.integers(0, 12))
        want = _dense_power(_dense_google(V, src.tolist(), dst.tolist(), D), V, k)
        got = pagerank(g.row_ptr, g.col, g.out_degree, D, k)
        assert np.allclose(got, want, atol=1e-14, rtol=0), (trial, k)


def test_ranks_sum_to_one_on_rmat_with_many_dangling_vertices():
    g = graphs.rmat_csr(12, 1 << 15, seed=5)
    assert (g.out_degree == 0).sum() > 100
    for k in (1, 3, 30):
        r = pagerank(g.row_ptr, g.col, g.out_degree, D, k)
        assert abs(r.sum() - 1.0) < 1e-12
        assert r.min() > 0


def test_many_iterations_reach_dominant_eigenvector_of_google_matrix():
    rng = np.random.default_rng(7)
    V, E = 48, 300
    src = rng.integers(0, V, size=E).astype(np.int32)
    dst = rng.integers(0, V // 2, size=E).astype(np.int32)      # upper half has no in-edges
    src[src >= 40] = 3                                           # vertices 40..47 become dangling
    g = graphs.csr_from_edges(V, src, dst)
    G = np.array(_dense_google(V, src.tolist(), dst.tolist(), D))
    w, vec = np.linalg.eig(G)
    i = int(np.argmax(w.real))
    assert w[i].real == pytest.approx(1.0, abs=1e-12)
    pi = np.abs(vec[:, i].real)
    pi /= pi.sum()
    r = pagerank(g.row_ptr, g.col, g.out_degree, D, 400)
    assert np.allclose(r, pi, atol=1e-12, rtol=0)


def test_thread_count_does_not_change_the_result():
    g = graphs.rmat_csr(12, 1 << 16, seed=9)
    a = pagerank(g.row_ptr, g.col, g.out_degree, D, 10, n_threads=1)
    b = pagerank(g.row_ptr, g.col, g.out_degree, D, 10, n_threads=4)
    assert np.array_equal(a, b)


def test_zero_iterations_and_edgeless_graph():
    g = graphs.csr_from_edges(5, np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert np.allclose(pagerank(g.row_ptr, g.col, g.out_degree, D, 0), 0.2)
    assert np.allclose(pagerank(g.row_ptr, g.col, g.out_degree, D, 9), 0.2, atol=1e-15)   # all mass dangling


# ---- the fp32, thread-parallel sibling that bench.py times as the CPU baseline (oracle/pagerank_f32.c)

def test_fp32_baseline_ring_and_stars_follow_the_closed_forms():
    from oracle.pagerank import pagerank_f32
    g = graphs.ring_csr(64)
    r = pagerank_f32(g.row_ptr, g.col, g.out_degree, D, 30)
    assert np.allclose(r, 1.0 / 64, rtol=1e-6, atol=0)
    n, V = 7, 8
    for kind, ratio, c_star in (("both", -D, ((1 - D) / V + D) / (1 + D)),
                                ("in", -D * n / V, ((1 - D) / V + D) / (1 + D * n / V)),
                                ("out", -D / V, 1.0 / (V + D))):
        g = graphs.star_csr(n, kind)
        for k in (1, 2, 5, 30):
            r = pagerank_f32(g.row_ptr, g.col, g.out_degree, D, k)
            assert r[0] == pytest.approx(_geometric(c_star, ratio, 1.0 / V, k), abs=2e-6), (kind, k)
            assert abs(float(r.astype(np.float64).sum()) - 1.0) < 1e-5


@pytest.mark.parametrize("threads", [1, 3, 0])
def test_fp32_baseline_agrees_with_the_fp64_oracle_and_ignores_the_thread_count(threads):
    from oracle.pagerank import pagerank_f32
    g = graphs.rmat_csr(12, 1 << 16, seed=5)
    want = pagerank(g.row_ptr, g.col, g.out_degree, D, 20)
    got = pagerank_f32(g.row_ptr, g.col, g.out_degree, D, 20, n_threads=threads)
    assert np.abs(got.astype(np.float64) - want).max() <= 1e-6
    one = pagerank_f32(g.row_ptr, g.col, g.out_degree, D, 20, n_threads=1)
    assert np.array_equal(got.view(np.uint32), one.view(np.uint32))
