"""The run variant that allocates no device memory (fr_pagerank_run_standalone_noalloc) against the ordinary
standalone run: same bits in ranks_out, on two calls in a row that share the library's static working array, the
second on a smaller graph; also at several launch sizes, and its refusals."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2409_06941_amd as fr          # noqa: E402
from oracle.pagerank import pagerank       # noqa: E402
from workloads import graphs               # noqa: E402


def _task(g, iterations):
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    bufs = (dev(g.row_ptr), dev(g.col), dev(g.out_degree), torch.full((g.n_vertices,), -1.0, dtype=torch.float32, device="cuda"))
    t = fr.PageRankTask(g.n_vertices, g.n_edges, *bufs, damping=0.85, iterations=iterations)
    return t, bufs


def test_noalloc_run_gives_the_bits_of_the_standalone_run_twice_in_a_row():
    big, small = graphs.rmat_csr(16, (1 << 20) + 4097, seed=21), graphs.rmat_csr(12, 30_011, seed=22)
    K = 9
    tasks = []
    for g in (big, small):
        print("standalone run V=%d E=%d" % (g.n_vertices, g.n_edges), flush=True)
        t, bufs = _task(g, K)
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())          # builds the layout, gives the reference
        ref = bufs[3].cpu().numpy().copy()
        want = pagerank(g.row_ptr, g.col, g.out_degree, 0.85, K)
        assert np.abs(ref.astype(np.float64) - want).max() <= 1e-5
        tasks.append((t, bufs, ref))
    try:
        for max_tiles in (0, 3):
            for (t, bufs, ref), g in zip(tasks, (big, small)):                # two calls in a row, the second smaller
                print("noalloc run V=%d max_tiles=%d" % (g.n_vertices, max_tiles), flush=True)
                bufs[3].fill_(-1.0)
                torch.cuda.synchronize()
                t.fr_pagerank_run_standalone_noalloc(0, torch.cuda.current_stream(), max_tiles)
                got = bufs[3].cpu().numpy()
                assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    finally:
        for t, _, _ in tasks:
            t.fr_pagerank_destroy()


def test_noalloc_run_refuses_what_it_cannot_do():
    g = graphs.rmat_csr(10, 5000, seed=23)
    t, bufs = _task(g, 3)
    try:
        with pytest.raises(fr.FreeRideError) as e:                            # no layout yet: it builds nothing
            t.fr_pagerank_run_standalone_noalloc(0, torch.cuda.current_stream())
        assert e.value.code == fr.FR_ERR_STATE
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
        with pytest.raises(fr.FreeRideError) as e:
            t.fr_pagerank_run_standalone_noalloc(64, torch.cuda.current_stream())
        assert e.value.code == fr.FR_ERR_ARG
    finally:
        t.fr_pagerank_destroy()
    # a graph whose messages and contributions do not fit the 64 MiB array
    g = graphs.fixed_outdeg_csr(1 << 22, 4, seed=24)                          # 16.8 M messages (67 MB) + 16.8 MB of contributions
    t, bufs = _task(g, 1)
    try:
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
        with pytest.raises(fr.FreeRideError) as e:
            t.fr_pagerank_run_standalone_noalloc(0, torch.cuda.current_stream())
        assert e.value.code == fr.FR_ERR_ARG
    finally:
        t.fr_pagerank_destroy()
