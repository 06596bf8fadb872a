"""GPU parity: the HIP PageRank path against the fp64 CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2409_06941_amd as fr          # noqa: E402
from oracle.pagerank import pagerank       # noqa: E402
from workloads import graphs               # noqa: E402

TOL = 1e-5     # max-abs, fp32 path vs fp64 oracle


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()


def _run(g, damping=0.85, iterations=30, max_tiles=0, mem_limit=1 << 40):
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    if col.numel() == 0:
        col = torch.zeros(4, dtype=torch.int32, device="cuda")
    ranks = torch.full((g.n_vertices,), -1.0, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, damping=damping, iterations=iterations,
                        mem_limit_bytes=mem_limit)
    try:
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), max_tiles)
    finally:
        t.fr_pagerank_destroy()
    return ranks.cpu().numpy()


def _check(g, iterations=30, damping=0.85):
    print("case V=%d E=%d K=%d" % (g.n_vertices, g.n_edges, iterations), flush=True)
    got = _run(g, damping, iterations)
    want = pagerank(g.row_ptr, g.col, g.out_degree, damping, iterations)
    err = np.abs(got.astype(np.float64) - want).max()
    assert err <= TOL, err
    assert abs(float(got.astype(np.float64).sum()) - 1.0) <= 1e-4
    big = want > 1.0 / g.n_vertices
    if big.any():
        assert (np.abs(got[big] - want[big]) / want[big]).max() <= 1e-4
    return got


def test_config1_rmat_matches_oracle():
    _check(graphs.rmat_csr(14, 1 << 18, seed=0), iterations=30)


@pytest.mark.parametrize("scale,edges,seed", [(10, 5000, 3), (13, 100_003, 4), (16, (1 << 20) + 4097, 5)])
def test_ragged_sizes_span_tiles_and_tails(scale, edges, seed):
    _check(graphs.rmat_csr(scale, edges, seed=seed), iterations=12)


@pytest.mark.parametrize("edges", [120, 300, 1200, 40_000])
def test_scatter_bins_of_any_length(edges):
    # the scatter sweep deals groups of eight message numbers to its threads whatever the bins' lengths:
    # from bins of a few messages (most groups cut by a bin's end) to bins of thousands, on 2^16 vertices
    src, dst = graphs.rmat_edges(16, edges, seed=12)
    g = graphs.csr_from_edges(1 << 16, src, dst)
    _check(g, iterations=7)


@pytest.mark.parametrize("rows,srcs", [(8192, 16384), (16384, 16384), (8192, 32768), (16384, 32768)])
def test_every_partition_size(rows, srcs):
    # graphs of 2^24 vertices and more get 16384-row gather tiles and 32768-source scatter tiles; here the sizes
    # are forced on a graph of 100003 vertices (ragged last tiles, merged ranges present)
    src, dst = graphs.rmat_edges(17, 1_500_007, seed=21)
    g = graphs.csr_from_edges(100_003, src % 100_003, dst % 100_003)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=9, rows_per_partition=rows,
                        sources_per_partition=srcs)
    t.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), 3)
    info = t.fr_pagerank_info()
    t.fr_pagerank_destroy()
    assert (info.rows_per_partition, info.sources_per_partition) == (rows, srcs) and info.merged_ranges > 0
    assert info.ranges == -(-g.n_vertices // rows) and 1 <= info.scatter_tiles <= 512
    got = ranks.cpu().numpy()
    want = pagerank(g.row_ptr, g.col, g.out_degree, 0.85, 9)
    assert np.abs(got.astype(np.float64) - want).max() <= TOL
    big = want > 1.0 / g.n_vertices
    assert (np.abs(got[big] - want[big]) / want[big]).max() <= 1e-4
    # same sizes, one launch per segment: same bits (across sizes the float sum of the dangling mass is grouped
    # differently, so the last bit may differ)
    ref = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ref, iterations=9, rows_per_partition=rows,
                        sources_per_partition=srcs)
    t.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), 0)
    t.fr_pagerank_destroy()
    assert np.array_equal(got.view(np.uint32), ref.cpu().numpy().view(np.uint32))


def test_partition_sizes_other_than_the_two_supported_are_refused():
    g = graphs.rmat_csr(10, 3000, seed=8)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2, rows_per_partition=4096)
    with pytest.raises(fr.FreeRideError) as e:
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    assert e.value.code == fr.FR_ERR_ARG
    t.fr_pagerank_destroy()


def test_non_power_of_two_vertices_fixed_outdeg():
    _check(graphs.fixed_outdeg_csr(10_007, 32, seed=3), iterations=20)


def test_ring_and_stars():
    r = _check(graphs.ring_csr(5000), iterations=10)
    assert np.all(r == np.float32(1.0 / 5000))
    for kind in ("both", "in", "out"):
        _check(graphs.star_csr(7, kind), iterations=30)


def test_hub_row_cut_by_many_pull_tiles():
    # one row with 20000 in-edges (five pull tiles) between many empty rows; every leaf row empty
    _check(graphs.star_csr(20_000, "in"), iterations=9)
    _check(graphs.star_csr(20_000, "both"), iterations=9)


def test_degenerate_inputs():
    empty = graphs.csr_from_edges(5000, np.zeros(0, np.int32), np.zeros(0, np.int32))
    _check(empty, iterations=4)                                   # no edges: all mass dangling
    _check(graphs.csr_from_edges(1, np.zeros(3, np.int32), np.zeros(3, np.int32)), iterations=5)   # one vertex, self-loops
    _check(graphs.rmat_csr(10, 3000, seed=8), iterations=0)      # zero iterations: r_0
    _check(graphs.rmat_csr(10, 3000, seed=8), iterations=1)
    _check(graphs.rmat_csr(10, 3000, seed=8), iterations=30, damping=0.5)


def test_any_chunking_gives_identical_bits():
    g = graphs.rmat_csr(15, (1 << 19) + 777, seed=6)
    whole = _run(g, iterations=8, max_tiles=0)
    for m in (1, 3, 50):
        part = _run(g, iterations=8, max_tiles=m)
        assert np.array_equal(whole.view(np.uint32), part.view(np.uint32)), m
    again = _run(g, iterations=8, max_tiles=0)
    assert np.array_equal(whole.view(np.uint32), again.view(np.uint32))


@pytest.mark.parametrize("cu_count", [16, 8])
def test_tiles_follow_the_cu_mask_of_the_stream(cu_count):
    # On a stream confined to a few CUs a launch has two workgroups per CU (at these sizes).  With 16 CUs and a skewed
    # graph of 8 M edges a slot's share of a sweep is short: the sweeps are cut into no more tiles than slots, light
    # pieces sharing tiles.  With 8 CUs and a uniform graph of 16.8 M edges the share is long: every piece is a tile and
    # the workgroups of a launch hand the tiles out among themselves.  Either way: the oracle's ranks, the same bits
    # whatever the chunking.
    if cu_count == 16:
        src, dst = graphs.rmat_edges(20, 8_000_000, seed=33)
        g = graphs.csr_from_edges(1 << 20, src, dst)
    else:
        g = graphs.fixed_outdeg_csr(1 << 20, 16, seed=34)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ctx = fr.Context(device_id=0, cu_count=cu_count)
    out = []
    for max_tiles in (0, 1, 3, 11):
        print("cu_count %d, %d tiles per launch" % (cu_count, max_tiles), flush=True)
        ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
        t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=6)
        t.fr_pagerank_run_standalone(0, ctx.fr_side_stream(), max_tiles)
        info = t.fr_pagerank_info()
        t.fr_pagerank_destroy()
        out.append(ranks.cpu().numpy())
    ctx.fr_destroy()
    pieces = info.nonempty_ranges + info.partial_rows - info.merged_ranges
    if cu_count == 16:
        assert info.gather_tiles <= 32 and info.scatter_tiles <= 32
        assert pieces > info.gather_tiles                                      # pieces share tiles
        assert info.merged_ranges > 0                                          # rows whose sums are joined from partial sums: the
                                                                               # chunkings agree bit for bit on a masked stream too
        assert -(-g.n_vertices // 16384) > info.scatter_tiles
    else:
        assert info.gather_tiles > 16 and info.scatter_tiles > 16             # more tiles than workgroups: handed out
        assert pieces == info.gather_tiles                                     # a tile is a piece
        assert info.scatter_tiles >= -(-g.n_vertices // 16384)
    want = pagerank(g.row_ptr, g.col, g.out_degree, 0.85, 6)
    assert np.abs(out[0].astype(np.float64) - want).max() <= TOL
    big = want > 1.0 / g.n_vertices
    assert (np.abs(out[0][big] - want[big]) / want[big]).max() <= 1e-4
    for o in out[1:]:
        assert np.array_equal(out[0].view(np.uint32), o.view(np.uint32))


def test_memory_limit_refuses_the_task():
    g = graphs.rmat_csr(12, 1 << 15, seed=2)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2, mem_limit_bytes=1 << 40)
    with pytest.raises(fr.FreeRideError) as e:          # layout facts exist only after InitSideTask
        t.fr_pagerank_info()
    assert e.value.code == fr.FR_ERR_STATE
    t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    info = t.fr_pagerank_info()
    t.fr_pagerank_destroy()
    caller = 4 * g.n_edges + 4 * (g.n_vertices + 1) + 8 * g.n_vertices
    assert info.bytes_peak >= info.bytes_resident > caller
    assert 0 < info.messages <= g.n_edges
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2, mem_limit_bytes=info.bytes_peak - 1)
    with pytest.raises(fr.FreeRideError) as e:
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    assert e.value.code == fr.FR_ERR_OOM
    t.fr_pagerank_destroy()
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2, mem_limit_bytes=info.bytes_peak)
    t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    t.fr_pagerank_destroy()


def _host_layout(g, rows_per_range):
    """Vertices renumbered by in-degree (largest first, ties by id; the vertices without in-edges by out-degree, largest
    first, then by id); sorted (range, source, row) keys of the edges."""
    V = g.n_vertices
    indeg = np.diff(g.row_ptr)
    tie = np.where(indeg == 0, -g.out_degree.astype(np.int64), 0)
    order = np.lexsort((np.arange(V), tie, -indeg.astype(np.int64)))
    new_id = np.empty(V, dtype=np.int64)
    new_id[order] = np.arange(V)
    row = new_id[np.repeat(np.arange(V), indeg)]
    src = new_id[g.col.astype(np.int64)]
    key = np.sort(((row // rows_per_range) << 46) | (src << 15) | (row % rows_per_range))
    return key


def test_layout_facts_match_the_graph():
    # messages = distinct (range, source) pairs; gather tiles hold whole pieces (runs of edges of one range)
    g = graphs.rmat_csr(15, 1 << 19, seed=6)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=1)
    t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    info = t.fr_pagerank_info()
    edges = t.fr_pagerank_tile_work(fr.FR_PR_SEG_GATHER)
    weights = t.fr_pagerank_tile_weights(fr.FR_PR_SEG_GATHER)
    msgs = t.fr_pagerank_tile_work(fr.FR_PR_SEG_SCATTER)
    srcs = t.fr_pagerank_tile_weights(fr.FR_PR_SEG_SCATTER)
    t.fr_pagerank_destroy()
    V, E = g.n_vertices, g.n_edges
    key = _host_layout(g, 8192)
    rng = key >> 46
    Q = -(-V // 8192)
    per_range = np.bincount(rng, minlength=Q)
    assert info.ranges == Q and info.nonempty_ranges == int((per_range > 0).sum())
    assert np.all(per_range[:info.nonempty_ranges] > 0)                 # ranges with edges come first
    starts = np.ones(E, dtype=bool)
    starts[1:] = (key[1:] >> 15) != (key[:-1] >> 15)
    repeats = np.zeros(E, dtype=bool)
    repeats[1:] = key[1:] == key[:-1]
    assert info.messages == int(starts.sum())
    assert info.gather_tiles == len(edges) <= 256 and sum(edges) == E
    # a tile ends where a range ends or, inside a range cut into several pieces, on a multiple of 512 edges
    bounds = np.concatenate([[0], np.cumsum(edges)])
    range_end = set(np.cumsum(per_range).tolist())
    assert all(int(b) in range_end or b % 512 == 0 for b in bounds[1:])
    assert info.merged_ranges > 0 and info.partial_rows >= 2 * info.merged_ranges
    # weights: 2 an edge, 6 more for an edge that repeats its predecessor, 147456 a piece; exact for tiles that begin
    # and end on multiples of 512 or at the ends of the stream (inside a chunk of 512 the weight is spread evenly)
    w_edge = 2 + 6 * repeats.astype(np.int64)
    cum = np.concatenate([[0], np.cumsum(w_edge)])
    pieces_total = 0
    for i, w in enumerate(weights):
        a, b = int(bounds[i]), int(bounds[i + 1])
        extra = w - (cum[b] - cum[a])
        if (a % 512 == 0) and (b % 512 == 0 or b == E):
            assert extra > 0 and extra % 147456 == 0
        pieces_total += round(extra / 147456)
    n_direct = info.nonempty_ranges - info.merged_ranges
    assert pieces_total == n_direct + info.partial_rows
    assert sum(msgs) == info.messages and len(msgs) == info.scatter_tiles
    assert len(msgs) <= 512                                             # no more tiles than workgroups side by side
    assert all(s >= 1 for s in srcs) and sum(srcs) >= V                 # sources + partial sums added up


def test_one_row_with_over_a_million_in_edges():
    # 3 vertices, one row with 1.2 million in-edges (multi-edges): its range is cut into several gather tiles whose
    # partial sums the scatter sweep (and, after the last iteration, the finishing pass) adds up
    n = 1_200_000
    src = np.concatenate([np.full(n, 1, np.int32), np.array([0, 2], np.int32)])
    dst = np.concatenate([np.zeros(n, np.int32), np.array([1, 1], np.int32)])
    g = graphs.csr_from_edges(3, src, dst)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(3, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(3, g.n_edges, rp, col, od, ranks, iterations=6)
    t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    info = t.fr_pagerank_info()
    weights = t.fr_pagerank_tile_weights(fr.FR_PR_SEG_GATHER)
    t.fr_pagerank_destroy()
    # all but one of the edges into the heavy row repeat their predecessor: weight 8 apiece
    assert info.merged_ranges == 1 and info.gather_tiles == info.partial_rows > 10
    assert sum(weights) == 2 * (n + 2) + 6 * (n - 1) + 147456 * info.partial_rows
    assert max(weights) <= 1.1 * sum(weights) / len(weights)            # tiles of about equal weight
    want = pagerank(g.row_ptr, g.col, g.out_degree, 0.85, 6)
    assert np.abs(ranks.cpu().numpy().astype(np.float64) - want).max() <= TOL


def test_malformed_csr_is_refused_before_any_kernel_uses_it():
    g = graphs.rmat_csr(10, 3000, seed=1)
    bad_col = g.col.copy()
    bad_col[1234] = g.n_vertices            # out of range source
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(bad_col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2)
    with pytest.raises(fr.FreeRideError) as e:
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    assert e.value.code == fr.FR_ERR_ARG
    t.fr_pagerank_destroy()
    bad_rp = g.row_ptr.copy()
    bad_rp[10] = bad_rp[11] + 1             # not monotone
    rp = _dev(bad_rp, torch.int32)
    col = _dev(g.col, torch.int32)
    t = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2)
    with pytest.raises(fr.FreeRideError) as e:
        t.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    assert e.value.code == fr.FR_ERR_ARG
    t.fr_pagerank_destroy()
