"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Paths and active sets: bit-exact.  Gradients: |gpu - oracle| <= 1e-6 + 1e-5 |oracle|.
"""
from pathlib import Path

import numpy as np
import pytest
import torch

import graphgen
import oracle

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(not torch.cuda.is_available(), reason="needs a GPU")]

if torch.cuda.is_available():
    import paper_2204_02662_amd as epp
    from _util import (assert_close, assert_paths_bit_exact, gpu_prepare, gpu_prepare_full, run_full, run_partial,
                       run_ifelse, dev)


@pytest.fixture(params=["one-launch", "general"])
def construction(request, monkeypatch):
    """Small graphs are prepared by a single-launch construction; with EPP_TUNE_SMALL_PREPARE=0 they
    go through the general one.  Tests on small graphs that take this fixture cover both."""
    monkeypatch.setenv("EPP_TUNE_SMALL_PREPARE", "1" if request.param == "one-launch" else "0")
    return request.param


def oprep(g, train, L):
    return oracle.prepare(g.n, g.rowptr, g.col, g.val, np.asarray(train, np.int32), L)


def check_layers(g, train, L, widths, seed, gs_list=(0,)):
    """Full comparison on a graph small enough for the oracle to do every row."""
    sets_o, paths_o = oprep(g, train, L)
    paths = gpu_prepare(g, train, L)
    assert_paths_bit_exact(paths, sets_o, paths_o, L)
    full = gpu_prepare_full(g)
    for l in range(L):
        F = widths[l]
        src = sets_o[L - l - 1]
        X = graphgen.normal_rows(g.n, F, src, seed + l)
        want = oracle.path_aggregate(g.n, paths_o[l], X)
        p = paths.path(l)
        for gs in gs_list:
            if gs:
                p.set_group_size(F, gs)
            got = run_partial(p, X)
            assert_close(got, want, f"partial l={l} F={F} gs={gs}")
            # rows outside the path are not touched; rows inside are overwritten
            mark = run_partial(p, X, poison=123.0)
            rows = sets_o[L - l].astype(bool)
            assert np.all(mark[~rows] == 123.0)
            assert_close(mark[rows], want[rows], f"partial overwrite l={l}")
        # never reads rows outside the source set
        Xp = X.copy()
        Xp[src == 0] = np.nan
        assert_close(run_partial(p, Xp), want, f"nan-poison l={l}")
        # the all-active kernel gives the same matrix (Theorem 1) and writes every row
        assert_close(run_full(full, X), oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X), f"full l={l}")
        # if-else selective scheduling on the whole graph: same rows written, same values,
        # inactive sources never read
        rows = sets_o[L - l].astype(bool)
        for Xi in (X, Xp):
            got = run_ifelse(full, paths, l, Xi)
            assert np.all(got[~rows] == 123.0)
            assert_close(got[rows], want[rows], f"if-else l={l}")
    return paths


def test_worked_example_on_gpu(construction):
    edges = [(0, 1), (1, 2), (1, 3), (1, 4), (2, 3), (3, 4)]
    g = graphgen.csr_from_edges(5, edges, self_loops=False, normalise=False)
    paths = check_layers(g, [2, 4], 2, [3, 5], 1)
    row_ids, rowptr, col, _ = (t.cpu().tolist() for t in paths.path(1).export())
    assert (row_ids, rowptr, col) == ([1, 3], [0, 2, 4], [2, 4, 2, 4])
    row_ids, rowptr, col, _ = (t.cpu().tolist() for t in paths.path(0).export())
    assert (row_ids, rowptr, col) == ([0, 1, 2, 3, 4], [0, 1, 2, 4, 5, 7], [1, 3, 1, 3, 1, 1, 3])


@pytest.mark.parametrize("seed", range(4))
def test_small_random_graphs(seed, construction):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(50, 400))
    sym = bool(seed & 1)
    edges = [(int(u), int(v)) for u, v in rng.integers(0, n, (4 * n, 2)) if u != v]
    g = graphgen.csr_from_edges(n, edges, self_loops=bool(seed & 2), symmetric=sym, normalise=sym)
    if not sym:
        g.val[:] = rng.uniform(0.25, 2.0, g.nnz).astype(np.float32)
    train = rng.choice(n, size=max(1, n // 10), replace=False)
    check_layers(g, train, 3, [int(x) for x in rng.integers(1, 70, 3)], 50 + seed, gs_list=(0, 1, 3))


@pytest.mark.parametrize("loops,sym", [(True, True), (False, True), (False, False), (True, False)])
def test_deep_paths_over_many_tiles(loops, sym):
    """Four levels over a few hundred edge tiles.  With self-loops N^k grows monotonically and
    every level after the first starts from the keep-mask of the level before; without them
    the sets are not nested and every level tests all entries again.  Same paths either way."""
    rng = np.random.default_rng(7 + 2 * loops + sym)
    n = 60_000
    edges = rng.integers(0, n, (250_000, 2))
    edges = edges[edges[:, 0] != edges[:, 1]]
    g = graphgen.csr_from_edges(n, [tuple(e) for e in edges.tolist()], self_loops=loops, symmetric=sym, normalise=sym)
    train = rng.choice(n, size=40, replace=False)
    L = 4
    sets_o, paths_o = oprep(g, train, L)
    nested = all(np.all(sets_o[k + 1][sets_o[k] != 0] != 0) for k in range(L))
    assert nested == loops
    sizes = [int((s != 0).sum()) for s in sets_o]
    assert sizes[0] < sizes[1] < sizes[2] < sizes[3]  # the frontier is still growing at every level
    paths = gpu_prepare(g, train, L)
    assert_paths_bit_exact(paths, sets_o, paths_o, L)


@pytest.mark.parametrize("F", [1, 2, 3, 4, 5, 6, 7, 8, 16, 31, 32, 41, 47, 64, 100, 128, 130, 256, 259, 300, 301])
def test_widths_on_skewed_graph(F):
    """Several tiles, hubs that get split, a ragged tail, every vector shape."""
    g = graphgen.random_graph("rmat", 5003, seed=21, raw_draws=90_000)
    train = graphgen.training_set(g.n, 300, 22)
    sets_o, paths_o = oprep(g, train, 2)
    paths = gpu_prepare(g, train, 2)
    for l in range(2):
        X = graphgen.normal_rows(g.n, F, sets_o[2 - l - 1], 23 + l)
        want = oracle.path_aggregate(g.n, paths_o[l], X)
        p = paths.path(l)
        for gs in (0, 16, 1 << 20):
            p.set_group_size(F, gs)
            assert_close(run_partial(p, X), want, f"F={F} l={l} gs={gs}")


def test_group_size_invariance_and_group_counts():
    g = graphgen.random_graph("chung_lu", 4000, seed=31, target_edges=40_000)
    train = graphgen.training_set(g.n, 400, 32)
    sets_o, paths_o = oprep(g, train, 2)
    paths = gpu_prepare(g, train, 2)
    F = 16
    X = graphgen.normal_rows(g.n, F, sets_o[1], 33)
    want = oracle.path_aggregate(g.n, paths_o[0], X)
    p = paths.path(0)
    ptr = paths_o[0].rowptr.astype(np.int64)
    nnz = int(ptr[-1])
    for gs in (1, 2, 3, 8, 64, 10 ** 6):
        p.set_group_size(F, gs)
        assert_close(run_partial(p, X), want, f"gs={gs}")
        i = p.info()
        # neighbour grouping: the edge array in consecutive chunks of gs entries; a row is
        # cut iff a chunk boundary falls strictly inside it
        assert i.group_size == gs and i.n_groups == -(-nnz // gs)
        assert i.n_split_rows == int(np.sum((ptr[1:] - 1) // gs > ptr[:-1] // gs))
    p.set_group_size(F, 0)
    assert p.info().group_size == p.select_group_size(F) >= 1


def test_special_cases_on_gpu(construction):
    rng = np.random.default_rng(3)
    n = 300
    edges = [(int(u), int(v)) for u, v in rng.integers(0, n, (900, 2)) if u != v]
    g = graphgen.csr_from_edges(n, edges, self_loops=False)
    # V_t = V, duplicates, single vertex, isolated vertex
    for train in (np.arange(n), [5, 5, 9, 5], [0], [int(np.flatnonzero(np.diff(g.rowptr) == 0)[0])]
                  if (np.diff(g.rowptr) == 0).any() else [1]):
        check_layers(g, train, 2, [4, 9], 40)
    # V_t empty: all paths empty, aggregate is a no-op
    paths = gpu_prepare(g, np.zeros(0, np.int32), 2)
    sets_o, paths_o = oprep(g, [], 2)
    assert_paths_bit_exact(paths, sets_o, paths_o, 2)
    X = graphgen.normal_rows(n, 8, None, 1)
    assert np.all(run_partial(paths.path(0), X, poison=5.0) == 5.0)
    # graph without edges
    g0 = graphgen.csr_from_edges(10, [], self_loops=False)
    paths = gpu_prepare(g0, [1, 2], 2)
    assert_paths_bit_exact(paths, *oprep(g0, [1, 2], 2), 2)
    assert np.all(run_full(gpu_prepare_full(g0), graphgen.normal_rows(10, 4, None, 1)) == 0.0)


def test_error_paths(construction):
    g = graphgen.csr_from_edges(10, [(0, 1), (1, 2)], self_loops=True)
    with pytest.raises(epp.EppError) as e:
        gpu_prepare(g, [10], 2)
    assert e.value.code == epp.EPP_ERR_OUT_OF_RANGE_ID
    with pytest.raises(epp.EppError) as e:
        gpu_prepare(g, [-1], 2)
    assert e.value.code == epp.EPP_ERR_OUT_OF_RANGE_ID
    with pytest.raises(epp.EppError) as e:
        gpu_prepare(g, [1], 0)
    assert e.value.code == epp.EPP_ERR_INVALID_ARG
    paths = gpu_prepare(g, [1], 1)
    x = torch.zeros(10, 4, device=dev())
    with pytest.raises(epp.EppError) as e:
        epp.epp_backward_aggregate(paths.path(0), x, torch.zeros_like(x))  # width 4 not prepared
    assert e.value.code == epp.EPP_ERR_INVALID_ARG and "prepare_width" in str(e.value)
    paths.path(0).prepare_width(4)
    epp.epp_backward_aggregate(paths.path(0), x, torch.zeros_like(x))
    with pytest.raises(epp.EppError):
        epp.epp_full_aggregate(paths.path(0), x, torch.zeros_like(x))  # not an all-active handle
    with pytest.raises(epp.EppError):
        epp.epp_backward_aggregate(paths.path(0), x, x)  # aliasing
    with pytest.raises(ValueError):
        epp.epp_backward_aggregate(paths.path(0), x[:9], torch.zeros_like(x[:9]))  # fewer rows than vertices
    # the caller's CSR is checked on the GPU before it is used as an index
    d = dev()
    rowptr, col, val = (torch.from_numpy(a).to(d) for a in (g.rowptr, g.col, g.val))
    ids = torch.tensor([1], dtype=torch.int32, device=d)
    for bad_col in (-1, 10, 2 ** 30):
        c = col.clone()
        c[3] = bad_col
        for call in (lambda: epp.epp_prepare(g.n, rowptr, c, val, ids, 2), lambda: epp.epp_prepare_full(g.n, rowptr, c, val)):
            with pytest.raises(epp.EppError) as e:
                call()
            assert e.value.code == epp.EPP_ERR_OUT_OF_RANGE_ID
    for pos, bad_ptr in ((0, 1), (4, 0), (4, g.nnz + 5), (g.n, g.nnz - 1)):
        r = rowptr.clone()
        r[pos] = bad_ptr
        for call in (lambda: epp.epp_prepare(g.n, r, col, val, ids, 2), lambda: epp.epp_prepare_full(g.n, r, col, val)):
            with pytest.raises(epp.EppError) as e:
                call()
            assert e.value.code == epp.EPP_ERR_INVALID_ARG, (pos, bad_ptr)


def test_run_to_run_determinism_of_every_row():
    """Rows cut by group boundaries are summed from per-group pieces in a fixed order (no
    floating-point atomics), so repeated launches agree bit for bit, cut rows included, and
    whatever grad_out held before."""
    g = graphgen.random_graph("rmat", 20_000, seed=61, raw_draws=300_000)
    train = graphgen.training_set(g.n, 2000, 62)
    sets_o, paths_o = oprep(g, train, 2)
    paths = gpu_prepare(g, train, 2)
    X32 = graphgen.normal_rows(g.n, 32, sets_o[1], 63)
    p = paths.path(0)
    ptr = paths_o[0].rowptr.astype(np.int64)
    for F, gs in ((32, 64), (32, 8), (7, 16)):  # long rows span many groups at gs = 8
        X = np.ascontiguousarray(X32[:, :F])
        p.set_group_size(F, gs)
        cut = (ptr[1:] - 1) // gs != ptr[:-1] // gs
        assert cut.sum() > 100 and p.info().n_split_rows == cut.sum()
        a = run_partial(p, X)
        b = run_partial(p, X, poison=float("nan"))
        c = run_partial(p, X, poison=3.0)
        rows = paths_o[0].row_ids
        assert np.array_equal(a[rows], b[rows]) and np.array_equal(a[rows], c[rows]), (F, gs)
        assert_close(a, oracle.path_aggregate(g.n, paths_o[0], X), f"F={F} gs={gs}")


def test_forward_aggregation_and_its_adjoint():
    """Alg. 1's forward aggregation on the all-active kernel (the library is handed the forward
    operator A), and the backward one on its transpose: each against the oracle, and
    <A X, G> = <X, A^T G> across the two GPU results.  A is directed and randomly weighted."""
    rng = np.random.default_rng(91)
    n, F = 6000, 24
    pairs = rng.integers(0, n, (60_000, 2))
    pairs = pairs[pairs[:, 0] != pairs[:, 1]]
    fwd = graphgen.csr_from_edges(n, [tuple(e) for e in pairs.tolist()], self_loops=True, symmetric=False,
                                  normalise=False)
    fwd.val[:] = rng.uniform(0.1, 1.0, fwd.nnz).astype(np.float32)
    # transpose on the host with plain index arithmetic: entry (v <- u, w) becomes (u <- v, w)
    dst = np.repeat(np.arange(n, dtype=np.int64), np.diff(fwd.rowptr))
    order = np.lexsort((dst, fwd.col))
    bwd = graphgen.Graph(n, np.concatenate([[0], np.cumsum(np.bincount(fwd.col, minlength=n))]).astype(np.int32),
                         dst[order].astype(np.int32), fwd.val[order].copy())
    X = graphgen.normal_rows(n, F, None, 92)
    G = graphgen.normal_rows(n, F, None, 93)
    AX = run_full(gpu_prepare_full(fwd), X)
    AtG = run_full(gpu_prepare_full(bwd), G)
    assert_close(AX, oracle.full_aggregate(n, fwd.rowptr, fwd.col, fwd.val, X), "forward")
    assert_close(AtG, oracle.full_aggregate(n, bwd.rowptr, bwd.col, bwd.val, G), "backward")
    lhs = float(np.sum(AX.astype(np.float64) * G)), float(np.sum(X.astype(np.float64) * AtG))
    assert abs(lhs[0] - lhs[1]) <= 1e-5 * max(abs(lhs[0]), 1.0), lhs


@pytest.mark.parametrize("k", [1, 2])
def test_small_configs_every_entry(k, construction):
    cfg = graphgen.make_config(k)
    check_layers(cfg.graph, cfg.train_ids, cfg.L, cfg.widths, cfg.seed(10))


def test_export_is_unchanged_by_aggregation_and_hot_cold_marking(monkeypatch):
    """Internal flags (row ends, cold sources) never leak into the canonical form, and the
    result does not depend on which sources are streamed."""
    g = graphgen.random_graph("rmat", 30_000, seed=71, raw_draws=400_000)
    train = graphgen.training_set(g.n, 3000, 72)
    sets_o, paths_o = oprep(g, train, 2)
    F = 64
    X = graphgen.normal_rows(g.n, F, sets_o[1], 73)
    want = oracle.path_aggregate(g.n, paths_o[0], X)
    for mb in ("0", "1", "2"):  # off / a budget of 1 or 2 MB: most sources of this path are cold
        monkeypatch.setenv("EPP_TUNE_HOT_MB", mb)
        paths = gpu_prepare(g, train, 2)
        p = paths.path(0)
        assert_close(run_partial(p, X), want, f"hot budget {mb} MB")
        Xp = X.copy()
        Xp[sets_o[1] == 0] = np.nan
        assert_close(run_partial(p, Xp), want, f"hot budget {mb} MB, nan-poison")
        assert_paths_bit_exact(paths, sets_o, paths_o, 2)


@pytest.mark.parametrize("F", [128, 130, 256])
@pytest.mark.parametrize("slices", ["1", "2", "3"])
@pytest.mark.parametrize("hot_mb", ["0", "1"])
def test_xcd_feature_slices_and_cold_marks_on_every_row(monkeypatch, F, slices, hot_mb):
    """The XCD feature-slicing launch shapes (2, 4 and 8 slices, whatever the library would pick
    by itself) with and without streamed (cold) sources, on a path whose rows are cut by many
    group boundaries: every row against the oracle, NaN poison outside the source set included."""
    g = graphgen.random_graph("rmat", 30_000, seed=171, raw_draws=400_000)
    train = graphgen.training_set(g.n, 3000, 172)
    sets_o, paths_o = oprep(g, train, 2)
    monkeypatch.setenv("EPP_TUNE_LOG2_SLICES", slices)
    monkeypatch.setenv("EPP_TUNE_HOT_MB", hot_mb)
    paths = gpu_prepare(g, train, 2)
    for l, gs in ((0, 24), (1, 0)):
        X = graphgen.normal_rows(g.n, F, sets_o[2 - l - 1], 173 + l)
        want = oracle.path_aggregate(g.n, paths_o[l], X)
        p = paths.path(l)
        if gs:
            p.set_group_size(F, gs)
            assert p.info().n_split_rows > 1000
        rows = sets_o[2 - l].astype(bool)
        got = run_partial(p, X, poison=9.0)
        assert np.all(got[~rows] == 9.0)
        assert_close(got[rows], want[rows], f"slices 2^{slices} hot {hot_mb} MB F={F} l={l}")
        Xp = X.copy()
        Xp[sets_o[2 - l - 1] == 0] = np.nan
        assert_close(run_partial(p, Xp), want, f"slices 2^{slices} hot {hot_mb} MB F={F} l={l}, nan-poison")


@pytest.mark.parametrize("F", [64, 67, 128, 130, 256])
@pytest.mark.parametrize("min_len", ["4", "40"])
def test_source_partitioned_layout_on_every_row(monkeypatch, F, min_len):
    """The source-partitioned layout (entries of long rows that reference the most referenced
    sources moved into one section per XCD, partial rows added up per vertex), forced on at a
    small size with a hot set far smaller than the source set: every row against the oracle,
    with the library's group size and with a small one that cuts many virtual rows, NaN poison
    outside the source set, rows outside the path untouched, bit-identical repeats; the same for
    the all-active graph, whose empty rows must still come out zero."""
    g = graphgen.random_graph("rmat", 30_000, seed=271, raw_draws=400_000)
    train = graphgen.training_set(g.n, 3000, 272)
    sets_o, paths_o = oprep(g, train, 2)
    monkeypatch.setenv("EPP_TUNE_PART", "2")
    monkeypatch.setenv("EPP_TUNE_PART_KB", "64")
    monkeypatch.setenv("EPP_TUNE_PART_MINLEN", min_len)
    paths = gpu_prepare(g, train, 2)
    for l, gs in ((0, 24), (0, 0), (1, 0)):
        X = graphgen.normal_rows(g.n, F, sets_o[2 - l - 1], 273 + l)
        want = oracle.path_aggregate(g.n, paths_o[l], X)
        p = paths.path(l)
        p.set_group_size(F, gs)
        rows = sets_o[2 - l].astype(bool)
        got = run_partial(p, X, poison=9.0)
        i = p.info()
        assert i.part_rows > 0 and i.part_hot_entries > 0 and i.part_partial_rows >= i.part_rows, i
        if gs:
            assert i.n_split_rows > 1000
        assert np.all(got[~rows] == 9.0)
        assert_close(got[rows], want[rows], f"partitioned F={F} l={l} gs={gs}")
        again = run_partial(p, X, poison=float("nan"))
        assert np.array_equal(got[rows], again[rows])
        Xp = X.copy()
        Xp[sets_o[2 - l - 1] == 0] = np.nan
        assert_close(run_partial(p, Xp), want, f"partitioned F={F} l={l} gs={gs}, nan-poison")
    assert_paths_bit_exact(paths, sets_o, paths_o, 2)  # the canonical form is not touched
    # the three kernels of a partitioned launch captured in a HIP graph: replays reproduce the eager result
    p = paths.path(0)
    p.prepare_width(F)
    gin = torch.from_numpy(graphgen.normal_rows(g.n, F, sets_o[1], 273)).to(dev())
    gout = torch.zeros_like(gin)
    epp.epp_backward_aggregate(p, gin, gout)
    torch.cuda.synchronize()
    eager = gout.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        epp.epp_backward_aggregate(p, gin, gout)
    for rep in range(3):
        gout.normal_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        rows_t = torch.from_numpy(sets_o[2].astype(bool)).to(dev())
        assert torch.equal(gout[rows_t], eager[rows_t]), f"replay {rep}"
    del graph
    full = gpu_prepare_full(g)
    X = graphgen.normal_rows(g.n, F, None, 279)
    got = run_full(full, X)
    assert full.info().part_rows > 0
    assert_close(got, oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X), f"partitioned all-active F={F}")
    # the if-else baseline keeps walking the graph in its given order, whatever layout the width has
    Xl = graphgen.normal_rows(g.n, F, sets_o[1], 273)
    got = run_ifelse(full, paths, 0, Xl)
    rows = sets_o[2].astype(bool)
    assert np.all(got[~rows] == 123.0)
    assert_close(got[rows], oracle.path_aggregate(g.n, paths_o[0], Xl)[rows], f"if-else beside the partition F={F}")


def test_canonical_entries_are_given_back_and_rebuilt(monkeypatch):
    """While every prepared width of a path runs on its source-partitioned copy the canonical
    entry array is not kept; export, a further width without such a copy, and a new group size
    rebuild it from the copy bit for bit (the recorded section ids put every entry back in its
    row's order)."""
    g = graphgen.random_graph("rmat", 30_000, seed=271, raw_draws=400_000)
    train = graphgen.training_set(g.n, 3000, 272)
    sets_o, paths_o = oprep(g, train, 2)
    monkeypatch.setenv("EPP_TUNE_PART", "2")
    monkeypatch.setenv("EPP_TUNE_PART_KB", "64")
    monkeypatch.setenv("EPP_TUNE_PART_MINLEN", "8")
    # (with streamed-source marks: set by the copy itself where the canonical array is about to be given
    # back, on the canonical array where it stays)
    monkeypatch.setenv("EPP_TUNE_HOT_MB", "1")
    held = {}
    for keep in ("1", "0"):
        monkeypatch.setenv("EPP_TUNE_KEEP_CANONICAL", keep)
        paths = gpu_prepare(g, train, 2)
        p = paths.path(0)
        X = graphgen.normal_rows(g.n, 128, sets_o[1], 281)
        want = oracle.path_aggregate(g.n, paths_o[0], X)
        assert_close(run_partial(p, X), want, f"keep={keep} F=128")
        assert p.info().part_rows > 0
        held[keep] = p.info().bytes
        if keep == "0":
            assert held["0"] <= held["1"] - 8 * p.info().nnz  # the canonical entries are not held
        assert_paths_bit_exact(paths, sets_o, paths_o, 2)  # export rebuilds them
        monkeypatch.setenv("EPP_TUNE_PART", "1")  # a narrow width never gets a partitioned copy by itself
        X16 = graphgen.normal_rows(g.n, 16, sets_o[1], 282)
        assert_close(run_partial(p, X16), oracle.path_aggregate(g.n, paths_o[0], X16), f"keep={keep} F=16 after F=128")
        assert p.info().part_rows == 0 and p.info().bytes >= held["1"] - (1 << 20)  # now it is needed, and stays
        assert_close(run_partial(p, X), want, f"keep={keep} F=128 again")
        monkeypatch.setenv("EPP_TUNE_PART", "2")
        p.set_group_size(128, 48)
        assert_close(run_partial(p, X), want, f"keep={keep} F=128 gs=48")
        assert_paths_bit_exact(paths, sets_o, paths_o, 2)


@pytest.mark.parametrize("L", [2, 3])
@pytest.mark.parametrize("layout", ["plain", "partitioned", "cold"])
def test_inner_path_runs_on_the_entries_of_the_next_outer_path(monkeypatch, L, layout):
    """With nested active sets the path of layer l is a sub-sequence of the path of layer l - 1.
    Forced on at any overlap (EPP_TUNE_SHARE_PCT=1), the inner path keeps no entry arrays and
    runs on the outer path's: here it holds a minority of the outer path's entries and rows, so most
    entries are skipped and most rows must stay untouched.  Every row of every layer against the
    oracle at lane widths of 4, 8 and 16 bytes, with small groups that cut many rows, sources
    outside the layer's source set poisoned (the outer path's extra entries must not be read),
    rows outside the layer's row set untouched, bit-identical repeats, the exported canonical
    form bit-exact, and the memory the sharing saves."""
    g = graphgen.random_graph("rmat", 30_000, seed=371, raw_draws=400_000)
    train = graphgen.training_set(g.n, 1500, 372)
    sets_o, paths_o = oprep(g, train, L)
    if layout == "partitioned":
        monkeypatch.setenv("EPP_TUNE_PART", "2")
        monkeypatch.setenv("EPP_TUNE_PART_KB", "64")
        monkeypatch.setenv("EPP_TUNE_PART_MINLEN", "8")
    if layout == "cold":
        monkeypatch.setenv("EPP_TUNE_HOT_MB", "1")
    held = {}
    for pct in ("0", "1"):
        monkeypatch.setenv("EPP_TUNE_SHARE_PCT", pct)
        paths = gpu_prepare(g, train, L)
        shares = [paths.path(l).info().shares_entries for l in range(L)]
        # the innermost path shares with the next one; a path whose marks serve an inner path keeps its arrays
        assert shares == ([0] * L if pct == "0" else [0] * (L - 2) + [0, 1]), shares
        for l in range(L):
            src, rows = sets_o[L - l - 1], sets_o[L - l].astype(bool)
            p = paths.path(l)
            for F in (128, 41, 6) if layout != "cold" else (128, 130):
                X = graphgen.normal_rows(g.n, F, src, 373 + l)
                want = oracle.path_aggregate(g.n, paths_o[l], X)
                for gs in (0, 24):
                    p.set_group_size(F, gs)
                    got = run_partial(p, X, poison=9.0)
                    assert np.all(got[~rows] == 9.0), f"share {pct} {layout} l={l} F={F} gs={gs}: row outside the path written"
                    assert_close(got[rows], want[rows], f"share {pct} {layout} l={l} F={F} gs={gs}")
                    again = run_partial(p, X, poison=float("nan"))
                    assert np.array_equal(got[rows], again[rows])
                    Xp = X.copy()
                    Xp[src == 0] = np.nan
                    assert_close(run_partial(p, Xp), want, f"share {pct} {layout} l={l} F={F} gs={gs}, nan-poison")
                i = p.info()
                if layout == "partitioned":
                    assert i.part_rows > 0
                if pct == "1" and shares[l]:
                    assert i.n_groups >= -(-paths_o[l - 1].col.size // 24)  # groups of the outer path's entries
        assert_paths_bit_exact(paths, sets_o, paths_o, L)
        held[pct] = sum(paths.path(l).info().bytes for l in range(L))
        if pct == "1":
            # the launches of the inner path captured in a HIP graph: replays reproduce the eager result
            l, F = L - 1, 128
            p = paths.path(l)
            p.prepare_width(F)
            gin = torch.from_numpy(graphgen.normal_rows(g.n, F, sets_o[L - l - 1], 379)).to(dev())
            gout = torch.zeros_like(gin)
            epp.epp_backward_aggregate(p, gin, gout)
            torch.cuda.synchronize()
            eager = gout.clone()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                epp.epp_backward_aggregate(p, gin, gout)
            rows_t = torch.from_numpy(sets_o[L - l].astype(bool)).to(dev())
            for rep in range(3):
                gout.fill_(float(rep))
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert torch.equal(gout[rows_t], eager[rows_t]), f"replay {rep}"
                assert torch.all(gout[~rows_t] == float(rep)), f"replay {rep}: row outside the path written"
            del graph
    # the shared path holds row ids and row pointer only
    assert held["1"] <= held["0"] - 8 * paths_o[L - 1].col.size + (1 << 16), held


def test_marks_of_a_path_do_not_depend_on_the_order_of_its_widths(monkeypatch):
    """One path used at two widths: the streamed-source marks are those of the wider width,
    whichever was prepared first, and results stay within tolerance either way."""
    g = graphgen.random_graph("rmat", 30_000, seed=71, raw_draws=400_000)
    train = graphgen.training_set(g.n, 3000, 72)
    sets_o, paths_o = oprep(g, train, 2)
    monkeypatch.setenv("EPP_TUNE_HOT_MB", "1")
    outs = []
    for order in ((64, 128), (128, 64)):
        paths = gpu_prepare(g, train, 2)
        p = paths.path(0)
        for F in order:
            p.prepare_width(F)
        res = {}
        for F in (64, 128):
            X = graphgen.normal_rows(g.n, F, sets_o[1], 75)
            res[F] = run_partial(p, X)
            assert_close(res[F], oracle.path_aggregate(g.n, paths_o[0], X), f"order {order} F={F}")
        outs.append(res)
        assert_paths_bit_exact(paths, sets_o, paths_o, 2)
    for F in (64, 128):  # same marks, same schedule, same summation order
        assert np.array_equal(outs[0][F], outs[1][F])


def test_caller_allocator_owns_every_byte_and_aggregation_never_allocates():
    """With the PyTorch-backed epp_alloc_t every device buffer of the handles is a block of
    PyTorch's caching allocator: preparing allocates through it, the aggregate calls allocate
    nothing at all (neither through it nor behind its back), destroying the handles gives every
    block back.  Without it the library falls back to hipMalloc and PyTorch sees none of it."""
    import gc

    g = graphgen.random_graph("rmat", 20_000, seed=61, raw_draws=300_000)
    train = graphgen.training_set(g.n, 2000, 62)
    sets_o, paths_o = oprep(g, train, 2)
    d = dev()
    rowptr, col, val = (torch.from_numpy(a).to(d) for a in (g.rowptr, g.col, g.val))
    ids = torch.from_numpy(np.ascontiguousarray(train, np.int32)).to(d)
    F = 32
    X = graphgen.normal_rows(g.n, F, sets_o[1], 63)
    gin = torch.from_numpy(X).to(d)
    gout = torch.zeros_like(gin)
    want = oracle.path_aggregate(g.n, paths_o[0], X)
    gc.collect()
    torch.cuda.synchronize()
    for use_torch in (True, False):
        live0, allocs0 = epp.alloc_stats["live"], epp.alloc_stats["allocs"]
        mem0 = torch.cuda.memory_allocated()
        free0 = torch.cuda.mem_get_info()[0]
        paths = epp.epp_prepare(g.n, rowptr, col, val, ids, 2, torch_allocator=use_torch)
        full = epp.epp_prepare_full(g.n, rowptr, col, val, torch_allocator=use_torch)
        p = paths.path(0)
        p.set_group_size(F, 16)  # cut rows: partial rows are allocated too
        full.prepare_width(F)
        torch.cuda.synchronize()
        held = p.info().bytes + full.info().bytes
        if use_torch:
            assert epp.alloc_stats["allocs"] > allocs0 and epp.alloc_stats["live"] > live0
            assert torch.cuda.memory_allocated() - mem0 >= held  # PyTorch accounts for every byte held
        else:
            assert epp.alloc_stats["allocs"] == allocs0
            assert torch.cuda.memory_allocated() == mem0
        # the aggregate calls: no allocation of any kind, no change of the device's free memory
        a1, m1, f1 = epp.alloc_stats["allocs"], torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
        for _ in range(3):
            epp.epp_backward_aggregate(p, gin, gout)
            epp.epp_full_aggregate(full, gin, gout)
            epp.epp_ifelse_aggregate(full, paths, 0, gin, gout)
            gout.zero_()
            epp.epp_backward_aggregate(p, gin, gout)
        assert (epp.alloc_stats["allocs"], torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]) == (a1, m1, f1)
        torch.cuda.synchronize()
        assert_close(gout.cpu().numpy(), want, f"torch allocator {use_torch}")
        del p, paths, full
        gc.collect()
        assert epp.alloc_stats["live"] == live0
        assert torch.cuda.memory_allocated() == mem0
        del free0


def test_deep_model_shares_the_saturated_path(construction):
    """Once N^{k+1} == N^k every deeper layer has the same execution path: it is built once."""
    n = 40
    g = graphgen.csr_from_edges(n, [(i, (i + 1) % n) for i in range(n)], self_loops=True)
    L = n // 2 + 4
    paths = check_layers(g, [0], L, [5] * L, 90)
    handles = [paths.path(l)._h for l in range(L)]
    # N^20 = N^21 = ... = V: level 20 (layer 3) is built, levels 21..23 (layers 2, 1, 0) share it
    assert handles[0] == handles[1] == handles[2] == handles[3]
    assert len(set(handles)) == L - 3
    # without self-loops the sets alternate and never reach a fixed point: nothing is shared
    g2 = graphgen.csr_from_edges(n, [(i, (i + 1) % n) for i in range(n)], self_loops=False, normalise=False)
    paths2 = check_layers(g2, [0], 6, [3] * 6, 91)
    assert len({paths2.path(l)._h for l in range(6)}) == 6


def test_epoch_captured_in_a_hip_graph_replays_correctly():
    """The aggregate entry points only enqueue kernels (the one-off work of a width is done by
    epp_path_prepare_width), so a whole epoch can be captured in a HIP graph without any eager
    call before it; every replay must reproduce the oracle's result (rows cut by group
    boundaries are summed from per-group partial rows by a second kernel inside the graph)."""
    cfg = graphgen.make_config(1)
    g, L = cfg.graph, cfg.L
    sets_o, paths_o = oprep(g, cfg.train_ids, L)
    paths = gpu_prepare(g, cfg.train_ids, L)
    d = dev()
    xs = [torch.from_numpy(graphgen.layer_gradient(cfg, l, sets_o[L - l - 1])).to(d) for l in range(L)]
    ys = [torch.zeros_like(x) for x in xs]
    ps = [paths.path(l) for l in range(L)]
    want = [oracle.path_aggregate(g.n, paths_o[l], xs[l].cpu().numpy()) for l in range(L)]

    def epoch():
        for l in range(L - 1, -1, -1):
            epp.epp_backward_aggregate(ps[l], xs[l], ys[l])

    for l in range(L):
        ps[l].prepare_width(xs[l].shape[1])  # allocates, synchronises: must happen before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        epoch()
    for rep in range(4):
        for y in ys:
            y.normal_()          # eager work between replays; rows of the path must be overwritten
        rows = [torch.from_numpy(sets_o[L - l].astype(bool)).to(d) for l in range(L)]
        keep = [ys[l][~rows[l]].clone() for l in range(L)]
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            got = ys[l].cpu().numpy()
            r = sets_o[L - l].astype(bool)
            assert_close(got[r], want[l][r], f"replay {rep} layer {l}")
            assert torch.equal(ys[l][~rows[l]], keep[l])  # rows outside the path untouched


def test_randomised_shapes(construction, monkeypatch):
    """Many small random problems: graph shape, direction, self-loops, depth, width, group size, and
    (general construction) how readily consecutive paths share their entries."""
    rng = np.random.default_rng(2024)
    for case in range(60):
        monkeypatch.setenv("EPP_TUNE_SHARE_PCT", str((95, 1, 50, 0)[case % 4]))
        n = int(rng.integers(1, 700))
        m = int(rng.integers(0, 6 * n + 1))
        sym = bool(rng.integers(0, 2))
        loops = bool(rng.integers(0, 2))
        edges = [(int(u), int(v)) for u, v in rng.integers(0, n, (m, 2)) if u != v]
        if case % 7 == 0 and n > 3:  # a hub that gets cut into many groups
            edges += [(0, int(v)) for v in range(1, n)]
        g = graphgen.csr_from_edges(n, edges, self_loops=loops, symmetric=sym, normalise=sym)
        if not sym:
            g.val[:] = rng.uniform(-2.0, 2.0, g.nnz).astype(np.float32)
        L = int(rng.integers(1, 5))
        train = rng.choice(n, size=int(rng.integers(0, n + 1)), replace=True)
        sets_o, paths_o = oprep(g, train, L)
        paths = gpu_prepare(g, train, L)
        assert_paths_bit_exact(paths, sets_o, paths_o, L)
        full = gpu_prepare_full(g)
        for l in range(L):
            F = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 33, 64, 65, 128, 129, 260]))
            X = graphgen.normal_rows(g.n, F, sets_o[L - l - 1], 1000 + case)
            want = oracle.path_aggregate(g.n, paths_o[l], X)
            p = paths.path(l)
            gs = int(rng.choice([0, 1, 2, 5, 7, 16, 40, 1000]))
            p.set_group_size(F, gs)
            rows = sets_o[L - l].astype(bool)
            got = run_partial(p, X, poison=-7.0)
            assert np.all(got[~rows] == -7.0), f"case {case} l={l}"
            assert_close(got[rows], want[rows], f"case {case} l={l} F={F} gs={gs} n={n}")
            assert_close(run_full(full, X), oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X), f"case {case} full")
            ie = run_ifelse(full, paths, l, X)
            assert np.all(ie[~rows] == 123.0)
            assert_close(ie[rows], want[rows], f"case {case} l={l} if-else")


def test_import_of_saved_paths():
    """Pre-processing scenario: paths exported once, imported into a fresh handle, give the same
    canonical arrays, active sets and gradients; malformed arrays are refused, not executed."""
    g = graphgen.random_graph("rmat", 3000, seed=95, raw_draws=40_000)
    train = graphgen.training_set(g.n, 50, 96)
    L, F = 3, 24
    sets_o, paths_o = oprep(g, train, L)
    paths = gpu_prepare(g, train, L)
    saved = [paths.path(l).export() for l in range(L)]
    d = dev()
    ids = torch.from_numpy(np.ascontiguousarray(train, np.int32)).to(d)
    again = epp.epp_paths_import(g.n, ids, saved)
    assert_paths_bit_exact(again, sets_o, paths_o, L)
    full = gpu_prepare_full(g)
    for l in range(L):
        X = graphgen.normal_rows(g.n, F, sets_o[L - l - 1], 97 + l)
        want = oracle.path_aggregate(g.n, paths_o[l], X)
        rows = sets_o[L - l].astype(bool)
        got = run_partial(again.path(l), X, poison=4.0)
        assert np.all(got[~rows] == 4.0)
        assert_close(got[rows], want[rows], f"imported layer {l}")
        assert_close(run_ifelse(full, again, l, X)[rows], want[rows], f"if-else on imported sets, layer {l}")
    # malformed inputs
    row_ids, rowptr, col, val = saved[0]
    bad = row_ids.clone()
    bad[[0, 1]] = bad[[1, 0]]                                      # not ascending
    with pytest.raises(epp.EppError) as e:
        epp.epp_paths_import(g.n, ids, [(bad, rowptr, col, val)] + saved[1:])
    assert e.value.code == epp.EPP_ERR_INVALID_ARG
    bad = col.clone()
    bad[5] = g.n                                                   # column out of range
    with pytest.raises(epp.EppError) as e:
        epp.epp_paths_import(g.n, ids, [(row_ids, rowptr, bad, val)] + saved[1:])
    assert e.value.code == epp.EPP_ERR_OUT_OF_RANGE_ID
    bad = rowptr.clone()
    bad[-1] += 1                                                   # does not end at nnz
    with pytest.raises(epp.EppError) as e:
        epp.epp_paths_import(g.n, ids, [(row_ids, bad, col, val)] + saved[1:])
    assert e.value.code == epp.EPP_ERR_INVALID_ARG
    bad = rowptr.clone()
    bad[3] = bad[2]                                                # an empty row
    with pytest.raises(epp.EppError):
        epp.epp_paths_import(g.n, ids, [(row_ids, bad, col, val)] + saved[1:])
    with pytest.raises(epp.EppError) as e:                         # training id out of range
        epp.epp_paths_import(g.n, torch.tensor([g.n], dtype=torch.int32, device=d), saved)
    assert e.value.code == epp.EPP_ERR_OUT_OF_RANGE_ID
