"""Pins for the CPU oracle: things the paper and the mathematics fix, none of which is the
oracle's own formula re-typed.  CPU only."""
from pathlib import Path

import numpy as np
import pytest

import graphgen
import oracle

GOLDEN = Path(__file__).resolve().parent / "golden"


# ----------------------------------------------------------------------------- helpers
def dense_from_csr(g):
    """Scatter the CSR into a dense fp64 matrix with plain loops (no sparse code)."""
    M = np.zeros((g.n, g.n), np.float64)
    S = np.zeros((g.n, g.n), bool)
    for v in range(g.n):
        for j in range(g.rowptr[v], g.rowptr[v + 1]):
            M[v, g.col[j]] += float(g.val[j])
            S[v, g.col[j]] = True
    return M, S


def dense_sets(S, train, L):
    """N^k by dense boolean matrix-vector products: x_{k+1} = S x_k."""
    x = np.zeros(S.shape[0], bool)
    x[list(train)] = True
    out = [x]
    for _ in range(L):
        x = (S.astype(np.int64) @ x.astype(np.int64)) > 0
        out.append(x)
    return out


def triple_loop_product(M, X):
    n, F = X.shape
    out = [[0.0] * F for _ in range(n)]
    for v in range(n):
        for u in range(n):
            m = M[v, u]
            if m != 0.0:
                for f in range(F):
                    out[v][f] += m * float(X[u, f])
    return np.array(out, np.float64).reshape(n, F)


def random_small_graph(rng, n, p, symmetric, self_loops, normalise):
    edges = [(u, v) for u in range(n) for v in range(n) if u != v and rng.random() < p]
    if symmetric:
        edges = [(u, v) for (u, v) in edges if u < v]
    g = graphgen.csr_from_edges(n, edges, self_loops=self_loops, symmetric=symmetric, normalise=normalise)
    if not normalise:  # distinct, non-symmetric weights so a transposed operand shows
        g.val[:] = rng.uniform(0.25, 2.0, g.nnz).astype(np.float32)
    return g


def prep(g, train, L):
    return oracle.prepare(g.n, g.rowptr, g.col, g.val, np.asarray(train, np.int32), L)


def parse_golden(path):
    d = {}
    for line in path.read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split(":", 1)
        d[k.strip()] = v.split()
    return d


# ------------------------------------------------------------- paper's worked example
def test_worked_example_sec4():
    """Sec. 4 example: V_t = {v3, v5}, L = 2; the printed vertex sets and message edges."""
    gold = parse_golden(GOLDEN / "worked_example.txt")
    n = int(gold["vertices"][0])
    edges = [tuple(int(x) - 1 for x in e.split("-")) for e in gold["graph_edges"]]
    g = graphgen.csr_from_edges(n, edges, self_loops=False, symmetric=True, normalise=False)
    train = [int(x) - 1 for x in gold["training_set"]]
    L = int(gold["layers"][0])
    sets, paths = prep(g, train, L)
    for l in range(L):
        want_rows = sorted(int(x) - 1 for x in gold[f"layer{l}_vertices"])
        want_edges = sorted(tuple(int(x) - 1 for x in e.split(">")) for e in gold[f"layer{l}_edges"])
        p = paths[l]
        assert p.row_ids.tolist() == want_rows
        assert np.flatnonzero(sets[L - l]).tolist() == want_rows
        got = sorted((int(p.col[j]), int(p.row_ids[r]))
                     for r in range(len(p.row_ids)) for j in range(p.rowptr[r], p.rowptr[r + 1]))
        assert got == want_edges
    # canonical CSR of both sub-graphs, derived by hand from the printed edge lists
    assert paths[1].rowptr.tolist() == [0, 2, 4] and paths[1].col.tolist() == [2, 4, 2, 4]
    assert paths[0].rowptr.tolist() == [0, 1, 2, 4, 5, 7] and paths[0].col.tolist() == [1, 3, 1, 3, 1, 1, 3]
    # N^1 does not contain V_t: k-neighbours are reached by exactly k edges
    assert np.flatnonzero(sets[1]).tolist() == [1, 3]
    # Sec. 2.2: group size 3 cuts v2's list (4 entries in the input graph) into 2 groups
    gs = int(gold["group_size"][0])
    len_v2 = int(g.rowptr[2] - g.rowptr[1])
    assert -(-len_v2 // gs) == int(gold["v2_groups"][0])


def test_worked_example_extra_pendant_vertex_changes_nothing():
    """A vertex hanging off v1 (not adjacent to v2/v4) is outside both paths."""
    edges = [(0, 1), (1, 2), (1, 3), (1, 4), (2, 3), (3, 4), (0, 5)]
    g = graphgen.csr_from_edges(6, edges, self_loops=False, normalise=False)
    _, paths = prep(g, [2, 4], 2)
    assert paths[1].row_ids.tolist() == [1, 3] and paths[1].col.tolist() == [2, 4, 2, 4]
    assert paths[0].row_ids.tolist() == [0, 1, 2, 3, 4] and paths[0].col.tolist() == [1, 3, 1, 3, 1, 1, 3]


# ------------------------------------------------------------------- dense brute force
@pytest.mark.parametrize("seed", range(6))
def test_sets_paths_and_values_against_dense(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 40))
    symmetric, self_loops, normalise = bool(seed & 1), bool(seed & 2), bool(seed & 1)
    g = random_small_graph(rng, n, 0.12, symmetric, self_loops, normalise)
    M, S = dense_from_csr(g)
    L = 3
    train = rng.choice(n, size=max(1, n // 6), replace=False)
    sets, paths = prep(g, train, L)
    dsets = dense_sets(S, train, L)
    for k in range(L + 1):
        assert np.array_equal(sets[k].astype(bool), dsets[k]), k
    for l in range(L):
        rows, src = dsets[L - l], dsets[L - l - 1]
        want_rows = np.flatnonzero(rows)
        p = paths[l]
        assert p.row_ids.tolist() == want_rows.tolist()
        cols, vals, ptr = [], [], [0]
        for v in want_rows:
            for u in range(n):          # ascending = input order
                if S[v, u] and src[u]:
                    cols.append(u)
                    vals.append(np.float32(M[v, u]))
            ptr.append(len(cols))
        assert p.col.tolist() == cols and p.rowptr.tolist() == ptr
        assert np.array_equal(p.val, np.array(vals, np.float32))
        F = int(rng.integers(1, 9))
        X = rng.standard_normal((n, F)).astype(np.float32)
        X[~src] = 0.0
        want = M @ X.astype(np.float64)
        np.testing.assert_allclose(oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X), want, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(oracle.path_aggregate(g.n, p, X), want, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(
            oracle.partial_aggregate(g.n, g.rowptr, g.col, g.val, sets[L - l], sets[L - l - 1], X),
            want, rtol=1e-6, atol=1e-7)


def test_full_aggregate_against_triple_loop():
    rng = np.random.default_rng(7)
    g = random_small_graph(rng, 17, 0.25, False, False, False)
    M, _ = dense_from_csr(g)
    X = rng.standard_normal((17, 5)).astype(np.float32)
    want = triple_loop_product(M, X)
    got = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X)
    assert np.array_equal(got, want.astype(np.float32))  # fp64 sum rounded once: exact match expected


def test_direction_on_directed_chain():
    """0 -> 1 -> 2 (u -> v puts u in row v).  Gradients flow along the arrows only."""
    g = graphgen.csr_from_edges(3, [(0, 1), (1, 2)], self_loops=False, symmetric=False, normalise=False)
    sets, paths = prep(g, [0], 2)
    assert [np.flatnonzero(s).tolist() for s in sets] == [[0], [1], [2]]
    assert paths[1].row_ids.tolist() == [1] and paths[1].col.tolist() == [0]
    assert paths[0].row_ids.tolist() == [2] and paths[0].col.tolist() == [1]
    sets, paths = prep(g, [2], 2)  # nothing pulls from vertex 2
    assert [int(s.sum()) for s in sets] == [1, 0, 0]
    assert all(p.row_ids.size == 0 and p.col.size == 0 and p.rowptr.tolist() == [0] for p in paths)


# ------------------------------------------------------------------------ closed forms
def test_complete_graph_gives_column_means():
    n, F = 9, 4
    g = graphgen.csr_from_edges(n, [(u, v) for u in range(n) for v in range(u)], self_loops=True)
    X = np.random.default_rng(1).standard_normal((n, F)).astype(np.float32)
    out = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X)
    np.testing.assert_allclose(out, np.tile(X.astype(np.float64).mean(0), (n, 1)), rtol=2e-6, atol=1e-7)
    sets, paths = prep(g, [3], 2)
    assert all(int(s.sum()) == n for s in sets[1:])
    assert paths[1].col.tolist() == [3] * n and paths[0].col.size == n * n


def test_star_graph_closed_form():
    n, F = 7, 3  # centre 0, leaves 1..6; with self-loops d_0 = n, d_leaf = 2
    g = graphgen.csr_from_edges(n, [(0, v) for v in range(1, n)], self_loops=True)
    X = np.random.default_rng(2).standard_normal((n, F)).astype(np.float64)
    out = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X.astype(np.float32))
    X = X.astype(np.float32).astype(np.float64)
    want = np.empty_like(X)
    want[0] = X[0] / n + X[1:].sum(0) / np.sqrt(2.0 * n)
    want[1:] = X[1:] / 2.0 + X[0] / np.sqrt(2.0 * n)
    np.testing.assert_allclose(out, want, rtol=2e-6, atol=1e-7)
    sets, _ = prep(g, [4], 2)
    assert np.flatnonzero(sets[1]).tolist() == [0, 4]
    assert int(sets[2].sum()) == n


def test_path_graph_frontiers_with_and_without_self_loops():
    n = 8
    chain = [(i, i + 1) for i in range(n - 1)]
    g = graphgen.csr_from_edges(n, chain, self_loops=False, normalise=False)
    sets, _ = prep(g, [0], 4)
    assert [np.flatnonzero(s).tolist() for s in sets] == [[0], [1], [0, 2], [1, 3], [0, 2, 4]]
    g = graphgen.csr_from_edges(n, chain, self_loops=True)
    sets, paths = prep(g, [0], 3)
    assert [np.flatnonzero(s).tolist() for s in sets] == [[0], [0, 1], [0, 1, 2], [0, 1, 2, 3]]
    # monotone growth with self-loops, every path row non-empty
    assert all(np.all(np.diff(p.rowptr) >= 1) for p in paths)
    assert [p.col.size for p in paths] == sorted(p.col.size for p in paths)[::-1]


def test_identity_graph():
    n = 6
    g = graphgen.csr_from_edges(n, [], self_loops=True)
    train = [1, 4]
    sets, paths = prep(g, train, 3)
    for s in sets:
        assert np.flatnonzero(s).tolist() == train
    X = graphgen.normal_rows(n, 5, sets[0], 3)
    for p in paths:
        assert p.row_ids.tolist() == train and p.col.tolist() == train
        assert np.array_equal(oracle.path_aggregate(n, p, X), X)


# --------------------------------------------------------------------- special cases
def test_special_training_sets():
    rng = np.random.default_rng(11)
    g = random_small_graph(rng, 30, 0.1, True, False, True)
    deg = np.diff(g.rowptr)
    # V_t = V: every path is the whole CSR minus rows with empty lists
    sets, paths = prep(g, np.arange(g.n), 2)
    for p in paths:
        assert p.row_ids.tolist() == np.flatnonzero(deg > 0).tolist()
        assert np.array_equal(p.col, g.col) and np.array_equal(p.val, g.val)
    # V_t empty
    sets, paths = prep(g, [], 2)
    assert all(s.sum() == 0 for s in sets) and all(p.col.size == 0 and p.row_ids.size == 0 for p in paths)
    # duplicates collapse
    a = prep(g, [3, 3, 7, 3], 2)
    b = prep(g, [7, 3], 2)
    for pa, pb in zip(a[1], b[1]):
        assert np.array_equal(pa.row_ids, pb.row_ids) and np.array_equal(pa.col, pb.col)
    # out-of-range id is an error
    with pytest.raises(ValueError):
        prep(g, [g.n], 1)
    with pytest.raises(ValueError):
        prep(g, [-1], 1)


def test_isolated_training_vertex_without_self_loop_contributes_nothing():
    g = graphgen.csr_from_edges(5, [(0, 1), (1, 2)], self_loops=False, normalise=False)
    sets, paths = prep(g, [4], 2)  # vertex 4 has no edges
    assert all(p.row_ids.size == 0 for p in paths) and sets[1].sum() == 0


def test_saturation_when_L_reaches_diameter():
    rng = np.random.default_rng(5)
    n = 40
    ring = [(i, (i + 1) % n) for i in range(n)]
    g = graphgen.csr_from_edges(n, ring, self_loops=True)
    sets, paths = prep(g, [0], n // 2 + 1)
    assert int(sets[-1].sum()) == n and int(sets[-2].sum()) == n
    assert np.array_equal(paths[0].col, g.col)  # last path is the whole graph


# ------------------------------------------------- Theorem 1 and library cross-check
@pytest.mark.parametrize("k", [1, 2])
def test_theorem1_and_scipy_on_small_configs(k):
    import scipy.sparse as sp

    cfg = graphgen.make_config(k)
    g = cfg.graph
    assert g.undirected_edges == cfg.target_edges and g.nnz == 2 * cfg.target_edges + g.n
    sets, paths = prep(g, cfg.train_ids, cfg.L)
    assert int(sets[0].sum()) == cfg.n_train
    A = sp.csr_matrix((g.val.astype(np.float64), g.col, g.rowptr), shape=(g.n, g.n))
    for l in range(cfg.L):
        rows, src = sets[cfg.L - l], sets[cfg.L - l - 1]
        X = graphgen.layer_gradient(cfg, l, src)
        assert not X[src == 0].any() and X[src != 0].all()
        full = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X)
        part = oracle.path_aggregate(g.n, paths[l], X)
        direct = oracle.partial_aggregate(g.n, g.rowptr, g.col, g.val, rows, src, X)
        # Alg. 2 gives exactly Alg. 1's result; rows outside N^{L-l} are exactly zero
        assert np.array_equal(full, part) and np.array_equal(full, direct)
        assert not full[rows == 0].any()
        np.testing.assert_allclose(full, A @ X.astype(np.float64), rtol=1e-6, atol=1e-7)
        # NaN poison: rows outside the source set are never read by the partial forms
        Xp = X.copy()
        Xp[src == 0] = np.nan
        assert np.array_equal(oracle.path_aggregate(g.n, paths[l], Xp), part)
        # with self-loops the sets grow monotonically
        assert not (src & ~rows).any()


def test_checksum_identities_medium_graph():
    """Column-sum and adjoint identities, computable without any sparse product."""
    g = graphgen.random_graph("rmat", 5000, seed=77, raw_draws=60000)
    F = 6
    X = graphgen.normal_rows(g.n, F, None, 5)
    out = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, X).astype(np.float64)
    colsum = np.zeros(g.n)
    np.add.at(colsum, g.col, g.val.astype(np.float64))
    np.testing.assert_allclose(out.sum(0), colsum @ X.astype(np.float64), rtol=1e-5, atol=1e-5)
    Y = np.random.default_rng(9).standard_normal((g.n, F))
    # <M X, Y> = <X, M^T Y>;  M^T Y accumulated edge by edge
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    MtY = np.zeros((g.n, F))
    np.add.at(MtY, g.col, g.val.astype(np.float64)[:, None] * Y[rows])
    np.testing.assert_allclose((out * Y).sum(), (X.astype(np.float64) * MtY).sum(), rtol=1e-6)


# ---------------------------------------------------------------- generator hygiene
def test_generator_invariants():
    g = graphgen.random_graph("chung_lu", 3000, seed=5, target_edges=7000)
    assert g.undirected_edges == 7000 and g.nnz == 2 * 7000 + 3000
    deg = np.diff(g.rowptr)
    rows = np.repeat(np.arange(g.n), deg)
    # ascending unique columns, self-loop present, structurally and numerically symmetric
    assert np.all((np.diff(g.col) > 0) | (np.diff(rows) > 0))
    assert np.all(np.isin(np.arange(g.n) * g.n + np.arange(g.n), rows.astype(np.int64) * g.n + g.col))
    import scipy.sparse as sp
    A = sp.csr_matrix((g.val, g.col, g.rowptr), shape=(g.n, g.n))
    assert (A != A.T).nnz == 0
    want = (1.0 / np.sqrt(deg[rows].astype(np.float64) * deg[g.col].astype(np.float64))).astype(np.float32)
    assert np.array_equal(g.val, want)
    g2 = graphgen.random_graph("chung_lu", 3000, seed=5, target_edges=7000)
    assert np.array_equal(g.col, g2.col) and np.array_equal(g.rowptr, g2.rowptr)
    t = graphgen.training_set(3000, 100, 1)
    assert len(set(t.tolist())) == 100
    tb = graphgen.training_set(3000, 100, 1, deg)
    assert len(set(tb.tolist())) == 100 and deg[tb].mean() > deg.mean()


def test_strided_row_sample_equals_the_full_result_on_the_sampled_rows():
    """oracle.path_aggregate(first, stride) is what the benchmark's cpu_baseline times: it must
    compute exactly the rows first, first + stride, ... of the full result and leave all others zero."""
    g = graphgen.random_graph("rmat", 3000, seed=5, raw_draws=40_000)
    train = graphgen.training_set(g.n, 200, 6)
    sets, paths = oracle.prepare(g.n, g.rowptr, g.col, g.val, train, 2)
    for l in range(2):
        X = graphgen.normal_rows(g.n, 5, sets[2 - l - 1], 7 + l)
        full = oracle.path_aggregate(g.n, paths[l], X)  # (pinned by the dense products above)
        assert full[paths[l].row_ids].any()
        R = paths[l].row_ids.size
        for first, stride in ((0, 1), (0, 7), (3, 7), (6, 7), (R - 1, R), (0, R + 5), (R, 3)):
            part = oracle.path_aggregate(g.n, paths[l], X, first=first, stride=stride)
            picked = paths[l].row_ids[first::stride]
            mask = np.zeros(g.n, bool)
            mask[picked] = True
            assert np.array_equal(part[mask], full[mask]), (l, first, stride)
            assert not part[~mask].any(), (l, first, stride)
