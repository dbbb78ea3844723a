"""Pins of the oracle's combination stage (Alg. 1, backward loop: W' = Y^T (x) X' and
Y' = X' (x) W^T), none of which re-uses the oracle's own matrix products."""
import numpy as np
import pytest

import graphgen
import oracle


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(np.float32)


def test_loop_by_loop_brute_force():
    n, fi, fo = 7, 3, 2
    Y, G, W = _rand((n, fi), 1), _rand((n, fo), 2), _rand((fi, fo), 3)
    member = np.array([1, 0, 1, 1, 0, 0, 1], np.uint8)
    for m in (None, member):
        Wg = np.zeros((fi, fo))
        Yg = np.zeros((n, fi))
        for v in range(n):
            if m is not None and not m[v]:
                continue
            for i in range(fi):
                for j in range(fo):
                    Wg[i, j] += float(Y[v, i]) * float(G[v, j])   # line "W' = Y^T (x) X'"
                    Yg[v, i] += float(G[v, j]) * float(W[i, j])   # line "Y' = X' (x) W^T"
        got_w, scale_w = oracle.weight_gradient(Y, G, m)
        got_y, scale_y = oracle.input_gradient(G, W, m)
        assert got_w.shape == (fi, fo) and got_y.shape == (n, fi)
        assert np.allclose(got_w, Wg, rtol=0, atol=1e-12)
        assert np.array_equal(got_y, Yg.astype(np.float32))
        assert np.all(scale_w >= np.abs(got_w) - 1e-12) and np.all(scale_y >= np.abs(Yg) - 1e-12)


def test_closed_forms():
    n, f = 11, 5
    G = _rand((n, f), 4)
    # W = identity: Y' = X'
    y, _ = oracle.input_gradient(G, np.eye(f, dtype=np.float32))
    assert np.array_equal(y, G)
    # W = a single 1 at (i, j): column i of Y' is column j of X', everything else zero
    W = np.zeros((3, f), np.float32)
    W[2, 4] = 1.0
    y, _ = oracle.input_gradient(G, W)
    assert np.array_equal(y[:, 2], G[:, 4]) and not y[:, :2].any()
    # Y = all ones: every row of W' is the column sum of X'
    w, _ = oracle.weight_gradient(np.ones((n, 3), np.float32), G)
    assert np.allclose(w, np.tile(G.astype(np.float64).sum(0), (3, 1)), atol=1e-12)
    # X' has one non-zero entry (v, j): W'[:, j] = Y[v, :] * value
    Y = _rand((n, 3), 5)
    E = np.zeros((n, f), np.float32)
    E[6, 1] = 2.5
    w, _ = oracle.weight_gradient(Y, E)
    assert np.allclose(w[:, 1], 2.5 * Y[6].astype(np.float64)) and not np.delete(w, 1, axis=1).any()


def test_trace_identity_links_the_two_products():
    """<W, W'>_F = <Y, Y'>_F  (both equal sum_v Y_v W X'_v^T): fails for a transposed operand
    in either product."""
    n, fi, fo = 40, 6, 9
    Y, G, W = _rand((n, fi), 6), _rand((n, fo), 7), _rand((fi, fo), 8)
    member = (np.arange(n) % 3 != 0).astype(np.uint8)
    for m in (None, member):
        w, _ = oracle.weight_gradient(Y, G, m)
        y, _ = oracle.input_gradient(G, W, m)
        lhs = float((W.astype(np.float64) * w).sum())
        rhs = float((Y.astype(np.float64) * y.astype(np.float64)).sum())
        assert abs(lhs - rhs) <= 1e-5 * max(1.0, abs(lhs))


def test_restricted_equals_unrestricted_when_skipped_rows_are_zero():
    """Theorem 1's consequence for the combination stage: all-zero rows of X' add nothing."""
    n, fi, fo = 60, 4, 7
    member = (np.arange(n) % 4 == 1).astype(np.uint8)
    G = _rand((n, fo), 9) * member[:, None]
    Y, W = _rand((n, fi), 10), _rand((fi, fo), 11)
    w_all, _ = oracle.weight_gradient(Y, G)
    w_res, _ = oracle.weight_gradient(Y, G, member)
    assert np.allclose(w_all, w_res, rtol=0, atol=1e-12)
    y_all, _ = oracle.input_gradient(G, W)
    y_res, _ = oracle.input_gradient(G, W, member)
    assert np.array_equal(y_all, y_res) and not y_res[member == 0].any()


@pytest.mark.parametrize("seed", [0, 1])
def test_finite_differences_of_the_forward_model(seed):
    """Forward model of Alg. 1 without the activation: Y = A X0, X1 = Y W, loss = <R, X1>.
    Its gradients are dl/dW = Y^T R (= Y^T X' with X' = R) and dl/dX0 = A^T (R W^T), i.e. the
    backward aggregation of Y' = X' W^T.  Checked by central differences in fp64 on a dense copy of the
    graph; the backward operator handed to the oracle is the transpose of the forward one."""
    g = graphgen.random_graph("chung_lu", 30, seed=300 + seed, target_edges=60)
    n, fi, fo = g.n, 3, 4
    A = np.zeros((n, n))
    for v in range(n):
        A[v, g.col[g.rowptr[v]:g.rowptr[v + 1]]] = g.val[g.rowptr[v]:g.rowptr[v + 1]]
    rng = np.random.Generator(np.random.PCG64(seed))
    A = A * rng.uniform(0.5, 1.5, A.shape)  # make it non-symmetric: forward A, backward A^T
    X0 = rng.standard_normal((n, fi))
    W = rng.standard_normal((fi, fo))
    R = rng.standard_normal((n, fo))

    def loss(X0_, W_):
        return float((R * ((A @ X0_) @ W_)).sum())

    Y = A @ X0
    w, _ = oracle.weight_gradient(Y.astype(np.float32), R.astype(np.float32))
    yg, _ = oracle.input_gradient(R.astype(np.float32), W.astype(np.float32))
    # backward operator M = A^T in CSR
    At = A.T
    rowptr = np.zeros(n + 1, np.int32)
    col, val = [], []
    for v in range(n):
        nz = np.flatnonzero(At[v])
        col += nz.tolist()
        val += At[v, nz].tolist()
        rowptr[v + 1] = len(col)
    xg = oracle.full_aggregate(n, rowptr, np.array(col, np.int32), np.array(val, np.float32), yg)
    h = 1e-4
    for (i, j) in [(0, 0), (2, 3), (1, 2)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[i, j] += h
        Wm[i, j] -= h
        fd = (loss(X0, Wp) - loss(X0, Wm)) / (2 * h)
        assert abs(fd - w[i, j]) <= 1e-4 * max(1.0, abs(fd))
    for (v, i) in [(0, 0), (7, 2), (29, 1)]:
        Xp, Xm = X0.copy(), X0.copy()
        Xp[v, i] += h
        Xm[v, i] -= h
        fd = (loss(Xp, W) - loss(Xm, W)) / (2 * h)
        assert abs(fd - xg[v, i]) <= 1e-4 * max(1.0, abs(fd))
