"""GPU parity of the combination stage on the active rows (Alg. 1, backward loop:
W' = Y^T (x) X', Y' = X' (x) W^T) against the fp64 oracle, through the C ABI.

Tolerance: every output is a dot product; any fp32 evaluation order is within
c * 2^-24 * sum_k |a_k b_k| of the exact value (c = number of additions on the longest chain;
the kernels keep chains to a few thousand and add the partial sums in double).  The test uses
|gpu - oracle| <= 1e-6 + 1e-5 * sum_k |a_k b_k|, the aggregation's tolerance with the condition-
free scale the oracle returns in place of |oracle|."""
import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2204_02662_amd as epp
from _util import dev, gpu_prepare, run_partial

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(np.float32)


def _close(got, want, scale, what):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bound = 1e-6 + 1e-5 * scale
    assert np.isfinite(got).all(), what
    assert (err <= bound).all(), f"{what}: worst {float((err - bound).max()):.3e} over the bound"


def _weight_gradient(paths, k, Y, G):
    d = dev()
    Yd, Gd = torch.from_numpy(Y).to(d), torch.from_numpy(G).to(d)
    Wg = torch.full((Y.shape[1], G.shape[1]), 5.0, device=d)
    ws = torch.empty(epp.epp_weight_gradient_workspace(paths, k, Y.shape[1], G.shape[1]), dtype=torch.uint8, device=d)
    epp.epp_weight_gradient(paths, k, Yd, Gd, Wg, ws)
    torch.cuda.synchronize()
    return Wg.cpu().numpy()


def _input_gradient(paths, k, G, W, poison=77.0):
    d = dev()
    Gd, Wd = torch.from_numpy(G).to(d), torch.from_numpy(W).to(d)
    Yg = torch.full((G.shape[0], W.shape[0]), poison, device=d)
    epp.epp_input_gradient(paths, k, Gd, Wd, Yg)
    torch.cuda.synchronize()
    return Yg.cpu().numpy()


SHAPES = [(1, 1), (3, 7), (16, 16), (41, 16), (16, 47), (64, 64), (65, 33), (40, 100), (128, 16), (130, 70)]


@pytest.mark.parametrize("Fi,Fo", SHAPES)
def test_combination_small_graphs(Fi, Fo):
    g = graphgen.random_graph("rmat", 1500, seed=400, raw_draws=9000)
    train = graphgen.training_set(g.n, 40, 401)
    L = 2
    sets_o, _ = oracle.prepare(g.n, g.rowptr, g.col, g.val, train, L)
    paths = gpu_prepare(g, train, L)
    Y, W = _rand((g.n, Fi), 402), _rand((Fi, Fo), 403)
    for k in (0, 1, 2, -1):
        member = None if k < 0 else sets_o[k]
        G = _rand((g.n, Fo), 404 + k)
        if member is not None:
            G[member == 0] = np.nan  # rows outside N^k must never be read
        want_w, scale_w = oracle.weight_gradient(Y, np.nan_to_num(G), member)
        got_w = _weight_gradient(paths, k, Y, G)
        _close(got_w, want_w, scale_w, f"W' k={k}")
        want_y, scale_y = oracle.input_gradient(np.nan_to_num(G), W, member)
        got_y = _input_gradient(paths, k, G, W)
        rows = np.ones(g.n, bool) if member is None else member.astype(bool)
        assert np.all(got_y[~rows] == 77.0), "rows outside N^k were written"
        _close(got_y[rows], want_y[rows], scale_y[rows], f"Y' k={k}")


def test_combination_many_rows_per_partial_sum():
    """More rows than one block of partial sums holds, ragged tail, all vertices active."""
    g = graphgen.random_graph("chung_lu", 70_001, seed=410, target_edges=150_000)
    train = np.arange(g.n, dtype=np.int32)
    paths = gpu_prepare(g, train, 1)
    Y, G, W = _rand((g.n, 24), 411), _rand((g.n, 10), 412), _rand((24, 10), 413)
    want_w, scale_w = oracle.weight_gradient(Y, G)
    for k in (0, 1, -1):
        _close(_weight_gradient(paths, k, Y, G), want_w, scale_w, f"W' k={k}")
    want_y, scale_y = oracle.input_gradient(G, W)
    _close(_input_gradient(paths, 0, G, W), want_y, scale_y, "Y'")


def test_combination_empty_and_errors():
    g = graphgen.random_graph("chung_lu", 300, seed=420, target_edges=600)
    paths = gpu_prepare(g, np.zeros(0, np.int32), 2)
    Y, G, W = _rand((g.n, 5), 421), _rand((g.n, 4), 422), _rand((5, 4), 423)
    assert not _weight_gradient(paths, 1, Y, G).any()            # empty N^k: W' = 0
    assert np.all(_input_gradient(paths, 1, G, W) == 77.0)       # and no row of Y' is written
    d = dev()
    Yd, Gd = torch.from_numpy(Y).to(d), torch.from_numpy(G).to(d)
    Wg = torch.zeros(5, 4, device=d)
    need = epp.epp_weight_gradient_workspace(paths, -1, 5, 4)
    assert need >= 5 * 4 * 4
    with pytest.raises(epp.EppError) as e:
        epp.epp_weight_gradient(paths, -1, Yd, Gd, Wg, torch.empty(need - 1, dtype=torch.uint8, device=d))
    assert e.value.code == epp.EPP_ERR_INVALID_ARG
    for bad_k in (-2, 3):
        with pytest.raises(epp.EppError):
            epp.epp_weight_gradient_workspace(paths, bad_k, 5, 4)
        with pytest.raises(epp.EppError):
            epp.epp_input_gradient(paths, bad_k, Gd, torch.from_numpy(W).to(d), torch.zeros(g.n, 5, device=d))
    with pytest.raises(ValueError):
        epp.epp_input_gradient(paths, 0, Gd[:-1].contiguous(), torch.from_numpy(W).to(d), torch.zeros(g.n - 1, 5, device=d))


def test_backward_chain_matches_the_dense_model():
    """Three layers of Alg. 1's backward loop (combination on active rows, then Alg. 2's
    aggregation over SG_l) against the same chain in the oracle on all vertices."""
    g = graphgen.random_graph("rmat", 4000, seed=430, raw_draws=30_000)
    train = graphgen.training_set(g.n, 25, 431)
    L, widths = 3, [12, 20, 9, 6]  # F_0 .. F_3
    sets_o, paths_o = oracle.prepare(g.n, g.rowptr, g.col, g.val, train, L)
    paths = gpu_prepare(g, train, L)
    G = np.zeros((g.n, widths[L]), np.float32)
    G[sets_o[0] == 1] = _rand((int(sets_o[0].sum()), widths[L]), 432)
    G_o = G.copy()
    for l in range(L - 1, -1, -1):
        k = L - l - 1
        Y, W = _rand((g.n, widths[l]), 440 + l), _rand((widths[l], widths[l + 1]), 450 + l) / 4
        want_w, scale_w = oracle.weight_gradient(Y, G_o)           # all vertices: the definition
        _close(_weight_gradient(paths, k, Y, G), want_w, scale_w, f"W' l={l}")
        yg_o, scale_y = oracle.input_gradient(G_o, W)
        yg = _input_gradient(paths, k, G, W, poison=0.0)
        _close(yg, yg_o, scale_y, f"Y' l={l}")
        G_o = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, yg_o)
        G = run_partial(paths.path(l), yg)
        assert not G[sets_o[k + 1] == 0].any()
        # the inputs of the two chains differ by rounding only; compare loosely here, the tight
        # per-operation checks are above
        assert np.allclose(G, G_o, rtol=1e-4, atol=1e-5)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("cfg_id", [4, 5])
def test_combination_at_benchmark_sizes(cfg_id):
    """Full-size configurations, widths as the combine study times them (F_L = F_{L-1}).
    W' is a reduction over millions of rows: the oracle computes a sampled 6 x 5 block of it
    (all rows, fp64); Y' is checked on every 997th active row, every column."""
    cfg = graphgen.make_config(cfg_id)
    g, L = cfg.graph, cfg.L
    print(f"[cfg {cfg_id}] oracle sets", flush=True)
    sets_o = oracle.active_sets(g.n, g.rowptr, g.col, cfg.train_ids, L)
    paths = gpu_prepare(g, cfg.train_ids, L)
    widths = list(cfg.widths) + [cfg.widths[L - 1]]
    d = dev()
    for l in range(L - 1, -1, -1):
        k = L - l - 1
        Fi, Fo = widths[l], widths[l + 1]
        member = sets_o[k]
        print(f"[cfg {cfg_id}] layer {l}: {Fi} x {Fo}, {int(member.sum())} active rows", flush=True)
        gen = torch.Generator(device=d)
        gen.manual_seed(cfg.seed(40 + l))
        Y = torch.randn(g.n, Fi, generator=gen, device=d)
        W = torch.randn(Fi, Fo, generator=gen, device=d)
        G = torch.randn(g.n, Fo, generator=gen, device=d)
        G[torch.from_numpy(member == 0).to(d)] = float("nan")  # never read outside N^k
        Wg = torch.empty(Fi, Fo, device=d)
        Yg = torch.full((g.n, Fi), 3.0, device=d)
        ws = torch.empty(epp.epp_weight_gradient_workspace(paths, k, Fi, Fo), dtype=torch.uint8, device=d)
        epp.epp_weight_gradient(paths, k, Y, G, Wg, ws)
        epp.epp_input_gradient(paths, k, G, W, Yg)
        torch.cuda.synchronize()
        Yh, Gh = Y.cpu().numpy(), np.nan_to_num(G.cpu().numpy())
        I = np.unique(np.linspace(0, Fi - 1, 6).astype(int))
        J = np.unique(np.linspace(0, Fo - 1, 5).astype(int))
        want_w, scale_w = oracle.weight_gradient(Yh[:, I], Gh[:, J], member)
        _close(Wg.cpu().numpy()[np.ix_(I, J)], want_w, scale_w, f"cfg {cfg_id} W' l={l}")
        rows = np.flatnonzero(member)[::997]
        sample = np.zeros(g.n, np.uint8)
        sample[rows] = 1
        want_y, scale_y = oracle.input_gradient(Gh, W.cpu().numpy(), sample)
        got_y = Yg.cpu().numpy()
        _close(got_y[rows], want_y[rows], scale_y[rows], f"cfg {cfg_id} Y' l={l}")
        assert np.all(got_y[member == 0] == 3.0)
        del Y, W, G, Wg, Yg, ws, Yh, Gh, got_y, want_y, scale_y


def test_backward_epoch_in_a_hip_graph():
    """Combination and aggregation of every layer, chained as in Alg. 1's backward loop, captured
    once in a HIP graph (after the widths have been prepared and a first eager epoch has run)
    and replayed with eager work in between: every replay must equal the eager epoch bit for bit
    on the weight gradients (fixed summation order) and within tolerance of the oracle chain."""
    g = graphgen.random_graph("chung_lu", 6000, seed=460, target_edges=30_000)
    train = graphgen.training_set(g.n, 60, 461)
    L, widths = 2, [24, 16, 8]
    sets_o, _ = oracle.prepare(g.n, g.rowptr, g.col, g.val, train, L)
    paths = gpu_prepare(g, train, L)
    d = dev()
    Ys = [torch.from_numpy(_rand((g.n, widths[l]), 462 + l)).to(d) for l in range(L)]
    Ws = [torch.from_numpy(_rand((widths[l], widths[l + 1]), 465 + l) / 4).to(d) for l in range(L)]
    G_top = np.zeros((g.n, widths[L]), np.float32)
    G_top[sets_o[0] == 1] = _rand((int(sets_o[0].sum()), widths[L]), 468)
    Gs = [torch.zeros(g.n, widths[l], device=d) for l in range(L)] + [torch.from_numpy(G_top).to(d)]
    Ygs = [torch.zeros(g.n, widths[l], device=d) for l in range(L)]
    Wgs = [torch.empty(widths[l], widths[l + 1], device=d) for l in range(L)]
    wss = [torch.empty(epp.epp_weight_gradient_workspace(paths, L - l - 1, widths[l], widths[l + 1]),
                       dtype=torch.uint8, device=d) for l in range(L)]
    ps = [paths.path(l) for l in range(L)]
    for l in range(L):
        ps[l].prepare_width(widths[l])

    def epoch():
        for l in range(L - 1, -1, -1):
            k = L - l - 1
            epp.epp_weight_gradient(paths, k, Ys[l], Gs[l + 1], Wgs[l], wss[l])
            epp.epp_input_gradient(paths, k, Gs[l + 1], Ws[l], Ygs[l])
            epp.epp_backward_aggregate(ps[l], Ygs[l], Gs[l])

    epoch()
    torch.cuda.synchronize()
    eager_w = [w.clone() for w in Wgs]
    eager_g0 = Gs[0].clone()
    # oracle chain on all vertices
    Go = G_top
    for l in range(L - 1, -1, -1):
        want_w, scale_w = oracle.weight_gradient(Ys[l].cpu().numpy(), Go)
        _close(eager_w[l].cpu().numpy(), want_w, scale_w, f"eager W' l={l}")
        yg, _ = oracle.input_gradient(Go, Ws[l].cpu().numpy())
        Go = oracle.full_aggregate(g.n, g.rowptr, g.col, g.val, yg)
    assert np.allclose(eager_g0.cpu().numpy(), Go, rtol=1e-4, atol=1e-5)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        epoch()
    for rep in range(3):
        for w in Wgs:
            w.fill_(float(rep + 1))          # eager work between replays
        for ws in wss:
            ws.fill_(255)                    # stale partial sums must not leak
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            assert torch.equal(Wgs[l], eager_w[l]), f"replay {rep} W' l={l}"
        assert torch.equal(Gs[0], eager_g0), f"replay {rep} gradient"
