"""GPU parity at the full benchmark sizes (configurations 3-5), in the launch configuration
the benchmark times (the library's own group-size selection).

Paths and active sets are compared bit for bit on every element.  Gradients are compared
with the oracle on a strided sample of path rows (every entry of those rows), and on all
rows through properties that hold at any size: Theorem 1 (partially-active result ==
all-active result, rows outside N^{L-l} untouched / zero), the NaN-poison test, and the
column-sum identity evaluated in fp64.
"""
import numpy as np
import pytest
import torch

import graphgen
import oracle

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(not torch.cuda.is_available(), reason="needs a GPU")]

if torch.cuda.is_available():
    import paper_2204_02662_amd as epp
    from _util import ATOL, RTOL, assert_close, assert_paths_bit_exact, dev, gpu_prepare, gpu_prepare_full

SAMPLE_STRIDE = {3: 16, 4: 64, 5: 128}


@pytest.mark.timeout(900)
@pytest.mark.parametrize("k", [3, 4, 5])
def test_large_config(k):
    print(f"[cfg {k}] generating", flush=True)
    cfg = graphgen.make_config(k)
    g, L = cfg.graph, cfg.L
    print(f"[cfg {k}] oracle paths", flush=True)
    sets_o, paths_o = oracle.prepare(g.n, g.rowptr, g.col, g.val, cfg.train_ids, L)
    print(f"[cfg {k}] gpu prepare", flush=True)
    paths = gpu_prepare(g, cfg.train_ids, L)
    assert_paths_bit_exact(paths, sets_o, paths_o, L)
    full = gpu_prepare_full(g)
    colsum = np.zeros(g.n, np.float64)
    np.add.at(colsum, g.col, g.val.astype(np.float64))
    stride = SAMPLE_STRIDE[k]
    for l in range(L - 1, -1, -1):
        F = cfg.widths[l]
        rows, src = sets_o[L - l].astype(bool), sets_o[L - l - 1]
        print(f"[cfg {k}] layer {l} F={F} rows={int(rows.sum())} nnz={paths_o[l].col.size}", flush=True)
        X = graphgen.layer_gradient(cfg, l, src)
        gin = torch.from_numpy(X).to(dev())
        gout = torch.full_like(gin, 123.0)
        epp.epp_backward_aggregate(paths.path(l), gin, gout)
        torch.cuda.synchronize()
        got = gout.cpu().numpy()
        # rows outside the path untouched
        assert np.all(got[~rows] == 123.0)
        # sampled rows against the oracle, every entry
        po = paths_o[l]
        want = oracle.path_aggregate(g.n, po, X, first=l % stride, stride=stride)
        sample = po.row_ids[l % stride::stride]
        assert_close(got[sample], want[sample], f"cfg {k} layer {l} sampled rows")
        # column-sum identity over all rows in fp64
        got[~rows] = 0.0
        lhs = got.astype(np.float64).sum(0)
        rhs = colsum @ X.astype(np.float64)
        scale = np.abs(colsum) @ np.abs(X.astype(np.float64))
        assert np.all(np.abs(lhs - rhs) <= 1e-6 * scale + 1e-6), f"cfg {k} layer {l} column sums"
        # Theorem 1 on every row: all-active kernel == partially-active kernel
        gfull = torch.full_like(gin, 55.0)
        epp.epp_full_aggregate(full, gin, gfull)
        torch.cuda.synchronize()
        full_np = gfull.cpu().numpy()
        assert not full_np[~rows].any()
        for a in range(0, g.n, 1 << 18):  # chunked to bound host memory
            fa, ga = full_np[a:a + (1 << 18)].astype(np.float64), got[a:a + (1 << 18)]
            assert np.all(np.abs(fa - ga) <= 2 * ATOL + 2 * RTOL * np.abs(ga)), \
                f"cfg {k} layer {l} partial vs all-active"
        assert_close(full_np[sample], want[sample], f"cfg {k} layer {l} all-active sampled rows")
        del gfull, full_np
        # NaN poison outside the source set leaves the partial result unchanged
        gin[torch.from_numpy(src == 0).to(dev())] = float("nan")
        gout2 = torch.zeros_like(gin)
        epp.epp_backward_aggregate(paths.path(l), gin, gout2)
        torch.cuda.synchronize()
        got2 = gout2.cpu().numpy()
        assert np.isfinite(got2).all()
        assert_close(got2[sample], want[sample], f"cfg {k} layer {l} nan-poison")
        # if-else selective scheduling baseline on the NaN-poisoned input: same rows, same values
        gout3 = torch.full_like(gin, 77.0)
        epp.epp_ifelse_aggregate(full, paths, l, gin, gout3)
        torch.cuda.synchronize()
        got3 = gout3.cpu().numpy()
        assert np.all(got3[~rows] == 77.0)
        assert_close(got3[sample], want[sample], f"cfg {k} layer {l} if-else")
        del gin, gout, gout2, gout3, got, got2, got3, X
