"""Measurement studies around the hot path (they need a GPU unless noted):

    python -m paper_2204_02662_amd.studies gs    --config 4          # group-size sweep per layer (Sec. 5, Fig. 4 analogue)
    python -m paper_2204_02662_amd.studies depth --config 4 --F 64   # L = 2..6 (multi-layer study, Fig. 10 analogue)
    python -m paper_2204_02662_amd.studies combine --config 5        # combination stage on active rows vs all rows
    python -m paper_2204_02662_amd.studies overlap --config 5        # path preparing hidden behind the forward pass
    python -m paper_2204_02662_amd.studies gsfit                      # regression for the group size re-fitted on a
                                                                      # generated corpus (Sec. 5's method on wave64)
    python -m paper_2204_02662_amd.studies l2model --config 5 --F 128 # expected L2 hit rate of the gathers from the
                                                                      # graph's reference counts (no GPU needed)

Both print one JSON object per measurement.  Synthetic inputs only (graphgen).
"""
from __future__ import annotations

import argparse
import json
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def _time_ms(fn, reps=7):
    import numpy as np
    import torch

    fn()
    fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in ev]))


def _inputs(paths, n, F, k, dev, seed):
    import torch

    src = paths.active_set(k).long()
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    x = torch.zeros(n, F, dtype=torch.float32, device=dev)
    x[src] = torch.randn(src.numel(), F, generator=gen, dtype=torch.float32, device=dev)
    return x, torch.zeros_like(x)


def gs_study(args):
    import torch

    import graphgen
    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    cfg = graphgen.make_config(args.config)
    g, L = cfg.graph, cfg.L
    rowptr, col, val = (torch.from_numpy(a).to(dev) for a in (g.rowptr, g.col, g.val))
    paths = epp.epp_prepare(g.n, rowptr, col, val, torch.from_numpy(cfg.train_ids).to(dev), L)
    for l in range(L - 1, -1, -1):
        F = cfg.widths[l]
        p = paths.path(l)
        x, y = _inputs(paths, g.n, F, L - l - 1, dev, cfg.seed(10 + l))
        info = p.info()
        chosen = p.select_group_size(F)
        # Sec. 5's regression, applied to the sub-graph (entries / 2 as its undirected edge count)
        paper = epp.epp_paper_linreg_group_size(max(info.n_rows, 1), info.nnz // 2)
        sweep = sorted(set([2 ** i for i in range(3, 14)] + [chosen, paper]))
        best = None
        for gs in sweep:
            p.set_group_size(F, gs)
            ms = _time_ms(lambda: epp.epp_backward_aggregate(p, x, y))
            i2 = p.info()
            rec = {"study": "gs", "workload": cfg.name, "l": l, "F": F, "rows": info.n_rows, "nnz": info.nnz,
                   "mean_len": info.nnz / max(info.n_rows, 1), "gs": gs, "ms": ms, "groups": i2.n_groups,
                   "cut_rows": i2.n_split_rows, "selector": gs == chosen, "paper_linreg": gs == paper}
            print(json.dumps(rec), flush=True)
            if best is None or ms < best[1]:
                best = (gs, ms)
        p.set_group_size(F, 0)
        ms_sel = _time_ms(lambda: epp.epp_backward_aggregate(p, x, y))
        print(json.dumps({"study": "gs-summary", "workload": cfg.name, "l": l, "F": F, "best_gs": best[0],
                          "best_ms": best[1], "selector_gs": chosen, "selector_ms": ms_sel,
                          "selector_over_best": ms_sel / best[1], "paper_linreg_gs": paper}), flush=True)
        del x, y


def depth_study(args):
    import torch

    import graphgen
    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    cfg = graphgen.make_config(args.config)
    g = cfg.graph
    F = args.F
    rowptr, col, val = (torch.from_numpy(a).to(dev) for a in (g.rowptr, g.col, g.val))
    train = torch.from_numpy(cfg.train_ids).to(dev)
    full = epp.epp_prepare_full(g.n, rowptr, col, val)
    csr_bytes = 8.0 * g.nnz + 4.0 * (g.n + 1)
    for L in [int(x) for x in args.Ls.split(",")]:
        paths = epp.epp_prepare(g.n, rowptr, col, val, train, L)
        part, allact, layers = 0.0, 0.0, []
        for l in range(L - 1, -1, -1):
            p = paths.path(l)
            x, y = _inputs(paths, g.n, F, L - l - 1, dev, cfg.seed(10 + l))
            p.prepare_width(F)
            full.prepare_width(F)
            a = _time_ms(lambda: epp.epp_backward_aggregate(p, x, y), reps=5)
            b = _time_ms(lambda: epp.epp_full_aggregate(full, x, y), reps=5)
            i = p.info()
            layers.append({"l": l, "rows": i.n_rows, "nnz": i.nnz, "partial_ms": a, "all_active_ms": b})
            part += a
            allact += b
            del x, y
        pbytes = sum({paths.path(l)._h: paths.path(l).info().bytes for l in range(L)}.values())  # shared paths once
        print(json.dumps({"study": "depth", "workload": cfg.name, "F": F, "L": L, "partial_ms_per_epoch": part,
                          "all_active_ms_per_epoch": allact, "speedup": allact / part,
                          "path_bytes_over_csr_bytes": pbytes / csr_bytes,
                          "path_bytes_over_csr_plus_gradients": pbytes / (csr_bytes + 2.0 * 4 * F * g.n * L),
                          "layers": layers}), flush=True)
        del paths


def combine_study(args):
    """Combination lines of Alg. 1's backward loop for every layer of a configuration: restricted
    to N^{L-l-1} (this library), over all rows (this library, k = -1) and over all rows with the
    vendor GEMM (torch.matmul).  Widths: W(l) is F_l x F_{l+1}, with F_L set to F_{L-1}."""
    import torch

    import graphgen
    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    cfg = graphgen.make_config(args.config)
    g, L = cfg.graph, cfg.L
    rowptr, col, val = (torch.from_numpy(a).to(dev) for a in (g.rowptr, g.col, g.val))
    paths = epp.epp_prepare(g.n, rowptr, col, val, torch.from_numpy(cfg.train_ids).to(dev), L)
    widths = list(cfg.widths) + [cfg.widths[L - 1]]
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed(30))
    for l in range(L - 1, -1, -1):
        k = L - l - 1
        Fi, Fo = widths[l], widths[l + 1]
        rows = paths.active_set(k).long()
        Y = torch.randn(g.n, Fi, generator=gen, device=dev)
        W = torch.randn(Fi, Fo, generator=gen, device=dev)
        G = torch.zeros(g.n, Fo, device=dev)
        G[rows] = torch.randn(rows.numel(), Fo, generator=gen, device=dev)
        Wg, Yg = torch.empty(Fi, Fo, device=dev), torch.zeros(g.n, Fi, device=dev)
        ws = torch.empty(max(epp.epp_weight_gradient_workspace(paths, k, Fi, Fo),
                             epp.epp_weight_gradient_workspace(paths, -1, Fi, Fo)), dtype=torch.uint8, device=dev)
        R = rows.numel()
        rec = {"study": "combine", "workload": cfg.name, "l": l, "k": k, "F_in": Fi, "F_out": Fo, "n": g.n,
               "active_rows": R}
        for name, kk in (("active", k), ("all_rows", -1)):
            rec[f"weight_grad_{name}_ms"] = _time_ms(lambda: epp.epp_weight_gradient(paths, kk, Y, G, Wg, ws))
            rec[f"input_grad_{name}_ms"] = _time_ms(lambda: epp.epp_input_gradient(paths, kk, G, W, Yg))
        rec["weight_grad_vendor_gemm_ms"] = _time_ms(lambda: torch.matmul(Y.t(), G, out=Wg))
        rec["input_grad_vendor_gemm_ms"] = _time_ms(lambda: torch.matmul(G, W.t(), out=Yg))
        # algorithmic bytes (each operand row once) and flops of the restricted products
        by = 4.0 * R * (Fi + Fo) + 4.0 * Fi * Fo
        fl = 2.0 * R * Fi * Fo
        for op in ("weight_grad", "input_grad"):
            ms = rec[f"{op}_active_ms"]
            rec[f"{op}_active_GBs"] = by / ms / 1e6
            rec[f"{op}_active_TFLOPs"] = fl / ms / 1e9
            rec[f"{op}_active_hbm_frac"] = by / ms / 1e6 / 8000.0
            rec[f"{op}_active_mfma_frac"] = fl / ms / 1e9 / 157.3
        print(json.dumps(rec), flush=True)
        del Y, W, G, Wg, Yg, ws


def shape_study(args):
    """The two combination kernels on `--rows` contiguous rows (k = -1: every vertex, no id
    list) of width `--F` x `--Fo`: the plain matrix-core shape, for counter runs."""
    import torch

    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    n, Fi, Fo = args.rows, args.F, args.Fo
    rowptr = torch.zeros(n + 1, dtype=torch.int32, device=dev)
    none_i, none_f = torch.zeros(0, dtype=torch.int32, device=dev), torch.zeros(0, device=dev)
    paths = epp.epp_prepare(n, rowptr, none_i, none_f, torch.zeros(1, dtype=torch.int32, device=dev), 1)
    Y, G, W = (torch.randn(a, b, device=dev) for a, b in ((n, Fi), (n, Fo), (Fi, Fo)))
    Wg, Yg = torch.empty(Fi, Fo, device=dev), torch.empty(n, Fi, device=dev)
    ws = torch.empty(epp.epp_weight_gradient_workspace(paths, -1, Fi, Fo), dtype=torch.uint8, device=dev)
    w_ms = _time_ms(lambda: epp.epp_weight_gradient(paths, -1, Y, G, Wg, ws))
    y_ms = _time_ms(lambda: epp.epp_input_gradient(paths, -1, G, W, Yg))
    fl = 2.0 * n * Fi * Fo
    print(json.dumps({"study": "shape", "rows": n, "F_in": Fi, "F_out": Fo, "weight_grad_ms": w_ms, "input_grad_ms": y_ms,
                      "weight_grad_TFLOPs": fl / w_ms / 1e9, "input_grad_TFLOPs": fl / y_ms / 1e9}), flush=True)


def overlap_study(args):
    """On-the-fly preparation (the paper's last experiment): epp_prepare on a second stream while
    the first forward pass (all-active aggregations of every layer, this build's own kernel) runs
    on the main stream.  Reports both alone, back to back, and overlapped."""
    import time

    import torch

    import graphgen
    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    cfg = graphgen.make_config(args.config)
    g, L = cfg.graph, cfg.L
    rowptr, col, val = (torch.from_numpy(a).to(dev) for a in (g.rowptr, g.col, g.val))
    train = torch.from_numpy(cfg.train_ids).to(dev)
    full = epp.epp_prepare_full(g.n, rowptr, col, val)
    xs = [torch.randn(g.n, cfg.widths[l], device=dev) for l in range(L)]
    ys = [torch.empty_like(x) for x in xs]

    def forward():
        for l in range(L):
            epp.epp_full_aggregate(full, xs[l], ys[l])

    def wall(fn, reps=5):
        out = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t) * 1e3)
        return sorted(out)[len(out) // 2]

    for l in range(L):
        full.prepare_width(cfg.widths[l])  # schedules of the all-active graph
    forward()
    side = torch.cuda.Stream()

    def prepare_only():
        epp.epp_prepare(g.n, rowptr, col, val, train, L)

    def overlapped():
        forward()                      # enqueued on the main stream, returns at once
        with torch.cuda.stream(side):  # prepare runs (and waits) on its own stream
            epp.epp_prepare(g.n, rowptr, col, val, train, L)

    f_ms, p_ms = wall(forward), wall(prepare_only)
    both_ms = wall(overlapped)
    print(json.dumps({"study": "overlap", "workload": cfg.name, "forward_all_active_ms": f_ms, "prepare_ms": p_ms,
                      "back_to_back_ms": f_ms + p_ms, "overlapped_ms": both_ms,
                      "prepare_cost_hidden": 1.0 - max(both_ms - f_ms, 0.0) / p_ms}), flush=True)


def gsfit_study(args):
    """Sec. 5's learning-based selection redone for this kernel: generate a corpus of power-law
    graphs (R-MAT and Chung-Lu, as the paper's corpus came from a generator), label every
    execution path and width with the best group size of an exhaustive power-of-two sweep (the
    paper's labelling method), fit a linear regression on structural features, and compare the
    loss over the best group size of (a) that regression, leave-one-graph-out, (b) the library's
    closed-form selector, (c) the paper's printed regression applied to the sub-graph."""
    import numpy as np
    import torch

    import graphgen
    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    sweep = [2 ** i for i in range(3, 13)]
    corpus = [(kind, 1 << ln, deg, frac) for kind in ("rmat", "chung_lu") for ln in args.log2n
              for deg in (4, 16, 64) for frac in (0.01, 0.1)]
    samples = []
    for gi, (kind, n, deg, frac) in enumerate(corpus):
        edges = n * deg // 2
        try:
            g = (graphgen.random_graph("rmat", n, seed=7000 + gi, raw_draws=edges) if kind == "rmat"
                 else graphgen.random_graph("chung_lu", n, seed=7000 + gi, target_edges=edges))
        except RuntimeError:
            continue  # the generator cannot reach this many distinct pairs
        train = graphgen.training_set(g.n, max(1, int(frac * n)), 7100 + gi)
        rowptr, col, val = (torch.from_numpy(a).to(dev) for a in (g.rowptr, g.col, g.val))
        L = 2
        paths = epp.epp_prepare(g.n, rowptr, col, val, torch.from_numpy(train).to(dev), L)
        for l in range(L):
            p = paths.path(l)
            info = p.info()
            if info.nnz == 0:
                continue
            for F in args.widths:
                x, y = _inputs(paths, g.n, F, L - l - 1, dev, 7200 + gi)
                times = {}
                for gs in sweep:
                    p.set_group_size(F, gs)
                    times[gs] = _time_ms(lambda: epp.epp_backward_aggregate(p, x, y), reps=5)
                p.set_group_size(F, 0)
                chosen = p.select_group_size(F)
                rec = {"study": "gsfit-sample", "graph": gi, "kind": kind, "n": n, "deg": deg, "train_frac": frac,
                       "l": l, "F": F, "rows": info.n_rows, "nnz": info.nnz, "max_len": info.max_len,
                       "len_hist": info.len_hist, "times_ms": times, "best_gs": min(times, key=times.get), "selector_gs": chosen,
                       "paper_linreg_gs": epp.epp_paper_linreg_group_size(max(info.n_rows, 1), info.nnz // 2)}
                samples.append(rec)
                print(json.dumps(rec), flush=True)
                del x, y
        del paths, rowptr, col, val

    def feats(r):
        return [np.log2(r["nnz"]), np.log2(r["nnz"] / r["rows"]), np.log2(r["F"]), 1.0]

    def loss(r, gs):  # time at the nearest swept group size over the best time
        near = min(sweep, key=lambda s_: abs(np.log2(s_) - np.log2(max(gs, 1))))
        return r["times_ms"][near] / r["times_ms"][r["best_gs"]]

    X = np.array([feats(r) for r in samples])
    yv = np.array([np.log2(r["best_gs"]) for r in samples])
    beta_all, *_ = np.linalg.lstsq(X, yv, rcond=None)
    graphs = sorted({r["graph"] for r in samples})
    loo = []
    for gi in graphs:  # leave one graph out
        tr = np.array([r["graph"] != gi for r in samples])
        b, *_ = np.linalg.lstsq(X[tr], yv[tr], rcond=None)
        loo += [loss(r, 2.0 ** float(np.dot(b, feats(r)))) for r in samples if r["graph"] == gi]
    sel = [loss(r, r["selector_gs"]) for r in samples]
    pap = [loss(r, r["paper_linreg_gs"]) for r in samples]

    def stats(v):
        v = np.array(v)
        return {"mean": float(v.mean()), "median": float(np.median(v)), "p90": float(np.quantile(v, 0.9)),
                "max": float(v.max())}

    print(json.dumps({"study": "gsfit-summary", "samples": len(samples), "graphs": len(graphs),
                      "features": ["log2 nnz", "log2 mean row length", "log2 F", "1"],
                      "beta_log2_gs": [float(b) for b in beta_all],
                      "r2": float(1 - ((X @ beta_all - yv) ** 2).sum() / ((yv - yv.mean()) ** 2).sum()),
                      "time_over_best": {"fitted_regression_leave_one_graph_out": stats(loo),
                                         "library_selector": stats(sel), "paper_regression_on_subgraph": stats(pap)}}),
          flush=True)


def lru_hit_rate_irm(counts, rows: int) -> float:
    """Hit rate of an LRU cache of `rows` places when item i is referenced with probability
    proportional to counts[i], independently of the past (Che's approximation)."""
    import numpy as np

    c = np.asarray(counts, np.float64)
    c = c[c > 0]
    if rows >= c.size:
        return 1.0
    resident = lambda t: (1.0 - np.exp(-c * t)).sum()
    lo, hi = 0.0, 1.0 / c.max()
    while resident(hi) < rows:
        hi *= 2
    for _ in range(100):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if resident(mid) < rows else (lo, mid)
    t = 0.5 * (lo + hi)
    return float((c * (1.0 - np.exp(-c * t))).sum() / c.sum())


def l2model_study(args):
    """What hit rate can one XCD's 4 MB L2 reach on the source rows of a graph?  From the reference
    counts alone (CPU only): the share of the references that goes to the C most referenced rows (a
    cache that held exactly those), and the hit rate of an LRU cache of C rows under the
    independent-reference model (Che's approximation: a row referenced with rate p hits with
    probability 1 - exp(-p T), where T makes the expected number of resident rows equal C), with
    all sources competing for the cache and with only the unstreamed ones (the hot/cold budget)."""
    import numpy as np

    import graphgen

    g = graphgen.make_config(args.config).graph
    cnt = np.sort(np.bincount(g.col, minlength=g.n).astype(np.float64))[::-1]
    nnz = cnt.sum()

    def lru_hit_rate(c, rows):  # (as a share of ALL references: streamed sources never hit)
        return lru_hit_rate_irm(c, rows) * float(c.sum() / nnz)

    row_bytes = 4 * args.F
    unstreamed = cnt[:(96 << 20) // row_bytes]
    for slices in (1, 2):
        rows = (4 << 20) * slices // row_bytes
        print(json.dumps({"config": args.config, "F": args.F, "xcd_feature_slices": slices, "rows_one_l2_holds": rows,
                          "share_of_references_to_that_many_top_rows": float(cnt[:rows].sum() / nnz),
                          "lru_hit_rate_all_sources_compete": lru_hit_rate(cnt, rows),
                          "lru_hit_rate_only_unstreamed_sources_compete": lru_hit_rate(unstreamed, rows)}), flush=True)
    part_rows = 8 * (3584 << 10) // row_bytes
    print(json.dumps({"config": args.config, "F": args.F, "rows_eight_l2s_hold_together": part_rows,
                      "share_of_references_to_that_many_top_rows": float(cnt[:part_rows].sum() / nnz)}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("study", choices=["gs", "depth", "combine", "gsfit", "overlap", "shape", "l2model"])
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--F", type=int, default=64)
    ap.add_argument("--Fo", type=int, default=128)
    ap.add_argument("--rows", type=int, default=4_600_000)
    ap.add_argument("--Ls", type=str, default="2,3,4,5,6")
    ap.add_argument("--log2n", type=lambda v: [int(x) for x in v.split(",")], default=[13, 15, 17, 19])
    ap.add_argument("--widths", type=lambda v: [int(x) for x in v.split(",")], default=[16, 64, 128])
    args = ap.parse_args()
    if args.study == "l2model":
        return l2model_study(args)
    import torch

    assert torch.cuda.is_available(), "the studies need a GPU"
    torch.cuda.set_device(0)
    {"gs": gs_study, "depth": depth_study, "combine": combine_study, "gsfit": gsfit_study,
     "overlap": overlap_study, "shape": shape_study}[args.study](args)


if __name__ == "__main__":
    main()
