"""Measurement studies around the hot path (they need a GPU):

    python -m paper_2204_02662_amd.studies gs    --config 4          # group-size sweep per layer (Sec. 5, Fig. 4 analogue)
    python -m paper_2204_02662_amd.studies depth --config 4 --F 64   # L = 2..6 (multi-layer study, Fig. 10 analogue)
    python -m paper_2204_02662_amd.studies combine --config 5        # combination stage on active rows vs all rows

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("study", choices=["gs", "depth", "combine"])
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--F", type=int, default=64)
    ap.add_argument("--Ls", type=str, default="2,3,4,5,6")
    args = ap.parse_args()
    import torch

    assert torch.cuda.is_available(), "the studies need a GPU"
    torch.cuda.set_device(0)
    {"gs": gs_study, "depth": depth_study, "combine": combine_study}[args.study](args)


if __name__ == "__main__":
    main()
