#!/usr/bin/env python3
"""Backward-aggregation benchmark on one MI355X.

A "step" is one epoch of backward aggregation: one launch of the partially-active kernel
per layer, l = L-1 ... 0 (Alg. 2), over synthetic inputs that are already resident in HBM.
Prints ONE JSON line: metric/value/unit (ms per epoch of the partially-active path on the
headline workload), per-layer times with algorithmic bytes and roofline fractions, the
dominant kernel's `roofline` object, the all-active and if-else comparisons, the one-off
`prepare_ms`, the other benchmark configurations in compact form (`configs`), and
`cpu_baseline` (the CPU oracle timed on this machine's host cores).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--only] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# the chip's own random-row gather rates (profiles/gather_rate_microbenchmark.md): lines of 128 bytes per
# second served by an XCD's L2 / from beyond it (memory-side cache or HBM alike)
GATHER_L2_LINES_PER_S = 235e9
GATHER_MISS_LINES_PER_S = 60e9


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def algorithmic_bytes(R: int, S: int, nnz: int, F: int) -> int:
    """Compulsory HBM bytes of one layer launch: the path's index arrays once (row ids,
    row pointer, column ids, weights), every distinct source row once, every output row once."""
    return 4 * (2 * R + 1) + 8 * nnz + 4 * F * S + 4 * F * R


def edge_bytes(R: int, nnz: int, F: int) -> int:
    """Bytes issued if no gathered row were ever reused: (8 + 4F) per entry + output."""
    return 4 * (2 * R + 1) + 8 * nnz + 4 * F * nnz + 4 * F * R


def kernel_source_hash() -> str:
    """Hash of the HIP sources the library is built from: counter summaries are stamped with it."""
    from paper_2204_02662_amd import build as _build
    return _build.source_hash()


def read_traffic(workload: str):
    """(HBM bytes per launch, L2 hit rate) of the aggregation kernel per layer, from the committed rocprofv3
    counter summary profiles/hbm_traffic.txt (lines `<workload> <layer> <fetch_bytes> <write_bytes> <l2 hit rate>`
    after a line `sources <hash>`).  The counters describe the kernels they were measured on: if the sources
    have changed since, nothing is returned (and the bench line carries traffic = null)."""
    f = ROOT / "profiles" / "hbm_traffic.txt"
    out, stamp = {}, None
    if f.exists():
        for line in f.read_text().splitlines():
            parts = line.split()
            if len(parts) == 2 and parts[0] == "sources":
                stamp = parts[1]
            elif len(parts) >= 4 and parts[0] == workload:
                out[int(parts[1])] = (float(parts[2]) + float(parts[3]), float(parts[4]) if len(parts) > 4 else None)
    if out and stamp != kernel_source_hash():
        log(f"profiles/hbm_traffic.txt was measured on sources {stamp}, the library is built from "
            f"{kernel_source_hash()}: counter-based fields (traffic, L2 hit rate) are reported as null")
        return {}
    return out


def cpu_baseline(cfg, budget_s: float):
    """The CPU oracle, as it stands, timed on this machine's host cores on a strided sample of
    path rows of every layer; scaled to a whole epoch by the share of entries sampled."""
    import numpy as np

    import graphgen
    import oracle

    g, L = cfg.graph, cfg.L
    threads = oracle.max_threads()
    log(f"cpu_baseline: oracle path preparing on {threads} threads")
    sets_o, paths_o = oracle.prepare(g.n, g.rowptr, g.col, g.val, cfg.train_ids, L)
    work = [paths_o[l].col.size * cfg.widths[l] for l in range(L)]
    total_work = float(sum(work))
    est_ms, sampled_s, strides = 0.0, 0.0, []
    est1_ms, sampled1_s, strides1 = 0.0, 0.0, []
    for l in range(L - 1, -1, -1):
        po, F = paths_o[l], cfg.widths[l]
        X = graphgen.layer_gradient(cfg, l, sets_o[L - l - 1])
        R = po.row_ids.size
        if R == 0:
            strides.append(1)
            continue
        # size the sample to this layer's share of the budget: start thin, then widen from
        # the measured rate until the run is long enough (cold caches make thin samples slow)
        lens = np.diff(po.rowptr)
        share = budget_s * work[l] / total_work
        stride = max(1, R // 2000)
        while True:
            t = time.perf_counter()
            oracle.path_aggregate(g.n, po, X, first=0, stride=stride)
            dt = max(time.perf_counter() - t, 1e-4)
            frac = lens[0::stride].sum() / max(po.col.size, 1)
            if stride == 1 or dt >= 0.5 * share:
                break
            stride = max(1, min(stride - 1, int(stride * dt / share)))
        est_ms += dt / max(frac, 1e-12) * 1e3
        sampled_s += dt
        strides.append(stride)
        # the same on one thread, on a sample thinned by the thread count (about the same wall time)
        stride1 = stride * threads
        if threads > 1 and R >= 64 * stride1:
            oracle.set_threads(1)
            t = time.perf_counter()
            oracle.path_aggregate(g.n, po, X, first=0, stride=stride1)
            dt1 = max(time.perf_counter() - t, 1e-4)
            oracle.set_threads(threads)
            est1_ms += dt1 / max(lens[0::stride1].sum() / max(po.col.size, 1), 1e-12) * 1e3
            sampled1_s += dt1
            strides1.append(stride1)
        else:
            est1_ms = float("nan")
        del X
    out = {
        "value": est_ms, "unit": "ms/epoch", "cores": threads, "kind": "oracle",
        "sample": (f"every k-th path row of each layer (k={strides} for l=L-1..0), all widths; "
                   f"{sampled_s:.1f} s of CPU work scaled by the share of entries sampled"),
    }
    if est1_ms == est1_ms and strides1:  # not NaN: every layer was large enough to thin
        out["one_thread"] = {"value": est1_ms, "unit": "ms/epoch", "cores": 1,
                             "sample": f"every k-th path row (k={strides1}); {sampled1_s:.1f} s of CPU work, scaled"}
    return out


def run_config(config_id: int, args, detail: bool):
    """One benchmark configuration: generate, prepare, time the partially-active epoch, the all-active
    and if-else baselines.  `detail` adds what only the headline workload reports (combination stage,
    flushed caches, per-epoch clearing of the output, counters).  Returns (result dict, cfg)."""
    import numpy as np
    import torch

    import graphgen
    import paper_2204_02662_amd as epp

    dev = torch.device("cuda", 0)
    t0 = time.perf_counter()
    cfg = graphgen.make_config(config_id)
    g, L = cfg.graph, cfg.L
    log(f"{cfg.name}: n={g.n} nnz={g.nnz} L={L} widths(l=0..)={cfg.widths} |V_t|={cfg.n_train} "
        f"generated in {time.perf_counter() - t0:.1f}s")

    rowptr, col, val = (torch.from_numpy(a).to(dev) for a in (g.rowptr, g.col, g.val))
    train = torch.from_numpy(cfg.train_ids).to(dev)
    # one pass over a 64-vertex graph with the same widths first: the HIP runtime loads every kernel's code
    # on its first launch in a process, which is not part of preparing this workload's paths
    tiny = graphgen.random_graph("chung_lu", 64, seed=1, target_edges=128)
    t_rowptr, t_col, t_val = (torch.from_numpy(a).to(dev) for a in (tiny.rowptr, tiny.col, tiny.val))
    os.environ["EPP_TUNE_SMALL_PREPARE"] = "0"  # (once through the general construction, then through the single-launch one)
    t_paths = epp.epp_prepare(tiny.n, t_rowptr, t_col, t_val, torch.arange(8, dtype=torch.int32, device=dev), L)
    del os.environ["EPP_TUNE_SMALL_PREPARE"]
    t_paths = epp.epp_prepare(tiny.n, t_rowptr, t_col, t_val, torch.arange(8, dtype=torch.int32, device=dev), L)
    for l in range(L):
        t_x = torch.zeros(tiny.n, cfg.widths[l], device=dev)
        t_paths.path(l).prepare_width(cfg.widths[l])
        epp.epp_backward_aggregate(t_paths.path(l), t_x, torch.zeros_like(t_x))
    del t_paths, t_rowptr, t_col, t_val, t_x
    # Preparation is timed twice: the first call makes PyTorch's caching allocator fetch the handle's memory
    # from the driver (hipMalloc, hundreds of microseconds per segment), the second finds it cached, as a
    # training process that has been running does.  `prepare_ms` is the second, `prepare_first_call_ms` the first.
    prepare_calls = []
    paths = None
    for _ in range(2):
        del paths
        torch.cuda.synchronize()
        t = time.perf_counter()
        paths = epp.epp_prepare(g.n, rowptr, col, val, train, L)
        torch.cuda.synchronize()
        prepare_calls.append((time.perf_counter() - t) * 1e3)
    prepare_ms = prepare_calls[1]
    full = None if args.no_all_active else epp.epp_prepare_full(g.n, rowptr, col, val)

    # inputs resident in HBM: N(0,1) on the source rows of each layer, zeros elsewhere
    gen = torch.Generator(device=dev)
    grad_in, grad_out, infos = [], [], []
    for l in range(L):
        F = cfg.widths[l]
        src = paths.active_set(L - l - 1).long()
        x = torch.zeros(g.n, F, dtype=torch.float32, device=dev)
        gen.manual_seed(cfg.seed(10 + l))
        x[src] = torch.randn(src.numel(), F, generator=gen, dtype=torch.float32, device=dev)
        grad_in.append(x)
        grad_out.append(torch.zeros(g.n, F, dtype=torch.float32, device=dev))
    del rowptr, col, val

    order = [l for l in range(L - 1, -1, -1) if not args.layers or str(l) in args.layers.split(",")]
    if args.calibrate_copy and detail:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        b.copy_(a)  # 1 GiB read + 1 GiB written by one elementwise kernel
        torch.cuda.synchronize()
        del a, b

    path_objs = [paths.path(l) for l in range(L)]

    def timed(run_layer, steps, warmup, between=None):
        """HIP events on the stream the kernels are launched on (PyTorch's current stream), one pair
        per layer launch; returns (wall ms per epoch, mean ms per layer) and leaves median/min in .spread."""
        for _ in range(warmup):
            for l in order:
                run_layer(l)
        torch.cuda.synchronize()
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in order]
              for _ in range(steps)]
        t = time.perf_counter()
        for s in range(steps):
            for i, l in enumerate(order):
                if between is not None:
                    between(l)  # outside the event pair
                ev[s][i][0].record()
                run_layer(l)
                ev[s][i][1].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t) * 1e3 / steps
        samples = {l: [ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(steps)] for i, l in enumerate(order)}
        per_layer = {l: float(np.mean(v)) for l, v in samples.items()}
        timed.spread = {l: (float(np.median(v)), float(np.min(v))) for l, v in samples.items()}
        return wall_ms, per_layer

    # one-off per (path, width): group table, partial rows, locality marks
    torch.cuda.synchronize()
    t = time.perf_counter()
    for l in order:
        path_objs[l].prepare_width(cfg.widths[l])
    torch.cuda.synchronize()
    schedule_ms = (time.perf_counter() - t) * 1e3

    run_partial = lambda l: epp.epp_backward_aggregate(path_objs[l], grad_in[l], grad_out[l])  # noqa: E731
    ms_partial, layer_ms = timed(run_partial, args.steps, args.warmup)
    layer_spread = timed.spread
    for l in range(L):
        infos.append(path_objs[l].info())

    layers = []
    for l in order:
        i, F = infos[l], cfg.widths[l]
        bmin, bedge = algorithmic_bytes(i.n_rows, i.n_src, i.nnz, F), edge_bytes(i.n_rows, i.nnz, F)
        ms = layer_ms[l]
        layers.append({
            "l": l, "F": F, "rows": i.n_rows, "sources": i.n_src, "nnz": i.nnz, "max_len": i.max_len,
            "group_size": i.group_size, "groups": i.n_groups, "split_rows": i.n_split_rows,
            # source-partitioned layout (zeros: not in use for this layer)
            "partitioned_rows": i.part_rows, "entries_in_xcd_sections": i.part_hot_entries,
            "partial_rows": i.part_partial_rows,
            # 1: the path keeps no entry arrays and runs on those of layer l - 1 (skipping that path's extra entries)
            "runs_on_entries_of_outer_path": i.shares_entries,
            "ms": ms, "ms_median": layer_spread[l][0], "ms_min": layer_spread[l][1], "algorithmic_bytes": bmin,
            "roofline_GBs": bmin / ms / 1e6 if ms > 0 else None,
            "roofline_frac": bmin / ms / 1e6 / HBM_PEAK_GBS if ms > 0 else None,
            "gather_GBs": bedge / ms / 1e6 if ms > 0 else None,
        })
    # the dominant launch: the layer with the most work (entries x width); by time the two widest layers of a
    # deep configuration are within a per cent of each other and would swap from run to run
    dom = max(layers, key=lambda d: (d["nnz"] * d["F"], d["ms"]))
    traffic, l2_hit = read_traffic(cfg.name).get(dom["l"], (None, None)) if detail else (None, None)
    lines = dom["nnz"] * ((dom["F"] * 4 + 127) // 128)
    model_ms = (lines * ((1.0 - l2_hit) / GATHER_MISS_LINES_PER_S + l2_hit / GATHER_L2_LINES_PER_S) * 1e3
                if l2_hit is not None else None)
    roofline = {
        "bound": "hbm", "kernel": f"k_aggregate (layer l={dom['l']}, F={dom['F']})",
        "achieved": dom["roofline_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": dom["roofline_frac"], "traffic": traffic,
        # the same launch by the counters: HBM-side bytes actually moved per second (rises when caching gets
        # worse; evidence, not an objective)
        "traffic_GBs": traffic / dom["ms"] / 1e6 if traffic else None,
        "traffic_frac_of_peak": traffic / dom["ms"] / 1e6 / HBM_PEAK_GBS if traffic else None,
        # time the gathered 128-byte lines alone would take at the measured gather rates of this chip
        "gather_rate_model": {"lines": lines, "l2_hit_rate": l2_hit, "model_ms": model_ms,
                              "measured_over_model": dom["ms"] / model_ms if model_ms else None},
    }

    result = {
        "config": {"workload": cfg.name, "n": g.n, "nnz": g.nnz, "undirected_edges": g.undirected_edges,
                   "L": L, "widths_l0_first": cfg.widths, "n_train": cfg.n_train,
                   "max_degree": int(np.diff(g.rowptr).max())},
        "roofline": roofline,
        "partially_active": {"ms_per_epoch": ms_partial, "sum_layer_ms": sum(layer_ms.values()), "layers": layers},
        "prepare_ms": prepare_ms,
        "prepare_first_call_ms": prepare_calls[0],
        "schedule_ms": schedule_ms,  # one-off epp_path_prepare_width of every layer
        # one-off path construction: two passes over the column ids, one over the kept weights,
        # the (col, val) pairs written once, row pointer read and filtered pointer written per level
        # (layers past the fixed point of the active sets are built once)
        "prepare_algorithmic_bytes": sum(8 * g.nnz + 12 * nz + 8 * (g.n + 1)
                                         for nz in {path_objs[l]._h: infos[l].nnz for l in range(L)}.values()),
        # layers past the fixed point of the active sets share one path object: count it once
        "path_bytes_over_csr_bytes": sum({path_objs[l]._h: infos[l].bytes for l in range(L)}.values())
        / (8.0 * g.nnz + 4.0 * (g.n + 1)),
    }

    if full is not None:
        for l in order:
            full.prepare_width(cfg.widths[l])
        k_full = max(3, args.steps // 4)
        ms_full, full_layer_ms = timed(lambda l: epp.epp_full_aggregate(full, grad_in[l], grad_out[l]), k_full,
                                       min(args.warmup, 2))
        fi = full.info()
        fl = []
        for l in order:
            F = cfg.widths[l]
            bmin = algorithmic_bytes(g.n, g.n, g.nnz, F)
            fl.append({"l": l, "F": F, "ms": full_layer_ms[l], "algorithmic_bytes": bmin,
                       "roofline_frac": bmin / full_layer_ms[l] / 1e6 / HBM_PEAK_GBS,
                       "group_size": fi.group_size if fi.sched_F == F else None})
        result["all_active"] = {"ms_per_epoch": ms_full, "steps": k_full, "layers": fl}
        result["speedup_partial_over_all_active"] = ms_full / ms_partial if ms_partial > 0 else None
        saved = ms_full - ms_partial
        result["break_even_epochs"] = (prepare_ms + result["schedule_ms"]) / saved if saved > 0 else None
        # if-else selective scheduling on the whole graph (the paper's straightforward alternative)
        ms_ie, ie_layer_ms = timed(lambda l: epp.epp_ifelse_aggregate(full, paths, l, grad_in[l], grad_out[l]), k_full,
                                   min(args.warmup, 2))
        result["if_else"] = {"ms_per_epoch": ms_ie, "steps": k_full,
                             "layers": [{"l": l, "F": cfg.widths[l], "ms": ie_layer_ms[l]} for l in order]}
        result["speedup_partial_over_if_else"] = ms_ie / ms_partial if ms_partial > 0 else None

    # combination stage of the backward loop on the active rows (reported beside the metric, never
    # part of it): W'(l) = Y(l)^T X'(l+1), Y'(l) = X'(l+1) W(l)^T with W(l) of F_l x F_{l+1}, F_L = F_{L-1}
    if detail and not args.no_combination and not args.layers:
        widths = list(cfg.widths) + [cfg.widths[L - 1]]
        comb = []
        for l in order:
            k, Fi, Fo = L - l - 1, widths[l], widths[l + 1]
            rows = paths.active_set(k).long()
            gen.manual_seed(cfg.seed(30 + l))
            Y = torch.randn(g.n, Fi, generator=gen, device=dev)
            W = torch.randn(Fi, Fo, generator=gen, device=dev)
            G = torch.zeros(g.n, Fo, device=dev)
            G[rows] = torch.randn(rows.numel(), Fo, generator=gen, device=dev)
            Wg = torch.empty(Fi, Fo, device=dev)
            ws = torch.empty(epp.epp_weight_gradient_workspace(paths, k, Fi, Fo), dtype=torch.uint8, device=dev)

            def ev_ms(fn, reps=5):
                fn()
                torch.cuda.synchronize()
                e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
                for a, b in e:
                    a.record()
                    fn()
                    b.record()
                torch.cuda.synchronize()
                return float(np.median([a.elapsed_time(b) for a, b in e]))

            R = rows.numel()
            w_ms = ev_ms(lambda: epp.epp_weight_gradient(paths, k, Y, G, Wg, ws))
            y_ms = ev_ms(lambda: epp.epp_input_gradient(paths, k, G, W, grad_out[l]))
            wv_ms = ev_ms(lambda: torch.matmul(Y.t(), G, out=Wg))
            yv_ms = ev_ms(lambda: torch.matmul(G, W.t(), out=grad_out[l]))
            grad_out[l].zero_()
            by, fl_ = 4.0 * R * (Fi + Fo) + 4.0 * Fi * Fo, 2.0 * R * Fi * Fo
            comb.append({"l": l, "k": k, "F_in": Fi, "F_out": Fo, "active_rows": R,
                         "weight_gradient_ms": w_ms, "input_gradient_ms": y_ms,
                         "vendor_gemm_all_rows_ms": {"weight_gradient": wv_ms, "input_gradient": yv_ms},
                         "algorithmic_bytes": by, "flops": fl_,
                         "weight_gradient_hbm_frac": by / w_ms / 1e6 / HBM_PEAK_GBS,
                         "weight_gradient_mfma_f32_frac": fl_ / w_ms / 1e9 / 157.3,
                         "input_gradient_hbm_frac": by / y_ms / 1e6 / HBM_PEAK_GBS,
                         "input_gradient_mfma_f32_frac": fl_ / y_ms / 1e9 / 157.3})
            del Y, W, G, Wg, ws
        result["combination_active_rows"] = {"dtype": "f32", "layers": comb}

    if detail and not args.layers:
        k_side = max(3, args.steps // 4)
        # training runs other kernels between two aggregations: the same epoch with the caches flushed
        # (1 GiB written) before every layer launch; the sum of the per-layer event times is reported
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        _, cold_layer_ms = timed(run_partial, k_side, 1, between=lambda l: scratch.fill_(1.0))
        result["partially_active"]["cold_cache_ms_per_epoch"] = sum(cold_layer_ms.values())
        del scratch

        # a caller that does not rely on "rows outside the path are never written" clears the whole
        # n x F output before every layer launch; the clearing is inside the timed region here
        def cleared(l):
            grad_out[l].zero_()
            run_partial(l)

        ms_cleared, _ = timed(cleared, k_side, 1)
        result["partially_active"]["ms_per_epoch_with_output_cleared_every_epoch"] = ms_cleared

    # launch-bound workloads: the same epoch captured once in a HIP graph and replayed
    if ms_partial < 1.0 and not args.layers:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for l in order:
                run_partial(l)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        result["partially_active"]["hip_graph_ms_per_epoch"] = (time.perf_counter() - t) * 1e3 / args.steps
        del graph
    del grad_in, grad_out, paths, full, path_objs
    torch.cuda.empty_cache()
    return result, cfg


def compact(r):
    """What the headline line keeps of a side configuration."""
    dom = max(r["partially_active"]["layers"], key=lambda d: (d["nnz"] * d["F"], d["ms"]))
    out = {
        "workload": r["config"]["workload"], "n": r["config"]["n"], "nnz": r["config"]["nnz"], "L": r["config"]["L"],
        "widths_l0_first": r["config"]["widths_l0_first"], "n_train": r["config"]["n_train"],
        "partial_ms_per_epoch": r["partially_active"]["ms_per_epoch"],
        "partial_layer_ms": {str(d["l"]): d["ms"] for d in r["partially_active"]["layers"]},
        "all_active_ms_per_epoch": r.get("all_active", {}).get("ms_per_epoch"),
        "if_else_ms_per_epoch": r.get("if_else", {}).get("ms_per_epoch"),
        "speedup_partial_over_all_active": r.get("speedup_partial_over_all_active"),
        "dominant_layer": {"l": dom["l"], "F": dom["F"], "ms": dom["ms"], "algorithmic_bytes": dom["algorithmic_bytes"],
                           "roofline_frac": dom["roofline_frac"]},
        "prepare_ms": r["prepare_ms"], "schedule_ms": r["schedule_ms"], "break_even_epochs": r.get("break_even_epochs"),
        "path_bytes_over_csr_bytes": r["path_bytes_over_csr_bytes"],
    }
    if "hip_graph_ms_per_epoch" in r["partially_active"]:
        out["hip_graph_ms_per_epoch"] = r["partially_active"]["hip_graph_ms_per_epoch"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=int(os.environ.get("EPP_BENCH_CONFIG", "5")),
                    help="headline workload (metric, roofline, cpu_baseline); default 5, the largest")
    ap.add_argument("--only", action="store_true", help="skip the compact report on the other configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-active", action="store_true")
    ap.add_argument("--no-combination", action="store_true", help="skip the combination-stage report")
    ap.add_argument("--cpu-budget-s", type=float, default=15.0)
    ap.add_argument("--layers", type=str, default="", help="comma list of layers to run (profiling); default all")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no multi-GPU part); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2204_02662_amd as epp

    epp.load_library()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    head, cfg = run_config(args.config, args, detail=True)
    ms_partial = head["partially_active"]["ms_per_epoch"]
    result = {
        "metric": "backward_aggregation_ms_per_epoch", "value": ms_partial, "unit": "ms/epoch",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_partial,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "kernel_sources": kernel_source_hash(),
    }
    result.update(head)

    # the other benchmark configurations, timed in this same run (compact form)
    if not args.only and not args.layers:
        side = {}
        for k in (1, 2, 3, 4, 5):
            if k == args.config:
                continue
            r, c = run_config(k, args, detail=False)
            side[f"cfg{k}"] = compact(r)
            del r, c
        result["configs"] = side

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.cpu_budget_s)
    else:
        result["cpu_baseline"] = None

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
