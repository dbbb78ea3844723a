"""Shared helpers of the GPU parity tests (test infrastructure: may use the oracle)."""
from __future__ import annotations

import numpy as np
import torch

import graphgen
import oracle
import paper_2204_02662_amd as epp

RTOL = 1e-5   # tolerance fixed by the task: |gpu - oracle| <= ATOL + RTOL * |oracle|
ATOL = 1e-6


def dev():
    return torch.device("cuda", 0)


def upload_graph(g):
    d = dev()
    return (torch.from_numpy(g.rowptr).to(d), torch.from_numpy(g.col).to(d), torch.from_numpy(g.val).to(d))


def gpu_prepare(g, train_ids, L):
    rowptr, col, val = upload_graph(g)
    ids = torch.from_numpy(np.ascontiguousarray(train_ids, np.int32)).to(dev())
    return epp.epp_prepare(g.n, rowptr, col, val, ids, L)


def gpu_prepare_full(g):
    rowptr, col, val = upload_graph(g)
    return epp.epp_prepare_full(g.n, rowptr, col, val)


def assert_paths_bit_exact(paths, sets_o, paths_o, L):
    """Execution paths and active sets from the library against the oracle, bit for bit."""
    assert paths.num_layers == L
    for k in range(L + 1):
        got = paths.active_set(k).cpu().numpy()
        assert np.array_equal(got, np.flatnonzero(sets_o[k]).astype(np.int32)), f"N^{k}"
    for l in range(L):
        p = paths.path(l)
        row_ids, rowptr, col, val = (t.cpu().numpy() for t in p.export())
        po = paths_o[l]
        assert np.array_equal(row_ids, po.row_ids), f"row_ids l={l}"
        assert np.array_equal(rowptr, po.rowptr), f"rowptr l={l}"
        assert np.array_equal(col, po.col), f"col l={l}"
        assert np.array_equal(val.view(np.int32), po.val.view(np.int32)), f"val l={l}"
        i = p.info()
        assert (i.n_rows, i.nnz, i.n_src) == (po.row_ids.size, po.col.size, int(sets_o[L - l - 1].sum()))
        lens = np.diff(po.rowptr)
        assert i.max_len == (int(lens.max()) if lens.size else 0)
        cls = np.where(lens <= 1, 0, np.ceil(np.log2(np.maximum(lens, 1))).astype(np.int64))
        assert i.len_hist == np.bincount(cls, minlength=32).tolist()


def assert_close(got: np.ndarray, want: np.ndarray, what=""):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bound = ATOL + RTOL * np.abs(want.astype(np.float64))
    bad = err > bound
    if bad.any() or not np.isfinite(got).all():
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} entries out of tolerance; worst at {idx}: "
                             f"got {got[idx]!r} want {want[idx]!r}")


def run_partial(path, X: np.ndarray, poison: float | None = None) -> np.ndarray:
    """grad_out starts at zero (or `poison` to show which rows are written)."""
    d = dev()
    gin = torch.from_numpy(X).to(d)
    gout = torch.zeros_like(gin) if poison is None else torch.full_like(gin, poison)
    path.prepare_width(gin.shape[1])  # one-off per (path, width); the aggregate call only enqueues
    epp.epp_backward_aggregate(path, gin, gout)
    torch.cuda.synchronize()
    return gout.cpu().numpy()


def run_full(full, X: np.ndarray) -> np.ndarray:
    d = dev()
    gin = torch.from_numpy(X).to(d)
    gout = torch.full_like(gin, 7.0)  # every row must be overwritten
    full.prepare_width(gin.shape[1])
    epp.epp_full_aggregate(full, gin, gout)
    torch.cuda.synchronize()
    return gout.cpu().numpy()


def run_ifelse(full, paths, l, X: np.ndarray, poison: float = 123.0) -> np.ndarray:
    """If-else selective scheduling baseline; grad_out starts at `poison`."""
    d = dev()
    gin = torch.from_numpy(X).to(d)
    gout = torch.full_like(gin, poison)
    full.prepare_width(gin.shape[1])
    epp.epp_ifelse_aggregate(full, paths, l, gin, gout)
    torch.cuda.synchronize()
    return gout.cpu().numpy()
