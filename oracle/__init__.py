"""CPU oracle for partially-active backward aggregation -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``epp_oracle.c`` (plain loops, fp64 accumulation).  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the
GPU library never does, and this package never imports the GPU library.

Notation follows the paper: ``sets[k]`` is the membership vector of N^k_{V_t} (Sec. 3,
Theorem 1), ``paths[l]`` is SG_l (Sec. 4) with rows N^{L-l} and sources N^{L-l-1}.
"""
from __future__ import annotations

import ctypes
import subprocess
from dataclasses import dataclass
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SO = _HERE / "libepp_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    src = _HERE / "epp_oracle.c"
    if force or not _SO.exists() or _SO.stat().st_mtime < src.stat().st_mtime:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", str(src), "-o", str(_SO)])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_SO))
        P, I64 = ctypes.c_void_p, ctypes.c_int64
        lib.oracle_mark_training.restype = ctypes.c_int
        lib.oracle_mark_training.argtypes = [I64, P, I64, P]
        lib.oracle_expand.restype = None
        lib.oracle_expand.argtypes = [I64, P, P, P, P]
        lib.oracle_path_size.restype = None
        lib.oracle_path_size.argtypes = [I64, P, P, P, P, P, P]
        lib.oracle_path_extract.restype = None
        lib.oracle_path_extract.argtypes = [I64] + [P] * 9
        lib.oracle_aggregate.restype = None
        lib.oracle_aggregate.argtypes = [I64, P, P, P, P, P, P, I64, I64, I64]
        lib.oracle_partial_aggregate.restype = None
        lib.oracle_partial_aggregate.argtypes = [I64, P, P, P, P, P, P, P, I64]
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data


def _i32(a):
    return np.ascontiguousarray(a, np.int32)


def _f32(a):
    return np.ascontiguousarray(a, np.float32)


@dataclass
class Path_:
    """Execution path SG_l in canonical form (rows ascending by vertex id, entries in
    input order, columns are original vertex ids)."""
    row_ids: np.ndarray  # int32 [R]
    rowptr: np.ndarray   # int32 [R+1]
    col: np.ndarray      # int32 [nnz]
    val: np.ndarray      # float32 [nnz]


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def set_threads(t: int) -> None:
    _load().oracle_set_threads(int(t))


def active_sets(n, rowptr, col, train_ids, L):
    """[N^0, ..., N^L] as uint8 membership vectors (Theorem 1)."""
    lib = _load()
    rowptr, col, train_ids = _i32(rowptr), _i32(col), _i32(train_ids)
    sets = [np.empty(n, np.uint8)]
    if lib.oracle_mark_training(n, _p(train_ids), train_ids.shape[0], _p(sets[0])) != 0:
        raise ValueError("training id out of range")
    for _ in range(L):
        nxt = np.empty(n, np.uint8)
        lib.oracle_expand(n, _p(rowptr), _p(col), _p(sets[-1]), _p(nxt))
        sets.append(nxt)
    return sets


def extract_path(n, rowptr, col, val, member_rows, member_src) -> Path_:
    """SG with vertex set ``member_rows`` and edge set N(v) ∩ ``member_src`` (Sec. 4)."""
    lib = _load()
    rowptr, col, val = _i32(rowptr), _i32(col), _f32(val)
    R, E = ctypes.c_int64(), ctypes.c_int64()
    lib.oracle_path_size(n, _p(rowptr), _p(col), _p(member_rows), _p(member_src),
                         ctypes.addressof(R), ctypes.addressof(E))
    p = Path_(np.empty(R.value, np.int32), np.empty(R.value + 1, np.int32),
              np.empty(E.value, np.int32), np.empty(E.value, np.float32))
    lib.oracle_path_extract(n, _p(rowptr), _p(col), _p(val), _p(member_rows), _p(member_src),
                            _p(p.row_ids), _p(p.rowptr), _p(p.col), _p(p.val))
    return p


def prepare(n, rowptr, col, val, train_ids, L):
    """Execution-path preparing: returns (sets, paths) with paths[l] = SG_l, l in [0, L)."""
    sets = active_sets(n, rowptr, col, train_ids, L)
    paths = [extract_path(n, rowptr, col, val, sets[L - l], sets[L - l - 1]) for l in range(L)]
    return sets, paths


def full_aggregate(n, rowptr, col, val, grad_in) -> np.ndarray:
    """All-active backward aggregation (Alg. 1): out = M · grad_in over every vertex."""
    lib = _load()
    rowptr, col, val, grad_in = _i32(rowptr), _i32(col), _f32(val), _f32(grad_in)
    F = grad_in.shape[1]
    out = np.zeros((n, F), np.float32)
    lib.oracle_aggregate(n, None, _p(rowptr), _p(col), _p(val), _p(grad_in), _p(out), F, 0, 1)
    return out


def path_aggregate(n, path: Path_, grad_in, first: int = 0, stride: int = 1) -> np.ndarray:
    """Aggregation over an extracted path; rows outside the path stay zero."""
    lib = _load()
    grad_in = _f32(grad_in)
    F = grad_in.shape[1]
    out = np.zeros((n, F), np.float32)
    lib.oracle_aggregate(path.row_ids.shape[0], _p(path.row_ids), _p(path.rowptr), _p(path.col),
                         _p(path.val), _p(grad_in), _p(out), F, first, stride)
    return out


def partial_aggregate(n, rowptr, col, val, member_rows, member_src, grad_in) -> np.ndarray:
    """Alg. 2's aggregation loop on the input graph with explicit membership tests."""
    lib = _load()
    rowptr, col, val, grad_in = _i32(rowptr), _i32(col), _f32(val), _f32(grad_in)
    F = grad_in.shape[1]
    out = np.empty((n, F), np.float32)
    lib.oracle_partial_aggregate(n, _p(rowptr), _p(col), _p(val), _p(member_rows), _p(member_src),
                                 _p(grad_in), _p(out), F)
    return out


# ---------------------------------------------------------------------------------------
# Combination stage of the backward pass (Alg. 1, backward loop: the two lines before the
# aggregation loop).  Plain definitions in fp64; numpy's matrix product is the only library
# step.  `member` restricts both products to the vertices whose rows of X^{(l+1)'} can be
# non-zero (Theorem 1: N^{L-l-1}); with member=None every vertex takes part, which is the
# definition itself.  Pinned by tests/test_oracle_combination.py (loop-by-loop brute force,
# closed forms, the trace identity <W, W'> = <Y, Y'>, finite differences of the forward
# model of Alg. 1, and restricted == unrestricted when the skipped rows are zero).

def _members(n, member):
    return np.arange(n) if member is None else np.flatnonzero(np.asarray(member))


def weight_gradient(Y, grad_X, member=None):
    """W' = Y^T (x) X'  (F_in x F_out), summed over the vertices of `member`.

    Returns (W' in fp64, A) where A[i, j] = sum_v |Y[v, i]| |X'[v, j]| is the scale that
    bounds the rounding error of any fp32 evaluation order."""
    Y = np.asarray(Y)
    grad_X = np.asarray(grad_X)
    assert Y.shape[0] == grad_X.shape[0]
    v = _members(Y.shape[0], member)
    Yv = Y[v].astype(np.float64)
    Xv = grad_X[v].astype(np.float64)
    return Yv.T @ Xv, np.abs(Yv).T @ np.abs(Xv)


def input_gradient(grad_X, W, member=None):
    """Y' = X' (x) W^T  (N x F_in); rows outside `member` are zero.

    Returns (Y' rounded once to fp32, A) with A[v, i] = sum_j |X'[v, j]| |W[i, j]|."""
    grad_X = np.asarray(grad_X)
    W = np.asarray(W)
    assert grad_X.shape[1] == W.shape[1]
    n = grad_X.shape[0]
    v = _members(n, member)
    out = np.zeros((n, W.shape[0]), np.float64)
    scale = np.zeros((n, W.shape[0]), np.float64)
    Xv = grad_X[v].astype(np.float64)
    Wd = W.astype(np.float64)
    out[v] = Xv @ Wd.T
    scale[v] = np.abs(Xv) @ np.abs(Wd).T
    return out.astype(np.float32), scale
