"""Seeded synthetic inputs for the backward-aggregation path.

Only *input data* lives here: graphs (pull-mode CSR of the normalised adjacency with
self-loops), training sets and upstream gradient matrices, in the shapes of the five
benchmark configurations.  Nothing in this package performs frontier expansion, path
extraction or aggregation; the CPU oracle and the GPU library both consume these arrays.

The heavy lifting is in ``graphgen.cpp`` (OpenMP, counter-based random numbers, result
independent of the thread count), loaded through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SO = _HERE / "libgraphgen.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile ``graphgen.cpp`` into ``libgraphgen.so`` next to it."""
    src = _HERE / "graphgen.cpp"
    if force or not _SO.exists() or _SO.stat().st_mtime < src.stat().st_mtime:
        subprocess.check_call(
            ["g++", "-O2", "-fopenmp", "-shared", "-fPIC", str(src), "-o", str(_SO)]
        )
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_SO))
        lib.gg_build.restype = ctypes.c_void_p
        lib.gg_build.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_double, ctypes.c_double,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int,
        ]
        for name in ("gg_n", "gg_nnz", "gg_undirected_edges", "gg_raw_draws"):
            getattr(lib, name).restype = ctypes.c_int64
            getattr(lib, name).argtypes = [ctypes.c_void_p]
        lib.gg_export.restype = None
        lib.gg_export.argtypes = [ctypes.c_void_p] * 4
        lib.gg_free.restype = None
        lib.gg_free.argtypes = [ctypes.c_void_p]
        lib.gg_normal_rows.restype = None
        lib.gg_normal_rows.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_uint64,
        ]
        _lib = lib
    return _lib


@dataclass
class Graph:
    """Pull-mode CSR: row v lists the sources u of edges u -> v, ascending and unique."""
    n: int
    rowptr: np.ndarray  # int32 [n+1]
    col: np.ndarray     # int32 [nnz]
    val: np.ndarray     # float32 [nnz]
    undirected_edges: int = 0
    raw_draws: int = 0

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])


def random_graph(kind: str, n: int, *, seed: int, target_edges: int = 0, raw_draws: int = 0,
                 gamma: float = 2.5, abc=(0.57, 0.19, 0.19), permute: bool = True) -> Graph:
    """Undirected Chung-Lu ('chung_lu') or R-MAT ('rmat') graph, symmetrised, with
    self-loops, vertex ids permuted, weights 1/sqrt(d_v d_u) with d = row length."""
    lib = _load()
    if kind == "chung_lu":
        h = lib.gg_build(0, n, gamma, 0.0, 0.0, target_edges, raw_draws, seed, int(permute))
    elif kind == "rmat":
        h = lib.gg_build(1, n, abc[0], abc[1], abc[2], target_edges, raw_draws, seed, int(permute))
    else:
        raise ValueError(kind)
    if not h:
        raise RuntimeError("graph generation failed (size out of range or target unreachable)")
    try:
        nnz = lib.gg_nnz(h)
        rowptr = np.empty(n + 1, np.int32)
        col = np.empty(nnz, np.int32)
        val = np.empty(nnz, np.float32)
        lib.gg_export(h, rowptr.ctypes.data, col.ctypes.data, val.ctypes.data)
        g = Graph(n, rowptr, col, val, lib.gg_undirected_edges(h), lib.gg_raw_draws(h))
    finally:
        lib.gg_free(h)
    return g


def csr_from_edges(n: int, edges, *, self_loops: bool, symmetric: bool = True,
                   normalise: bool = True) -> Graph:
    """Small hand-written graphs for tests: ``edges`` is a list of (u, v) pairs, 0-based.
    ``symmetric`` stores both directions; otherwise (u, v) means u -> v, i.e. u appears
    in row v.  ``normalise`` gives 1/sqrt(d_v d_u) with d = row length, else weight 1."""
    rows = [set() for _ in range(n)]
    for u, v in edges:
        rows[v].add(u)
        if symmetric:
            rows[u].add(v)
    if self_loops:
        for v in range(n):
            rows[v].add(v)
    rowptr = np.zeros(n + 1, np.int32)
    for v in range(n):
        rowptr[v + 1] = rowptr[v] + len(rows[v])
    col = np.array([u for v in range(n) for u in sorted(rows[v])], np.int32).reshape(-1)
    deg = np.diff(rowptr).astype(np.float64)
    if normalise and col.size:
        dv = np.repeat(deg, np.diff(rowptr))
        du = np.maximum(deg[col], 1.0)
        val = (1.0 / np.sqrt(dv * du)).astype(np.float32)
    else:
        val = np.ones(col.shape[0], np.float32)
    return Graph(n, rowptr, col, val, len(edges), len(edges))


def normal_rows(n: int, F: int, member: np.ndarray | None, seed: int) -> np.ndarray:
    """n x F fp32 matrix, N(0,1) on rows with member[v] != 0 (all rows if None), exact
    zeros elsewhere."""
    lib = _load()
    out = np.zeros((n, F), np.float32)
    mptr = None
    if member is not None:
        member = np.ascontiguousarray(member, np.uint8)
        assert member.shape == (n,)
        mptr = member.ctypes.data
    lib.gg_normal_rows(out.ctypes.data, n, F, mptr, seed)
    return out


def training_set(n: int, count: int, seed: int, degree: np.ndarray | None = None) -> np.ndarray:
    """``count`` distinct vertex ids (int32, in draw order, not sorted).  Uniform without
    replacement, or with P(v) proportional to degree[v] + 1 when ``degree`` is given
    (exponential-key weighted sampling without replacement)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if degree is None:
        ids = rng.choice(n, size=count, replace=False)
    else:
        w = degree.astype(np.float64) + 1.0
        keys = np.log(1.0 - rng.random(n)) / w  # log(u)/w, u in (0,1]
        ids = np.argpartition(keys, n - count)[n - count:]
        ids = ids[np.argsort(-keys[ids], kind="stable")]
    return ids.astype(np.int32)


@dataclass
class Config:
    """One benchmark configuration.  ``widths[l]`` is the gradient width F_l of layer l
    (layer L-1 runs first in an epoch and has the training set as its sources)."""
    index: int
    name: str
    kind: str
    n: int
    L: int
    widths: list
    n_train: int
    target_edges: int = 0
    raw_draws: int = 0
    degree_biased_train: bool = False
    abc: tuple = (0.57, 0.19, 0.19)
    gamma: float = 2.5
    graph: Graph | None = field(default=None, repr=False)
    train_ids: np.ndarray | None = field(default=None, repr=False)

    def seed(self, purpose: int) -> int:
        return 1000 * self.index + purpose


def config_spec(k: int) -> Config:
    """Shape of configuration k in 1..5 (no data generated)."""
    if k == 1:
        return Config(1, "cfg1-citation-2708", "chung_lu", 2708, 2, [16, 7], 140, target_edges=5278)
    if k == 2:
        return Config(2, "cfg2-sparse-19717", "chung_lu", 19717, 2, [16, 3], 60, target_edges=44324)
    if k == 3:
        return Config(3, "cfg3-social-rmat-232965", "rmat", 232965, 2, [16, 41],
                      int(round(0.66 * 232965)), target_edges=57_300_000)
    if k == 4:
        return Config(4, "cfg4-copurchase-2449029", "chung_lu", 2449029, 3, [64, 64, 47], 196615,
                      target_edges=61_900_000)
    if k == 5:
        n = 1 << 23
        return Config(5, "cfg5-stress-rmat23", "rmat", n, 3, [128, 128, 16], int(round(0.01 * n)),
                      raw_draws=16 * n, degree_biased_train=True)
    raise ValueError(f"no configuration {k}")


def _cache_dir() -> Path | None:
    d = os.environ.get("EPP_GRAPH_CACHE", "/tmp/epp_graphgen_cache")
    if d in ("", "0", "off"):
        return None
    p = Path(d)
    try:
        p.mkdir(parents=True, exist_ok=True)
    except OSError:
        return None
    return p


def make_config(k: int, *, cache: bool = True) -> Config:
    """Generate (or load from the on-disk cache) graph and training set of configuration k."""
    cfg = config_spec(k)
    cdir = _cache_dir() if cache else None
    tag = f"v1_cfg{k}"
    if cdir is not None and (cdir / f"{tag}_meta.npy").exists():
        meta = np.load(cdir / f"{tag}_meta.npy")
        cfg.graph = Graph(cfg.n, np.load(cdir / f"{tag}_rowptr.npy"), np.load(cdir / f"{tag}_col.npy"),
                          np.load(cdir / f"{tag}_val.npy"), int(meta[0]), int(meta[1]))
    else:
        cfg.graph = random_graph(cfg.kind, cfg.n, seed=cfg.seed(1), target_edges=cfg.target_edges,
                                 raw_draws=cfg.raw_draws, gamma=cfg.gamma, abc=cfg.abc)
        if cdir is not None:
            g = cfg.graph
            np.save(cdir / f"{tag}_rowptr.npy", g.rowptr)
            np.save(cdir / f"{tag}_col.npy", g.col)
            np.save(cdir / f"{tag}_val.npy", g.val)
            np.save(cdir / f"{tag}_meta.npy", np.array([g.undirected_edges, g.raw_draws], np.int64))
    deg = np.diff(cfg.graph.rowptr) - 1 if cfg.degree_biased_train else None
    cfg.train_ids = training_set(cfg.n, cfg.n_train, cfg.seed(2), deg)
    return cfg


def layer_gradient(cfg: Config, l: int, member: np.ndarray | None) -> np.ndarray:
    """Input gradient matrix of layer l: N(0,1) on the rows flagged in ``member`` (the
    layer's source set), zeros elsewhere; width ``cfg.widths[l]``."""
    return normal_rows(cfg.n, cfg.widths[l], member, cfg.seed(10 + l))
