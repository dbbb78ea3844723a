"""Thin Python binding of libepp (C ABI, see include/epp.h).

Argument marshalling only: every step of the path runs inside the HIP library.  PyTorch
supplies device memory (tensors) and the current stream.  There is no CPU fallback: if the
shared library is missing or cannot be loaded, importing the functions below raises.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from pathlib import Path

import torch

PKG = Path(__file__).resolve().parent
SO = PKG / "libepp.so"

EPP_OK = 0
EPP_ERR_INVALID_ARG = -1
EPP_ERR_OUT_OF_RANGE_ID = -2
EPP_ERR_TOO_LARGE = -3
EPP_ERR_ALLOC = -4
EPP_ERR_HIP = -5

EXPORTED = [
    "epp_prepare", "epp_prepare_full", "epp_num_layers", "epp_get_path", "epp_path_info",
    "epp_path_export", "epp_active_set_export", "epp_select_group_size", "epp_path_set_group_size",
    "epp_backward_aggregate", "epp_full_aggregate", "epp_destroy_paths", "epp_destroy_path",
    "epp_last_error", "epp_paper_linreg_group_size", "epp_ifelse_aggregate",
    "epp_weight_gradient_workspace", "epp_weight_gradient", "epp_input_gradient", "epp_paths_import",
    "epp_path_prepare_width", "epp_weight_gradient_static",
]


class EppError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libepp error {code}: {message}")
        self.code = code


class _Csr(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("nnz", ctypes.c_int64), ("rowptr", ctypes.c_void_p),
                ("col", ctypes.c_void_p), ("val", ctypes.c_void_p)]


class _PathArrays(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("nnz", ctypes.c_int64), ("row_ids", ctypes.c_void_p),
                ("rowptr", ctypes.c_void_p), ("col", ctypes.c_void_p), ("val", ctypes.c_void_p)]


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class _Alloc(ctypes.Structure):
    _fields_ = [("alloc", _ALLOC_FN), ("free", _FREE_FN), ("ctx", ctypes.c_void_p)]


#: calls and bytes that went through the PyTorch-backed allocator handed to the library
alloc_stats = {"allocs": 0, "frees": 0, "bytes": 0, "live": 0}


def _torch_alloc(nbytes, _ctx):
    """epp_alloc_t.alloc: a block of PyTorch's caching allocator on the current device and stream."""
    try:
        ptr = torch.cuda.caching_allocator_alloc(int(nbytes))
    except Exception:  # out of memory: the library reports EPP_ERR_ALLOC
        return None
    alloc_stats["allocs"] += 1
    alloc_stats["bytes"] += int(nbytes)
    alloc_stats["live"] += 1
    return ptr


def _torch_free(ptr, _ctx):
    """epp_alloc_t.free: the block goes back to the caching allocator (stream-ordered reuse)."""
    alloc_stats["frees"] += 1
    alloc_stats["live"] -= 1
    torch.cuda.caching_allocator_delete(ptr)


_TORCH_ALLOC = _Alloc(_ALLOC_FN(_torch_alloc), _FREE_FN(_torch_free), None)


def _allocator(use_torch: bool):
    """Pointer to the PyTorch-backed epp_alloc_t, or NULL for the library's own hipMalloc."""
    return ctypes.byref(_TORCH_ALLOC) if use_torch else None


class _PathInfo(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("n_rows", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("n_src", ctypes.c_int64), ("max_len", ctypes.c_int64), ("len_hist", ctypes.c_int64 * 32),
                ("bytes", ctypes.c_int64), ("sched_F", ctypes.c_int32), ("group_size", ctypes.c_int32),
                ("n_groups", ctypes.c_int64), ("n_split_rows", ctypes.c_int64),
                ("part_rows", ctypes.c_int64), ("part_hot_entries", ctypes.c_int64),
                ("part_partial_rows", ctypes.c_int64), ("shares_entries", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libepp.so (built by ``paper_2204_02662_amd.build``); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not SO.exists():
        raise FileNotFoundError(f"{SO} not built: run `python -m paper_2204_02662_amd.build`")
    lib = ctypes.CDLL(str(SO))
    P, I, I64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    A = ctypes.POINTER(_Alloc)
    lib.epp_prepare.argtypes = [ctypes.POINTER(_Csr), P, I64, I, A, P, ctypes.POINTER(P)]
    lib.epp_prepare_full.argtypes = [ctypes.POINTER(_Csr), A, P, ctypes.POINTER(P)]
    lib.epp_path_prepare_width.argtypes = [P, I, P]
    lib.epp_num_layers.argtypes = [P]
    lib.epp_get_path.argtypes = [P, I]
    lib.epp_get_path.restype = P
    lib.epp_path_info.argtypes = [P, ctypes.POINTER(_PathInfo)]
    lib.epp_path_export.argtypes = [P, P, P, P, P, P]
    lib.epp_active_set_export.argtypes = [P, I, P, ctypes.POINTER(I64), P]
    lib.epp_select_group_size.argtypes = [P, I]
    lib.epp_path_set_group_size.argtypes = [P, I, I, P]
    lib.epp_paper_linreg_group_size.argtypes = [I64, I64]
    lib.epp_backward_aggregate.argtypes = [P, P, P, I, P]
    lib.epp_full_aggregate.argtypes = [P, P, P, I, P]
    lib.epp_ifelse_aggregate.argtypes = [P, P, I, P, P, I, P]
    lib.epp_weight_gradient_workspace.argtypes = [P, I, I, I]
    lib.epp_weight_gradient_workspace.restype = I64
    lib.epp_weight_gradient.argtypes = [P, I, P, I, P, I, P, P, I64, P]
    lib.epp_weight_gradient_static.argtypes = [P, I, P, I, P, I, P, P]
    lib.epp_input_gradient.argtypes = [P, I, P, I, P, I, P, P]
    lib.epp_paths_import.argtypes = [I64, I, P, I64, ctypes.POINTER(_PathArrays), A, P, ctypes.POINTER(P)]
    lib.epp_destroy_paths.argtypes = [P]
    lib.epp_destroy_paths.restype = None
    lib.epp_destroy_path.argtypes = [P]
    lib.epp_destroy_path.restype = None
    lib.epp_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int) -> int:
    if rc < 0:
        raise EppError(rc, load_library().epp_last_error().decode())
    return rc


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    return t


def _csr(n, rowptr, col, val):
    _dev(rowptr, torch.int32), _dev(col, torch.int32), _dev(val, torch.float32)
    if rowptr.numel() != n + 1 or col.numel() != val.numel():
        raise ValueError("inconsistent CSR arrays")
    return _Csr(n, col.numel(), rowptr.data_ptr(), col.data_ptr(), val.data_ptr())


@dataclass
class PathInfo:
    n: int
    n_rows: int
    nnz: int
    n_src: int
    max_len: int
    len_hist: list
    bytes: int
    sched_F: int
    group_size: int
    n_groups: int
    n_split_rows: int
    part_rows: int = 0
    part_hot_entries: int = 0
    part_partial_rows: int = 0
    shares_entries: int = 0


class Path_:
    """One execution path SG_l (or the all-active graph).  Borrowed from a Paths object
    unless ``owned``."""

    def __init__(self, handle: int, owned: bool, keepalive=None):
        self._h = handle
        self._owned = owned
        self._keepalive = keepalive
        self._n = None

    @property
    def n(self) -> int:
        """Vertices of the input graph (rows of the gradient matrices)."""
        if self._n is None:
            self._n = self.info().n
        return self._n

    def info(self) -> PathInfo:
        raw = _PathInfo()
        _check(load_library().epp_path_info(self._h, ctypes.byref(raw)))
        return PathInfo(raw.n, raw.n_rows, raw.nnz, raw.n_src, raw.max_len, list(raw.len_hist), raw.bytes,
                        raw.sched_F, raw.group_size, raw.n_groups, raw.n_split_rows, raw.part_rows,
                        raw.part_hot_entries, raw.part_partial_rows, raw.shares_entries)

    def export(self):
        """(row_ids, rowptr, col, val) device tensors in canonical form."""
        i = self.info()
        dev = torch.device("cuda", torch.cuda.current_device())
        row_ids = torch.empty(i.n_rows, dtype=torch.int32, device=dev)
        rowptr = torch.empty(i.n_rows + 1, dtype=torch.int32, device=dev)
        col = torch.empty(i.nnz, dtype=torch.int32, device=dev)
        val = torch.empty(i.nnz, dtype=torch.float32, device=dev)
        _check(load_library().epp_path_export(self._h, row_ids.data_ptr(), rowptr.data_ptr(), col.data_ptr(),
                                              val.data_ptr(), _stream()))
        return row_ids, rowptr, col, val

    def select_group_size(self, F: int) -> int:
        return _check(load_library().epp_select_group_size(self._h, F))

    def set_group_size(self, F: int, gs: int) -> None:
        _check(load_library().epp_path_set_group_size(self._h, F, gs, _stream()))

    def prepare_width(self, F: int) -> None:
        """One-off schedule of this path for gradient width F (allocates, synchronises); required
        before the aggregate calls, which only enqueue."""
        _check(load_library().epp_path_prepare_width(self._h, F, _stream()))

    def __del__(self):
        if getattr(self, "_owned", False) and self._h and _lib is not None:
            _lib.epp_destroy_path(self._h)
            self._h = None


class Paths:
    """All L execution paths and the sets N^0..N^L (handle from epp_prepare)."""

    def __init__(self, handle: int):
        self._h = handle

    @property
    def num_layers(self) -> int:
        return _check(load_library().epp_num_layers(self._h))

    @property
    def n(self) -> int:
        """Vertices of the input graph."""
        return self.path(0).info().n

    def path(self, l: int) -> Path_:
        h = load_library().epp_get_path(self._h, l)
        if not h:
            raise EppError(EPP_ERR_INVALID_ARG, load_library().epp_last_error().decode())
        return Path_(h, owned=False, keepalive=self)

    def active_set(self, k: int) -> torch.Tensor:
        """Ascending vertex ids of N^k (device int32 tensor)."""
        lib = load_library()
        cnt = ctypes.c_int64(0)
        _check(lib.epp_active_set_export(self._h, k, None, ctypes.byref(cnt), _stream()))
        ids = torch.empty(cnt.value, dtype=torch.int32, device=torch.device("cuda", torch.cuda.current_device()))
        _check(lib.epp_active_set_export(self._h, k, ids.data_ptr(), ctypes.byref(cnt), _stream()))
        return ids

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.epp_destroy_paths(self._h)
            self._h = None


def epp_prepare(n: int, rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor, train_ids: torch.Tensor,
                L: int, torch_allocator: bool = True) -> Paths:
    """Execution paths of (graph, training set, L).  With ``torch_allocator`` every device buffer of
    the handle comes from PyTorch's caching allocator (epp_alloc_t), otherwise from hipMalloc."""
    lib = load_library()
    csr = _csr(n, rowptr, col, val)
    _dev(train_ids, torch.int32)
    out = ctypes.c_void_p()
    _check(lib.epp_prepare(ctypes.byref(csr), train_ids.data_ptr(), train_ids.numel(), L, _allocator(torch_allocator),
                           _stream(), ctypes.byref(out)))
    return Paths(out.value)


def epp_prepare_full(n: int, rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor,
                     torch_allocator: bool = True) -> Path_:
    lib = load_library()
    csr = _csr(n, rowptr, col, val)
    out = ctypes.c_void_p()
    _check(lib.epp_prepare_full(ctypes.byref(csr), _allocator(torch_allocator), _stream(), ctypes.byref(out)))
    return Path_(out.value, owned=True)


def epp_paper_linreg_group_size(vertices: int, undirected_edges: int) -> int:
    """Sec. 5 linear-regression group size (comparison only)."""
    return _check(load_library().epp_paper_linreg_group_size(vertices, undirected_edges))


def _grads(path: Path_, grad_in: torch.Tensor, grad_out: torch.Tensor) -> int:
    _dev(grad_in, torch.float32), _dev(grad_out, torch.float32)
    if grad_in.dim() != 2 or grad_in.shape != grad_out.shape:
        raise ValueError("grad_in and grad_out must be n x F matrices of the same shape")
    if grad_in.shape[0] != path.n:  # the kernels index rows by vertex id: fewer rows would be read out of bounds
        raise ValueError(f"gradient matrices have {grad_in.shape[0]} rows, the graph has {path.n} vertices")
    return grad_in.shape[1]


def epp_backward_aggregate(path: Path_, grad_in: torch.Tensor, grad_out: torch.Tensor) -> None:
    F = _grads(path, grad_in, grad_out)
    _check(load_library().epp_backward_aggregate(path._h, grad_in.data_ptr(), grad_out.data_ptr(), F, _stream()))


def epp_full_aggregate(full: Path_, grad_in: torch.Tensor, grad_out: torch.Tensor) -> None:
    F = _grads(full, grad_in, grad_out)
    _check(load_library().epp_full_aggregate(full._h, grad_in.data_ptr(), grad_out.data_ptr(), F, _stream()))


def epp_ifelse_aggregate(full: Path_, paths: Paths, l: int, grad_in: torch.Tensor, grad_out: torch.Tensor) -> None:
    """If-else selective scheduling baseline (Sec. 4): all-active traversal with activity tests."""
    F = _grads(full, grad_in, grad_out)
    _check(load_library().epp_ifelse_aggregate(full._h, paths._h, l, grad_in.data_ptr(), grad_out.data_ptr(), F,
                                               _stream()))


def _matrix(t: torch.Tensor, what: str) -> torch.Tensor:
    _dev(t, torch.float32)
    if t.dim() != 2:
        raise ValueError(f"{what} must be a matrix")
    return t


def epp_weight_gradient_workspace(paths: Paths, k: int, F_in: int, F_out: int) -> int:
    return _check(load_library().epp_weight_gradient_workspace(paths._h, k, F_in, F_out))


def epp_weight_gradient(paths: Paths, k: int, Y: torch.Tensor, grad_X: torch.Tensor, grad_W: torch.Tensor,
                        workspace: torch.Tensor) -> None:
    """W' = Y^T (x) X' over the rows of N^k (k = -1: all rows); `workspace` is a CUDA uint8 tensor of
    at least epp_weight_gradient_workspace(...) bytes."""
    _matrix(Y, "Y"), _matrix(grad_X, "grad_X"), _matrix(grad_W, "grad_W")
    if Y.shape[0] != paths.n or grad_X.shape[0] != paths.n or grad_W.shape != (Y.shape[1], grad_X.shape[1]):
        raise ValueError("shapes: Y n x F_in, grad_X n x F_out, grad_W F_in x F_out")
    if not workspace.is_cuda or workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous CUDA uint8 tensor")
    _check(load_library().epp_weight_gradient(paths._h, k, Y.data_ptr(), Y.shape[1], grad_X.data_ptr(), grad_X.shape[1],
                                              grad_W.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))


def epp_weight_gradient_static(paths: Paths, k: int, Y: torch.Tensor, grad_X: torch.Tensor,
                               grad_W: torch.Tensor) -> None:
    """epp_weight_gradient without a workspace: the partial sums use the library's static device array
    (no allocation anywhere; F_in * F_out <= 8,388,608; calls on one GPU must not overlap)."""
    _matrix(Y, "Y"), _matrix(grad_X, "grad_X"), _matrix(grad_W, "grad_W")
    if Y.shape[0] != paths.n or grad_X.shape[0] != paths.n or grad_W.shape != (Y.shape[1], grad_X.shape[1]):
        raise ValueError("shapes: Y n x F_in, grad_X n x F_out, grad_W F_in x F_out")
    _check(load_library().epp_weight_gradient_static(paths._h, k, Y.data_ptr(), Y.shape[1], grad_X.data_ptr(),
                                                     grad_X.shape[1], grad_W.data_ptr(), _stream()))


def epp_input_gradient(paths: Paths, k: int, grad_X: torch.Tensor, W: torch.Tensor, grad_Y: torch.Tensor) -> None:
    """Y' = X' (x) W^T on the rows of N^k (k = -1: all rows); other rows of grad_Y are not touched."""
    _matrix(grad_X, "grad_X"), _matrix(W, "W"), _matrix(grad_Y, "grad_Y")
    if grad_X.shape[0] != paths.n or W.shape[1] != grad_X.shape[1] or grad_Y.shape != (grad_X.shape[0], W.shape[0]):
        raise ValueError("shapes: grad_X n x F_out, W F_in x F_out, grad_Y n x F_in")
    _check(load_library().epp_input_gradient(paths._h, k, grad_X.data_ptr(), grad_X.shape[1], W.data_ptr(), W.shape[0],
                                             grad_Y.data_ptr(), _stream()))


def epp_paths_import(n: int, train_ids: torch.Tensor, layers, torch_allocator: bool = True) -> Paths:
    """Handle from saved paths: ``layers[l]`` = (row_ids, rowptr, col, val) device tensors of SG_l in the
    canonical form that ``Path_.export()`` returns."""
    _dev(train_ids, torch.int32)
    arr = (_PathArrays * len(layers))()
    for l, (row_ids, rowptr, col, val) in enumerate(layers):
        _dev(row_ids, torch.int32), _dev(rowptr, torch.int32), _dev(col, torch.int32), _dev(val, torch.float32)
        if rowptr.numel() != row_ids.numel() + 1 or col.numel() != val.numel():
            raise ValueError(f"layer {l}: inconsistent array lengths")
        arr[l] = _PathArrays(row_ids.numel(), col.numel(), row_ids.data_ptr(), rowptr.data_ptr(), col.data_ptr(),
                             val.data_ptr())
    out = ctypes.c_void_p()
    _check(load_library().epp_paths_import(n, len(layers), train_ids.data_ptr(), train_ids.numel(), arr,
                                           _allocator(torch_allocator), _stream(), ctypes.byref(out)))
    return Paths(out.value)
