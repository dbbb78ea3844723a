"""The entry point that allocates nothing (epp_weight_gradient_static) against the entry point it is
a variant of (epp_weight_gradient), through the C ABI, on calls in a row that share the static
device array: the second call has a smaller input than the first, so anything it wrongly read
from what the first left behind would show.

Bar: the combination stage's tolerance, |a - b| <= 1e-6 + 1e-5 * sum_k |y_k x_k| (the two entry
points may cut the rows into different blocks of partial sums); bit-equal where the blocks are
the same.  The oracle is checked beside it, so both are right and not merely alike."""
import ctypes

import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2204_02662_amd as epp
from _util import dev, gpu_prepare

pytestmark = pytest.mark.gpu

BLOCK_LIMIT = 8_388_608  # F_in * F_out the static array can hold (32 MiB of floats)


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(np.float32)


def _both(paths, k, sets_o, Fi, Fo, seed):
    """One weight gradient through both entry points; returns (static, workspace, oracle, scale)."""
    d = dev()
    n = paths.n
    Y = _rand((n, Fi), seed)
    G = np.zeros((n, Fo), np.float32)
    member = None
    if k >= 0:
        member = sets_o[k] != 0
        G[member] = _rand((int(member.sum()), Fo), seed + 1)
    else:
        G[:] = _rand((n, Fo), seed + 1)
    Yd, Gd = torch.from_numpy(Y).to(d), torch.from_numpy(G).to(d)
    ws = torch.empty(epp.epp_weight_gradient_workspace(paths, k, Fi, Fo), dtype=torch.uint8, device=d)
    a = torch.full((Fi, Fo), 3.0, device=d)
    b = torch.full((Fi, Fo), 4.0, device=d)
    # (the runtime itself may set memory aside when a kernel is launched for the first time in a
    # process; that is not the entry point's doing, so the bookkeeping below brackets a second call)
    epp.epp_weight_gradient_static(paths, k, Yd, Gd, a)
    torch.cuda.synchronize()
    a.fill_(3.0)
    mem, free = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
    allocs = epp.alloc_stats["allocs"]
    epp.epp_weight_gradient_static(paths, k, Yd, Gd, a)
    # no allocation of any kind: not through PyTorch, not through the library's allocator callback,
    # not behind both (the device's free memory is unchanged)
    assert (torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0], epp.alloc_stats["allocs"]) == (mem, free, allocs)
    epp.epp_weight_gradient(paths, k, Yd, Gd, b, ws)
    torch.cuda.synchronize()
    want, scale = oracle.weight_gradient(Y, G, member)
    return a.cpu().numpy(), b.cpu().numpy(), want, scale


def _check(a, b, want, scale, what):
    bound = 1e-6 + 1e-5 * scale
    assert np.isfinite(a).all(), what
    assert (np.abs(a.astype(np.float64) - b.astype(np.float64)) <= bound).all(), f"{what}: static vs workspace"
    assert (np.abs(a.astype(np.float64) - want) <= bound).all(), f"{what}: static vs oracle"
    assert (np.abs(b.astype(np.float64) - want) <= bound).all(), f"{what}: workspace vs oracle"


def test_static_scratch_weight_gradient_matches_the_workspace_one():
    g = graphgen.random_graph("rmat", 40_000, seed=801, raw_draws=500_000)
    train = graphgen.training_set(g.n, 4000, 802)
    L = 2
    sets_o, _ = oracle.prepare(g.n, g.rowptr, g.col, g.val, train, L)
    paths = gpu_prepare(g, train, L)
    sizes = [int((s != 0).sum()) for s in sets_o]
    assert sizes[0] < sizes[1] < sizes[2]
    # first call: the largest row set (k = -1, all vertices) and wide matrices, so that the array's
    # limit on the number of blocks binds and the two entry points cut the rows differently;
    # second call: far fewer rows (k = 0) and a narrow shape -- it uses a small part of what the
    # first call wrote; then odd widths, then the first shape again
    calls = [(-1, 1024, 1024), (0, 16, 7), (1, 41, 47), (2, 130, 70), (-1, 1024, 1024), (0, 1, 1)]
    first = None
    for i, (k, Fi, Fo) in enumerate(calls):
        a, b, want, scale = _both(paths, k, sets_o, Fi, Fo, 810 + 2 * (i % 4))
        _check(a, b, want, scale, f"call {i}: k={k} {Fi}x{Fo}")
        if (Fi, Fo) != (1024, 1024):  # the array holds as many blocks as the workspace would: same blocks, same sums
            assert np.array_equal(a, b), f"call {i}: same blocks of rows must give the same bits"
        if (k, Fi, Fo) == calls[0]:
            if first is None:
                first = a
            else:
                assert np.array_equal(a, first)  # same input, same result after other calls used the array


def test_static_scratch_limits_and_empty_sets():
    g = graphgen.random_graph("chung_lu", 3000, seed=821, target_edges=9000)
    paths = gpu_prepare(g, np.zeros(0, np.int32), 2)  # empty training set: every N^k is empty
    d = dev()
    Y = torch.randn(g.n, 8, device=d)
    G = torch.zeros(g.n, 5, device=d)
    Wg = torch.full((8, 5), 9.0, device=d)
    epp.epp_weight_gradient_static(paths, 0, Y, G, Wg)
    torch.cuda.synchronize()
    assert not Wg.any()
    # beyond the array's size the call is refused on the host (no kernel is launched)
    lib = epp.load_library()
    p = ctypes.c_void_p(256)
    rc = lib.epp_weight_gradient_static(paths._h, 0, p, 4096, p, 4096, p, None)
    assert rc == epp.EPP_ERR_TOO_LARGE and b"exceeds" in lib.epp_last_error()
    assert 4096 * 2048 == BLOCK_LIMIT
    assert lib.epp_weight_gradient_static(paths._h, 0, p, 4096, p, 2049, p, None) == epp.EPP_ERR_TOO_LARGE
    assert lib.epp_weight_gradient_static(paths._h, 7, p, 4, p, 4, p, None) == epp.EPP_ERR_INVALID_ARG
    assert lib.epp_weight_gradient_static(None, 0, p, 4, p, 4, p, None) == epp.EPP_ERR_INVALID_ARG
