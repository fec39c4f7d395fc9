"""GPU test of the allocation-free entry point gp_edges_by_source_static: through the C ABI, against
gp_edges_by_source (which takes a caller's workspace), bit for bit, on two calls in a row, the second
with a smaller input (the static scratch keeps the first call's contents), plus its size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _both(lib, ctx, pos, gptr, cutoff, cap):
    e, _ = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), cutoff, cap)
    N, E = e["n_atoms"], e["n_edges"]
    want_ptr, want_list = lib.gp_edges_by_source(ctx, e)                 # workspace variant
    out_ptr = torch.full((N + 1,), -7, dtype=torch.int32, device="cuda:0")
    out_list = torch.full((E,), -7, dtype=torch.int32, device="cuda:0")
    # torch's count of allocation requests (it only grows; tensors of earlier tests may be freed at any time)
    before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    raw = lib.load()
    rc = raw.gp_edges_by_source_static(ctx._h, C.c_void_p(e["src"].data_ptr()), C.c_int64(N), C.c_int64(E),
                                       C.c_void_p(out_ptr.data_ptr()), C.c_void_p(out_list.data_ptr()))
    assert rc == 0, raw.gp_last_error(ctx._h)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
    assert torch.equal(out_ptr, want_ptr) and torch.equal(out_list, want_list)
    # and against the definition: edge ids grouped by source atom, ascending within a group
    src = e["src"].cpu().numpy()
    assert np.array_equal(out_list.cpu().numpy(), np.lexsort((np.arange(E), src)))
    assert np.array_equal(np.diff(out_ptr.cpu().numpy()), np.bincount(src, minlength=N))
    return N, E


def test_edges_by_source_static_two_calls_second_smaller(lib):
    ctx = lib.Context(0)
    pos, gptr = synth.slab_adsorbate_positions(4, 8, 5, 4, 40, seed=3)    # 800 atoms, capped: in- and out-lists differ
    n1, e1 = _both(lib, ctx, pos, gptr, 6.0, 50)
    pos2, gptr2 = synth.cube_positions(30, 6.0, 0.9, seed=1)              # smaller: fewer atoms, fewer edges
    n2, e2 = _both(lib, ctx, pos2, gptr2, 4.0, 0)
    assert n2 < n1 and e2 < e1 and e2 > 0


def test_edges_by_source_static_limits_and_empty(lib):
    ctx = lib.Context(0)
    raw = lib.load()
    out_ptr = torch.full((6,), -7, dtype=torch.int32, device="cuda:0")
    rc = raw.gp_edges_by_source_static(ctx._h, None, C.c_int64(5), C.c_int64(0), C.c_void_p(out_ptr.data_ptr()), None)
    torch.cuda.synchronize()
    assert rc == 0 and not out_ptr.any()
    dummy = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    for n_atoms, n_edges in ((65537, 8), (8, 2097153)):
        rc = raw.gp_edges_by_source_static(ctx._h, C.c_void_p(dummy.data_ptr()), C.c_int64(n_atoms), C.c_int64(n_edges),
                                           C.c_void_p(dummy.data_ptr()), C.c_void_p(dummy.data_ptr()))
        assert rc == -5 and b"static scratch" in raw.gp_last_error(ctx._h)
