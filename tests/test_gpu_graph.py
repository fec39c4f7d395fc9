"""GPU parity: edge and triplet lists from the HIP library vs the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _gpu_graph(lib, ctx, pos, gptr, cutoff, cap):
    dpos = H.to_dev(pos, torch.float32)
    dptr = H.to_dev(gptr, torch.int32)
    e, t = lib.build_graph(ctx, dpos, dptr, cutoff, cap)
    torch.cuda.synchronize()
    return e, t


def _check(lib, ctx, pos, gptr, cutoff, cap):
    ref = H.oracle_graph(pos, gptr, cutoff, cap)
    e, t = _gpu_graph(lib, ctx, pos, gptr, cutoff, cap)
    assert e["n_edges"] == len(ref["src"])
    assert t["n_triplets"] == len(ref["idx_kj"])
    assert np.array_equal(e["src"].cpu().numpy(), ref["src"])
    assert np.array_equal(e["dst"].cpu().numpy(), ref["dst"])
    assert np.array_equal(e["row_ptr"].cpu().numpy(), ref["row_ptr"])
    idx_kj, idx_ji = t["idx_kj"].cpu().numpy(), t["idx_ji"].cpu().numpy()
    assert np.array_equal(idx_kj, ref["idx_kj"])
    assert np.array_equal(idx_ji, ref["idx_ji"])
    assert np.array_equal(t["seg_ptr_ji"].cpu().numpy().astype(np.int64), ref["seg"])
    # kj-major view: a permutation of the triplets sorted by (idx_kj, idx_ji)
    perm = t["perm_kj"].cpu().numpy().astype(np.int64)
    assert np.array_equal(np.sort(perm), np.arange(len(perm)))
    key = idx_kj[perm].astype(np.int64) * (len(ref["src"]) + 1) + idx_ji[perm]
    assert np.all(np.diff(key) > 0)
    assert np.array_equal(t["idx_ji_kj"].cpu().numpy(), idx_ji[perm])
    seg_kj = np.zeros(len(ref["src"]) + 1, dtype=np.int64)
    np.add.at(seg_kj, idx_kj.astype(np.int64) + 1, 1)
    assert np.array_equal(t["seg_ptr_kj"].cpu().numpy().astype(np.int64), np.cumsum(seg_kj))
    # distances and unit vectors against fp64
    p = pos.astype(np.float64)
    vec = p[ref["dst"]] - p[ref["src"]]
    d = np.linalg.norm(vec, axis=1)
    if len(d):
        assert np.abs(e["dist"].cpu().numpy() - d).max() < 2e-6 * max(1.0, d.max())
        assert np.abs(e["unit"].cpu().numpy() - vec / d[:, None]).max() < 2e-6
    return ref


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg1_graph(lib, ctx, seed):
    w = synth.get_workload("cfg1")
    pos, gptr = synth.make_positions(w, seed)
    _check(lib, ctx, pos, gptr, w.dims.cutoff, w.max_neighbors)


@pytest.mark.parametrize("cap", [0, 5, 12, 50])
def test_capped_multi_graph(lib, ctx, cap):
    pos, gptr = synth.slab_adsorbate_positions(3, 4, 3, 3, 7, seed=cap)
    ref = _check(lib, ctx, pos, gptr, 6.0, cap)
    assert len(ref["src"]) > 0


def test_cfg2_full_graph(lib, ctx):
    w = synth.get_workload("cfg2")
    pos, gptr = synth.make_positions(w, 0)
    ref = _check(lib, ctx, pos, gptr, w.dims.cutoff, w.max_neighbors)
    assert len(ref["idx_kj"]) > 1_000_000


def test_more_than_one_wave_of_sources_and_long_segments(lib, ctx):
    # 150 atoms in one structure, large cutoff: > 64 sources per target, > 64 triplets per edge
    pos, gptr = synth.cube_positions(150, 9.0, 0.9, seed=3)
    ref = _check(lib, ctx, pos, gptr, 7.5, 0)
    assert np.diff(ref["row_ptr"]).max() > 64
    ref = _check(lib, ctx, pos, gptr, 7.5, 70)
    assert np.diff(ref["row_ptr"]).max() == 70


def test_degenerate_inputs(lib, ctx):
    # no atoms
    e, t = _gpu_graph(lib, ctx, np.zeros((0, 3), np.float32), np.array([0], np.int32), 5.0, 0)
    assert e["n_edges"] == 0 and t["n_triplets"] == 0
    # one atom: no edges
    e, t = _gpu_graph(lib, ctx, np.zeros((1, 3), np.float32), np.array([0, 1], np.int32), 5.0, 0)
    assert e["n_edges"] == 0 and t["n_triplets"] == 0
    assert e["row_ptr"].cpu().tolist() == [0, 0]
    # two atoms in range: two edges, no triplet (k == i is excluded)
    pos = np.array([[0, 0, 0], [1, 0, 0]], np.float32)
    e, t = _gpu_graph(lib, ctx, pos, np.array([0, 2], np.int32), 5.0, 0)
    assert e["n_edges"] == 2 and t["n_triplets"] == 0
    assert t["seg_ptr_ji"].cpu().tolist() == [0, 0, 0] and t["seg_ptr_kj"].cpu().tolist() == [0, 0, 0]
    # two structures never connect; an empty structure in between is allowed
    pos = np.array([[0, 0, 0], [1, 0, 0], [0.5, 0, 0]], np.float32)
    e, t = _gpu_graph(lib, ctx, pos, np.array([0, 2, 2, 3], np.int32), 5.0, 0)
    assert e["n_edges"] == 2
    # three collinear atoms all in range: 6 edges, 6 triplets
    pos = np.array([[0, 0, 0], [1, 0, 0], [2, 0, 0]], np.float32)
    _check(lib, ctx, pos, np.array([0, 3], np.int32), 5.0, 0)


def test_error_codes(lib, ctx):
    import ctypes as C
    L = lib.load()
    pos = H.to_dev(np.zeros((4, 3), np.float32), torch.float32)
    gptr = H.to_dev(np.array([0, 4], np.int32), torch.int32)
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda:0")
    n = C.c_int64()
    rc = L.gp_edges_count(ctx._h, C.c_void_p(pos.data_ptr()), C.c_void_p(gptr.data_ptr()), C.c_int64(4), C.c_int32(1),
                          C.c_float(-1.0), C.c_int32(0), C.c_void_p(ws.data_ptr()), C.c_size_t(4096), C.byref(n))
    assert rc == -1 and b"cutoff" in L.gp_last_error(ctx._h)
    rc = L.gp_edges_count(ctx._h, C.c_void_p(pos.data_ptr()), C.c_void_p(gptr.data_ptr()), C.c_int64(4), C.c_int32(1),
                          C.c_float(2.0), C.c_int32(0), C.c_void_p(ws.data_ptr()), C.c_size_t(8), C.byref(n))
    assert rc == -2
    rc = L.gp_edges_count(ctx._h, None, C.c_void_p(gptr.data_ptr()), C.c_int64(4), C.c_int32(1),
                          C.c_float(2.0), C.c_int32(0), C.c_void_p(ws.data_ptr()), C.c_size_t(4096), C.byref(n))
    assert rc == -1
    rc = L.gp_edges_count(ctx._h, C.c_void_p(pos.data_ptr()), C.c_void_p(gptr.data_ptr()), C.c_int64(-4), C.c_int32(1),
                          C.c_float(2.0), C.c_int32(0), C.c_void_p(ws.data_ptr()), C.c_size_t(4096), C.byref(n))
    assert rc == -1
