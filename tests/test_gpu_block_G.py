"""GPU parity: the variant-G (bilinear) interaction block, forward and backward, vs the fp64 oracle.

Tolerance: relative L2 error <= 1e-4 per tensor for the fp32 path.
"""
import numpy as np
import pytest
import torch

import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
TOL = 1e-4
ROW_FACTOR = 4.0     # a row may deviate this much more than the whole tensor (single rows do not average rounding noise)
ELEM_FACTOR = 16.0   # the same for tensors whose rows are single numbers (one value per triplet): nothing averages there, and
                     # an element's rounding error scales with the size of ITS terms, whose distribution has a long tail


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _parity(lib, ctx, workload, seed, n_blocks, pos_gptr, tol=TOL):
    from paper_2203_09697_amd.binding_g import StackG
    dims = workload.dims
    pos, gptr = pos_gptr
    ref = H.oracle_graph(pos, gptr, dims.cutoff, workload.max_neighbors)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), dims.cutoff,
                           workload.max_neighbors)
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    E = len(ref["src"])
    W_list = [synth.weights_G(dims, seed=200 + seed + b) for b in range(n_blocks)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=seed + 7)
    ob = H.oracle_basis_G(pos, ref, dims)
    out_ref, gm_ref, gW_ref, grbf_ref, gcos_ref = H.oracle_stack_G(ref, ob, dims, W_list, m, gup, want_grad_cos=True)
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    assert H.rel_l2(gb["rbf"].cpu().numpy(), ob["rbf"].numpy()) < 1e-5
    stack = StackG(ctx, dims, [lib.weights_to_device(W) for W in W_list], t, gb)
    out = stack.forward(H.to_dev(m, torch.float32))
    grbf = torch.empty((E, dims.num_radial), dtype=torch.float32, device="cuda:0")
    gcos = torch.empty(t["n_triplets"], dtype=torch.float32, device="cuda:0")
    gm, gW = stack.backward(H.to_dev(gup, torch.float32), grad_rbf=grbf, grad_cos_kj=gcos)
    torch.cuda.synchronize()
    pairs = {"m_out": (out, out_ref), "grad_m": (gm, gm_ref), "grad_rbf": (grbf, grbf_ref), "grad_cos_kj": (gcos, gcos_ref)}
    for b in range(n_blocks):
        for k in gW_ref[b]:
            pairs[f"block{b}.{k}"] = (gW[b][k], gW_ref[b][k])
    errs, rows = {}, {}
    for k, (got, want) in pairs.items():
        got = got.cpu().numpy()
        errs[k] = H.rel_l2(got, want)
        rows[k] = H.row_err(got, want)
    print("rel-L2  ", {k: "%.1e" % v for k, v in errs.items()})
    print("row max ", {k: "%.1e" % v for k, v in rows.items()})
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
    # per-row bound: no row (edge, triplet, weight row) may be off by more than ROW_FACTOR times the tensor bound
    bad = {k: v for k, v in rows.items() if not v <= (ELEM_FACTOR if pairs[k][1].ndim == 1 else ROW_FACTOR) * tol}
    assert not bad, ("per-row", bad)
    return errs


def test_block_G_small_dims(lib, ctx):
    w = synth.get_workload("cfg3", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0, dtype="f32")
    _parity(lib, ctx, w, 0, 2, synth.cube_positions(30, 6.0, 0.9, seed=1))


def test_block_G_cfg3_shape_one_structure(lib, ctx):
    # configuration-3 layer widths on one of its 8 structures (200 atoms, cap 50)
    w = synth.get_workload("cfg3", dtype="f32")
    _parity(lib, ctx, w, 1, 1, synth.slab_adsorbate_positions(1, 8, 5, 4, 40, seed=2))


def test_block_G_cfg4_widths_small_graph(lib, ctx):
    # configuration-4 layer widths (emb 1024, emb_trip 128) on a 60-atom box with long segments
    w = synth.get_workload("cfg4", dtype="f32", cutoff=6.0)
    _parity(lib, ctx, w, 2, 1, synth.box_positions(60, 0.08, 0.9, seed=3))


# ---- radial factor of the triplet basis at the target edge (the mirrored form) ----
def test_block_G_radial_at_target_small_dims(lib, ctx):
    w = synth.get_workload("cfg3", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0, dtype="f32", radial_at_target=True)
    _parity(lib, ctx, w, 0, 2, synth.cube_positions(30, 6.0, 0.9, seed=1))


def test_block_G_radial_at_target_cfg3_shape(lib, ctx):
    w = synth.get_workload("cfg3", dtype="f32", radial_at_target=True)
    _parity(lib, ctx, w, 1, 1, synth.slab_adsorbate_positions(1, 8, 5, 4, 40, seed=2))


@pytest.fixture
def trip_mode(lib, ctx, request):
    # 0: per-edge vector triplet kernels, 1: matrix-core kernels whenever usable (here: on the mirrored views)
    lib.gp_set_triplet_mfma(ctx, request.param)
    yield request.param
    lib.gp_set_triplet_mfma(ctx, -1)


@pytest.mark.parametrize("trip_mode", [0, 1], indirect=True)
def test_block_G_radial_at_target_cfg4_widths_bf16(lib, ctx, trip_mode):
    w = synth.get_workload("cfg4", cutoff=6.0, radial_at_target=True)
    assert w.dims.dtype == "bf16"
    _parity(lib, ctx, w, 2, 1, synth.box_positions(60, 0.08, 0.9, seed=3), tol=2e-2)


@pytest.mark.parametrize("trip_mode", [0, 1], indirect=True)
def test_block_G_radial_at_target_bf16_capped_two_structures(lib, ctx, trip_mode):
    # neighbour cap (in- and out-edge lists of an atom differ) and two structures, configuration-3 widths
    w = synth.get_workload("cfg3", radial_at_target=True)
    _parity(lib, ctx, w, 3, 1, synth.slab_adsorbate_positions(2, 4, 4, 4, 16, seed=4), tol=2e-2)


# ---- symmetric message passing (the two messages on a bond are coupled) ----
def test_reverse_edges_bit_exact(lib, ctx):
    from oracle import graph as ograph
    for cap, seed in ((0, 1), (9, 2), (3, 3)):
        pos, gptr = synth.slab_adsorbate_positions(2, 4, 3, 3, 7, seed=seed)
        ref = H.oracle_graph(pos, gptr, 5.0, cap)
        e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), 5.0, cap)
        want = ograph.reverse_edges(ref["src"], ref["dst"])
        assert np.array_equal(t["id_swap"].cpu().numpy(), want)
        assert (want < 0).any() == (cap > 0)


def test_block_G_symmetric_small_dims(lib, ctx):
    w = synth.get_workload("cfg3", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0, dtype="f32", symmetric=True)
    _parity(lib, ctx, w, 0, 2, synth.cube_positions(30, 6.0, 0.9, seed=1))


def test_block_G_symmetric_cfg3_shape_capped(lib, ctx):
    # the neighbour cap leaves some edges without an opposite edge
    from dataclasses import replace
    w = replace(synth.get_workload("cfg3", dtype="f32", symmetric=True), max_neighbors=20)
    _parity(lib, ctx, w, 1, 1, synth.slab_adsorbate_positions(1, 8, 5, 4, 40, seed=2))


@pytest.mark.parametrize("trip_mode", [0, 1], indirect=True)
def test_block_G_symmetric_and_radial_at_target_bf16(lib, ctx, trip_mode):
    w = synth.get_workload("cfg4", cutoff=6.0, symmetric=True, radial_at_target=True)
    _parity(lib, ctx, w, 2, 1, synth.box_positions(60, 0.08, 0.9, seed=3), tol=2e-2)
