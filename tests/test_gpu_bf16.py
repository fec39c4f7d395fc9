"""GPU parity of the bf16-operand (fp32-accumulate) MFMA path: dense layer and the variant-G block.

Bar: relative L2 error <= 2e-2 per tensor against the fp64 oracle fed the unrounded fp32 inputs
(the target's bf16 figure).  The dense layer is additionally checked against the exact product of
the bf16-rounded operands, which pins the MFMA operand layout independently of rounding noise.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import block as oblock
from tests import helpers as H
from tests.test_gpu_block_G import _parity

pytestmark = pytest.mark.gpu
F64 = torch.float64


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


@pytest.mark.parametrize("rows,k,n,act", [(1, 8, 4, 0), (37, 32, 16, 1), (300, 6, 32, 0), (1000, 256, 256, 1),
                                            (513, 64, 512, 1), (2049, 1024, 64, 0), (129, 42, 8, 0), (5, 7, 3, 1),
                                            (700, 1024, 1024, 0)])
def test_linear_forward_bf16(lib, ctx, rows, k, n, act):
    rng = np.random.default_rng(rows + k)
    x = rng.standard_normal((rows, k)).astype(np.float32)
    W = synth.glorot(rng, (k, n))
    b = rng.uniform(-0.5, 0.5, n).astype(np.float32)
    out = lib.gp_linear_forward(ctx, H.to_dev(x, torch.float32), H.to_dev(W, torch.float32),
                                H.to_dev(b, torch.float32), act, bf16=True).cpu().numpy()
    bt = torch.tensor(b, dtype=F64)
    z = torch.tensor(x, dtype=F64) @ torch.tensor(W, dtype=F64) + bt
    ref = (oblock.act(z) if act else z).numpy()
    assert H.rel_l2(out, ref) < 2e-2
    # exact product of the rounded operands (rounding by the library's round-to-nearest-even cast)
    xr = torch.tensor(x).bfloat16().to(F64)
    Wr = torch.tensor(W).bfloat16().to(F64)
    zr = xr @ Wr + bt
    refr = (oblock.act(zr) if act else zr).numpy()
    assert H.rel_l2(out, refr) < 2e-5


@pytest.fixture(params=[1, 2, 3, 0], ids=["matrix-core triplets", "matrix-core triplets, two-kernel forward",
                                          "matrix-core triplets, y on the vector units", "vector triplets"])
def trip_mode(request, lib, ctx):
    """All forms of the triplet sums of the bf16 block: per centre atom on the matrix cores (forced on: these graphs
    are below the density at which the library picks it by itself), with the forward sum in one pass (y evaluated
    in registers) or as two kernels (per-triplet y buffer), and per edge on the vector units."""
    lib.gp_set_triplet_mfma(ctx, request.param)
    yield request.param
    lib.gp_set_triplet_mfma(ctx, -1)


def test_block_G_bf16_small_dims(lib, ctx):
    w = synth.get_workload("cfg3", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0)
    assert w.dims.dtype == "bf16"
    _parity(lib, ctx, w, 0, 2, synth.cube_positions(30, 6.0, 0.9, seed=1), tol=2e-2)


def test_block_G_bf16_cfg3_shape_one_structure(lib, ctx, trip_mode):
    w = synth.get_workload("cfg3")
    _parity(lib, ctx, w, 1, 1, synth.slab_adsorbate_positions(1, 8, 5, 4, 40, seed=2), tol=2e-2)


def test_block_G_bf16_cfg4_widths_small_graph(lib, ctx, trip_mode):
    w = synth.get_workload("cfg4", cutoff=6.0)
    _parity(lib, ctx, w, 2, 1, synth.box_positions(60, 0.08, 0.9, seed=3), tol=2e-2)


def test_block_G_bf16_narrow_cbf_eight_spherical(lib, ctx, trip_mode):
    # emb_cbf below the 16 rows an edge occupies in a matrix-core tile, num_spherical = 8, trip width 32;
    # capped neighbour lists make some edges one-directional (no row left out of their segments)
    from dataclasses import replace
    w = replace(synth.get_workload("cfg3", emb=64, int_emb=32, emb_rbf=8, emb_cbf=5, emb_bil=16, num_radial=16,
                                   num_spherical=8), max_neighbors=12)
    _parity(lib, ctx, w, 3, 1, synth.slab_adsorbate_positions(2, 4, 4, 3, 10, seed=5), tol=2e-2)


def test_block_G_bf16_dense_box_unequal_shares(lib, ctx, trip_mode):
    # 90 atoms, cutoff 7: in-degrees from about 30 to 90, so the largest atom's rows are cut into two shares of the
    # backward matrix-core kernels while atoms of 57..64 rows stay whole (the larger share)
    from dataclasses import replace
    w = replace(synth.get_workload("cfg3", emb=64, emb_rbf=8, cutoff=7.0), max_neighbors=0)
    _parity(lib, ctx, w, 5, 1, synth.box_positions(90, 0.08, 0.9, seed=6), tol=2e-2)


def test_block_G_bf16_tall_odd_widths(lib, ctx):
    # More than 8192 edges, so that the layers run in the global->LDS GEMM kernels (their tall-matrix condition), at
    # widths that leave partial tiles in every one of them: 96 and 40 output columns in the 128- and 64-wide tiles,
    # contractions of 256, 640 and 1536, one 256-wide column tile for the gated layer with its low-rank factor.
    from dataclasses import replace
    w = replace(synth.get_workload("cfg3", emb=256, int_emb=96, emb_rbf=16, emb_cbf=16, emb_bil=40, num_radial=32,
                                   num_spherical=7, cutoff=5.0), max_neighbors=0)
    pos_gptr = synth.box_positions(330, 0.08, 0.9, seed=9)
    ref = H.oracle_graph(pos_gptr[0], pos_gptr[1], w.dims.cutoff, 0)
    assert len(ref["src"]) > 8192, len(ref["src"])
    _parity(lib, ctx, w, 7, 1, pos_gptr, tol=2e-2)


def test_stack_G_bf16_handoff_between_blocks(lib, ctx):
    # Three bf16 blocks with the messages (and gradients) handed from block to block as bf16 against the same stack with
    # fp32 hand-over.  A block reads its input only as bf16 GEMM operands, so the forward result must be bit-identical;
    # the gradients are rounded once more on their way down and may differ by bf16 rounding noise.
    from paper_2203_09697_amd.binding_g import StackG, gp_block_G_stacks_bf16
    w = synth.get_workload("cfg3", emb=64, emb_rbf=8)
    dims = w.dims
    assert gp_block_G_stacks_bf16(dims)
    pos, gptr = synth.slab_adsorbate_positions(2, 4, 4, 3, 10, seed=4)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), dims.cutoff, w.max_neighbors)
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    E = e["n_edges"]
    W_list = [lib.weights_to_device(synth.weights_G(dims, seed=300 + b)) for b in range(3)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=3)
    res = {}
    for handoff in (False, True):
        stack = StackG(ctx, dims, W_list, t, gb, handoff_bf16=handoff)
        assert stack.half_m == handoff and stack.half_g == handoff
        out = stack.forward(H.to_dev(m, torch.float32)).clone()
        grbf = torch.empty((E, dims.num_radial), dtype=torch.float32, device="cuda:0")
        gm, gW = stack.backward(H.to_dev(gup, torch.float32), grad_rbf=grbf)
        torch.cuda.synchronize()
        res[handoff] = (out.cpu().numpy(), gm.clone().cpu().numpy(), grbf.cpu().numpy(),
                        {k: v.clone().cpu().numpy() for k, v in gW[0].items()})
    assert np.array_equal(res[False][0], res[True][0])
    assert H.rel_l2(res[True][1], res[False][1]) < 1e-2
    assert H.rel_l2(res[True][2], res[False][2]) < 1e-2
    for k in res[False][3]:
        assert H.rel_l2(res[True][3][k], res[False][3][k]) < 1e-2, k


def test_block_G_bf16_symmetric_two_blocks(lib, ctx):
    # two symmetric bf16 blocks: the messages go from the first to the second as bf16, the gradient comes back as fp32
    # (the opposite-edge gather of a symmetric block's backward pass reads fp32)
    from paper_2203_09697_amd.binding_g import StackG
    w = synth.get_workload("cfg3", emb=64, emb_rbf=8, symmetric=True)
    pos_gptr = synth.slab_adsorbate_positions(2, 4, 4, 3, 10, seed=8)
    _parity(lib, ctx, w, 9, 2, pos_gptr, tol=2e-2)
    e, t = lib.build_graph(ctx, H.to_dev(pos_gptr[0], torch.float32), H.to_dev(pos_gptr[1], torch.int32), w.dims.cutoff, w.max_neighbors)
    gb = lib.gp_basis_forward(ctx, w.dims, e, t)
    stack = StackG(ctx, w.dims, [lib.weights_to_device(synth.weights_G(w.dims, seed=b)) for b in range(2)], t, gb)
    assert stack.half_m and not stack.half_g
