"""GPU parity: basis functions, dense layer, TripletUpdate/TripletAggr kernels and the whole
variant-D interaction block (forward and backward) against the fp64 oracle.

Tolerance: relative L2 error <= 1e-4 per tensor (fp32 path), as the target states.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import block as oblock
from tests import helpers as H

pytestmark = pytest.mark.gpu
TOL = 1e-4
F64 = torch.float64


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _case(lib, ctx, workload, seed, pos_gptr=None):
    pos, gptr = pos_gptr if pos_gptr is not None else synth.make_positions(workload, seed)
    dims = workload.dims
    ref = H.oracle_graph(pos, gptr, dims.cutoff, workload.max_neighbors)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), dims.cutoff,
                           workload.max_neighbors)
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    return pos, ref, e, t


@pytest.mark.parametrize("name,seed", [("cfg1", 0), ("cfg1", 1)])
def test_basis_D(lib, ctx, name, seed):
    w = synth.get_workload(name)
    pos, ref, e, t = _case(lib, ctx, w, seed)
    ob = H.oracle_basis_D(pos, ref, w.dims)
    gb = lib.gp_basis_forward(ctx, w.dims, e, t, want_sbf=True)
    torch.cuda.synchronize()
    assert H.rel_l2(gb["rbf"].cpu().numpy(), ob["rbf"].numpy()) < 1e-5
    assert H.rel_l2(gb["rad"].cpu().numpy(), ob["rad"].numpy()) < 1e-5
    assert np.abs(gb["cos_alpha"].cpu().numpy() - ob["cos_alpha"].numpy()).max() < 1e-5
    assert H.rel_l2(gb["sbf"].cpu().numpy(), ob["sbf"].numpy()) < 1e-5
    perm = t["perm_kj"].cpu().numpy()
    assert np.array_equal(gb["cos_alpha_kj"].cpu().numpy(), gb["cos_alpha"].cpu().numpy()[perm])


def test_basis_D_large_cutoff_small_arguments(lib, ctx):
    # small d/c makes the Bessel arguments fall below the order l (series branch)
    w = synth.get_workload("cfg1", cutoff=12.0)
    pos, ref, e, t = _case(lib, ctx, w, 3)
    ob = H.oracle_basis_D(pos, ref, w.dims)
    gb = lib.gp_basis_forward(ctx, w.dims, e, t)
    rad_g, rad_o = gb["rad"].cpu().numpy(), ob["rad"].numpy()
    assert H.rel_l2(rad_g, rad_o) < 1e-5
    # column-wise too: the high-l columns are tiny and must not be swamped
    for col in range(rad_o.shape[1]):
        assert H.rel_l2(rad_g[:, col], rad_o[:, col]) < 1e-4, col


@pytest.fixture(params=[1, 0], ids=["fp32 as three bf16 planes", "fp32 matrix-core instruction"])
def f32_gemm(lib, ctx, request):
    lib.gp_set_f32_gemm(ctx, request.param)
    yield request.param
    lib.gp_set_f32_gemm(ctx, 1)


@pytest.mark.parametrize("rows,k,n,act", [(1, 4, 4, 0), (37, 32, 16, 1), (300, 6, 32, 0), (1000, 256, 256, 1),
                                            (513, 64, 256, 1), (2049, 256, 64, 0), (129, 42, 8, 0), (5, 7, 3, 1),
                                            (16400, 72, 2048, 1)])   # the last: enough tiles for the 128 x 128 form
def test_linear_forward(lib, ctx, rows, k, n, act, f32_gemm):
    rng = np.random.default_rng(rows + k)
    x = rng.standard_normal((rows, k)).astype(np.float32)
    W = synth.glorot(rng, (k, n))
    b = rng.uniform(-0.5, 0.5, n).astype(np.float32)
    out = lib.gp_linear_forward(ctx, H.to_dev(x, torch.float32), H.to_dev(W, torch.float32),
                                H.to_dev(b, torch.float32), act)
    z = torch.tensor(x, dtype=F64) @ torch.tensor(W, dtype=F64) + torch.tensor(b, dtype=F64)
    ref = oblock.act(z) if act else z
    assert H.rel_l2(out.cpu().numpy(), ref.numpy()) < 1e-5


def test_split_gemm_is_as_exact_as_fp32(lib, ctx):
    # Operands with 24 significant bits and a wide range of magnitudes: the product through three bf16 planes per
    # operand must sit as close to the fp64 product as the one the fp32-operand instruction gives (both accumulate
    # in fp32), far below what a single bf16 plane would give (about 4e-3).
    rng = np.random.default_rng(11)
    rows, k, n = 4099, 1000, 264
    x = (rng.standard_normal((rows, k)) * np.exp(rng.uniform(-6, 6, (rows, 1)))).astype(np.float32)
    W = (rng.standard_normal((k, n)) * np.exp(rng.uniform(-3, 3, (1, n)))).astype(np.float32)
    b = np.zeros(n, np.float32)
    ref = (torch.tensor(x, dtype=F64) @ torch.tensor(W, dtype=F64)).numpy()
    err = {}
    for mode in (1, 0):
        lib.gp_set_f32_gemm(ctx, mode)
        out = lib.gp_linear_forward(ctx, H.to_dev(x, torch.float32), H.to_dev(W, torch.float32), H.to_dev(b, torch.float32), 0)
        err[mode] = H.rel_l2(out.cpu().numpy(), ref)
    lib.gp_set_f32_gemm(ctx, 1)
    print("fp32 GEMM rel-L2 against fp64: three bf16 planes %.3e, fp32 instruction %.3e" % (err[1], err[0]))
    assert err[0] < 1e-6 and err[1] < 1e-6
    assert err[1] < 2.0 * err[0] + 1e-7


@pytest.mark.parametrize("width", [3, 16, 32, 64, 128, 200])
def test_streaming_triplet_kernels(lib, ctx, width):
    pos, gptr = synth.cube_positions(40, 7.0, 0.9, seed=width)
    g = H.oracle_graph(pos, gptr, 4.0, 0)
    E, T = len(g["src"]), len(g["idx_kj"])
    assert T > 1000 and np.diff(g["seg"]).max() > 8
    rng = np.random.default_rng(width)
    x = rng.standard_normal((E, width)).astype(np.float32)
    s = rng.standard_normal((T, width)).astype(np.float32)
    ga = rng.standard_normal((E, width)).astype(np.float32)
    dg = H.graph_from_oracle(g)
    a = lib.gp_triplet_aggregate_fwd(ctx, dg, H.to_dev(x, torch.float32), H.to_dev(s, torch.float32))
    xt = torch.tensor(x, dtype=F64, requires_grad=True)
    st = torch.tensor(s, dtype=F64, requires_grad=True)
    ref = oblock.triplet_aggregate_D(xt, st, g["idx_kj"], g["idx_ji"], E)
    assert H.rel_l2(a.cpu().numpy(), ref.detach().numpy()) < 1e-6
    gx_ref, gs_ref = torch.autograd.grad((ref * torch.tensor(ga, dtype=F64)).sum(), [xt, st])
    gx, gs = lib.gp_triplet_aggregate_bwd(ctx, dg, H.to_dev(x, torch.float32), H.to_dev(s, torch.float32),
                                          H.to_dev(ga, torch.float32))
    assert H.rel_l2(gx.cpu().numpy(), gx_ref.numpy()) < 1e-6
    assert H.rel_l2(gs.cpu().numpy(), gs_ref.numpy()) < 1e-6
    # sorted-segment reductions are bit-reproducible
    a2 = lib.gp_triplet_aggregate_fwd(ctx, dg, H.to_dev(x, torch.float32), H.to_dev(s, torch.float32))
    assert torch.equal(a, a2)


def test_partition_property_on_gpu(lib, ctx):
    # Sec. 2.2: aggregates of triplet subsets (one per processing unit) add up to the full aggregate
    pos, gptr = synth.cube_positions(40, 7.0, 0.9, seed=9)
    g = H.oracle_graph(pos, gptr, 4.0, 0)
    E, T = len(g["src"]), len(g["idx_kj"])
    rng = np.random.default_rng(0)
    x = H.to_dev(rng.standard_normal((E, 64)), torch.float32)
    s = rng.standard_normal((T, 64)).astype(np.float32)
    full = lib.gp_triplet_aggregate_fwd(ctx, H.graph_from_oracle(g), x, H.to_dev(s, torch.float32))
    owner = rng.integers(0, 3, size=T)
    total = torch.zeros_like(full)
    for p in range(3):
        sel = owner == p
        seg = np.zeros(E + 1, dtype=np.int64)
        np.add.at(seg, g["idx_ji"][sel].astype(np.int64) + 1, 1)
        sub = dict(src=g["src"], idx_kj=g["idx_kj"][sel], idx_ji=g["idx_ji"][sel], seg=np.cumsum(seg))
        total += lib.gp_triplet_aggregate_fwd(ctx, H.graph_from_oracle(sub), x, H.to_dev(s[sel], torch.float32))
    assert H.rel_l2(total.cpu().numpy(), full.cpu().numpy()) < 1e-6


def _block_parity(lib, ctx, workload, seed, n_blocks, pos_gptr=None, bias_scale=0.1):
    from paper_2203_09697_amd.stack import StackD
    dims = workload.dims
    pos, ref, e, t = _case(lib, ctx, workload, seed, pos_gptr)
    E = len(ref["src"])
    W_list = [synth.weights_D(dims, seed=100 + seed + b, bias_scale=bias_scale) for b in range(n_blocks)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=seed + 7)
    ob = H.oracle_basis_D(pos, ref, dims)
    out_ref, gm_ref, gW_ref = H.oracle_stack_D(ref, ob, dims, W_list, m, gup)
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    stack = StackD(ctx, dims, [lib.weights_to_device(W) for W in W_list], t, gb)
    out = stack.forward(H.to_dev(m, torch.float32))
    gm, gW = stack.backward(H.to_dev(gup, torch.float32))
    torch.cuda.synchronize()
    errs = {"m_out": H.rel_l2(out.cpu().numpy(), out_ref), "grad_m": H.rel_l2(gm.cpu().numpy(), gm_ref)}
    for b in range(n_blocks):
        for k in gW_ref[b]:
            errs[f"block{b}.{k}"] = H.rel_l2(gW[b][k].cpu().numpy(), gW_ref[b][k])
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
    return errs


@pytest.mark.parametrize("seed", [0, 1])
def test_block_D_cfg1(lib, ctx, seed):
    _block_parity(lib, ctx, synth.get_workload("cfg1"), seed, n_blocks=1)


def test_block_D_cfg1_two_blocks_zero_bias(lib, ctx):
    _block_parity(lib, ctx, synth.get_workload("cfg1"), 2, n_blocks=2, bias_scale=0.0)


@pytest.fixture
def triplet_form(lib, ctx, request):
    # 0: per-edge vector kernels, -1: the library's choice (matrix-core kernels where the widths allow)
    lib.gp_set_triplet_mfma(ctx, request.param)
    yield request.param
    lib.gp_set_triplet_mfma(ctx, -1)


def test_block_D_cfg2_shape_fp32_instruction(lib, ctx):
    # the same block with its GEMMs on the fp32-operand matrix-core instruction (not the default)
    lib.gp_set_f32_gemm(ctx, 0)
    try:
        w = synth.get_workload("cfg2")
        _block_parity(lib, ctx, w, 5, n_blocks=2, pos_gptr=synth.slab_adsorbate_positions(2, 4, 4, 4, 16, seed=5))
    finally:
        lib.gp_set_f32_gemm(ctx, 1)


@pytest.mark.parametrize("triplet_form", [-1, 0], indirect=True)
def test_block_D_cfg2_shape_two_graphs(lib, ctx, triplet_form):
    # configuration-2 layer widths and neighbour cap on 2 of its 16 structures (oracle in seconds)
    w = synth.get_workload("cfg2")
    pos_gptr = synth.slab_adsorbate_positions(2, 4, 4, 4, 16, seed=5)
    _block_parity(lib, ctx, w, 5, n_blocks=2, pos_gptr=pos_gptr)


@pytest.mark.parametrize("int_emb,num_spherical", [(32, 7), (96, 8), (128, 3), (64, 1)])
def test_block_D_matrix_core_widths(lib, ctx, int_emb, num_spherical):
    # every column-block count of the per-centre-atom fp32 matrix-core kernels (basis_emb 8), with fewer and with
    # all 8 spherical orders, on one capped structure
    w = synth.get_workload("cfg2", emb=64, int_emb=int_emb, num_spherical=num_spherical, n_res_before=1, n_res_after=1)
    pos_gptr = synth.slab_adsorbate_positions(1, 4, 4, 4, 16, seed=9)
    _block_parity(lib, ctx, w, 6, n_blocks=1, pos_gptr=pos_gptr)


@pytest.mark.parametrize("triplet_form", [-1, 0], indirect=True)
def test_block_D_basis_gradients(lib, ctx, triplet_form):
    """Gradients with respect to the radial basis, the radial part of the spherical basis and cos(alpha) of a two-block
    stack (the second block overwrites, the first adds) against autograd of the oracle, in which the per-triplet
    spherical basis is the product rad[kj] * Y_l0(cos alpha) of the two leaves."""
    from oracle import basis as obasis
    from paper_2203_09697_amd.stack import StackD
    w = synth.get_workload("cfg2")
    dims = w.dims
    pos, ref, e, t = _case(lib, ctx, w, 5, synth.slab_adsorbate_positions(2, 4, 4, 4, 16, seed=5))
    E, T = len(ref["src"]), len(ref["idx_kj"])
    W_list = [synth.weights_D(dims, seed=200 + b, bias_scale=0.1) for b in range(2)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=12)
    ob = H.oracle_basis_D(pos, ref, dims)
    rbf = ob["rbf"].detach().clone().requires_grad_(True)
    rad = ob["rad"].detach().clone().requires_grad_(True)                 # [E, S * R]
    ca = ob["cos_alpha"].detach().clone().requires_grad_(True)
    kj = torch.as_tensor(ref["idx_kj"], dtype=torch.long)
    S, R = dims.num_spherical, dims.num_radial
    sbf = (rad.reshape(E, S, R)[kj] * obasis.y_l0(ca, S)[:, :, None]).reshape(T, S * R)
    out = oblock.stack_D(torch.tensor(m, dtype=F64), rbf, sbf, ref["idx_kj"], ref["idx_ji"], [H.t64(W) for W in W_list],
                         dims.n_res_before, dims.n_res_after)
    g_rbf, g_rad, g_ca = torch.autograd.grad((out * torch.tensor(gup, dtype=F64)).sum(), [rbf, rad, ca])
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    stack = StackD(ctx, dims, [lib.weights_to_device(W) for W in W_list], t, gb)
    stack.forward(H.to_dev(m, torch.float32))
    bg = {"grad_rbf": torch.full((E, R), 7.0, dtype=torch.float32, device="cuda:0"),      # must be overwritten
          "grad_rad": torch.full((E, S * R), 7.0, dtype=torch.float32, device="cuda:0"),
          "grad_cos_kj": torch.full((T,), 7.0, dtype=torch.float32, device="cuda:0")}
    stack.backward(H.to_dev(gup, torch.float32), basis_grads=bg)
    torch.cuda.synchronize()
    order = t["perm_kj"].cpu().numpy()
    errs = {"grad_rbf": H.rel_l2(bg["grad_rbf"].cpu().numpy(), g_rbf.numpy()),
            "grad_rad": H.rel_l2(bg["grad_rad"].cpu().numpy(), g_rad.numpy()),
            "grad_cos_kj": H.rel_l2(bg["grad_cos_kj"].cpu().numpy(), g_ca.numpy()[order])}
    print(errs)
    assert all(v <= TOL for v in errs.values()), errs
    assert g_ca.abs().max() > 1e-8 and g_rad.abs().max() > 1e-8


@pytest.mark.timeout(600)
def test_block_D_xl_widths_small_structure(lib, ctx):
    # the widest DimeNet++ the paper trains (Sec. 4.1: hidden width 2048, triplet width 256) on a structure small
    # enough for the oracle; int_emb 256 is beyond the matrix-core triplet kernels (128) and runs the per-edge form
    w = synth.get_workload("xl")
    assert w.dims.emb == 2048 and w.dims.int_emb == 256
    pos_gptr = synth.slab_adsorbate_positions(1, 3, 3, 3, 6, seed=11)
    _block_parity(lib, ctx, w, 8, n_blocks=1, pos_gptr=pos_gptr)


def test_block_D_odd_widths(lib, ctx):
    # widths that are not multiples of the tile sizes or of 4: exercises every ragged path
    w = synth.get_workload("cfg1", emb=36, int_emb=20, basis_emb=3, num_radial=5, num_spherical=4,
                           n_res_before=2, n_res_after=1)
    _block_parity(lib, ctx, w, 4, n_blocks=1)


@pytest.mark.parametrize("f32_gemm", [1, 0], indirect=True, ids=["fp32 as three bf16 planes", "fp32 matrix-core instruction"])
def test_block_D_partial_tiles(lib, ctx, f32_gemm):
    # widths that are multiples of 4 (16-byte rows: the vector loaders and the three-plane weight-gradient kernel) but of
    # no tile size: 200 and 72 columns in 128-, 64- and 32-wide tiles, contractions of 200, 72, 12 with a partial last slab
    w = synth.get_workload("cfg1", emb=200, int_emb=72, basis_emb=8, num_radial=12, num_spherical=5,
                           n_res_before=1, n_res_after=1)
    _block_parity(lib, ctx, w, 6, n_blocks=1)


def test_block_D_deterministic(lib, ctx):
    from paper_2203_09697_amd.stack import StackD
    w = synth.get_workload("cfg1")
    pos, ref, e, t = _case(lib, ctx, w, 0)
    W = lib.weights_to_device(synth.weights_D(w.dims, seed=1, bias_scale=0.1))
    m, gup = synth.edge_embeddings(len(ref["src"]), w.dims.emb, seed=2)
    gb = lib.gp_basis_forward(ctx, w.dims, e, t)
    st = StackD(ctx, w.dims, [W], t, gb)
    o1 = st.forward(H.to_dev(m, torch.float32)).clone()
    g1, gw1 = st.backward(H.to_dev(gup, torch.float32))
    g1 = g1.clone(); gw1 = {k: v.clone() for k, v in gw1[0].items()}
    o2 = st.forward(H.to_dev(m, torch.float32))
    g2, gw2 = st.backward(H.to_dev(gup, torch.float32))
    assert torch.equal(o1, o2) and torch.equal(g1, g2)
    assert all(torch.equal(gw1[k], gw2[0][k]) for k in gw1)


def test_block_D_two_streams_match_one_stream(lib, ctx):
    # With the side stream on, graphs of 2048 edges or more run the layers after the triplet sum as two row halves on
    # two streams and parts of the backward pass beside the main chain; the forward is the same arithmetic per row,
    # so it must agree bit for bit with the single-stream run, and the gradients (one sum taken in another order) closely.
    from paper_2203_09697_amd.stack import StackD
    w = synth.get_workload("cfg2")
    pos, ref, e, t = _case(lib, ctx, w, 5, synth.slab_adsorbate_positions(2, 4, 4, 4, 16, seed=5))
    E = len(ref["src"])
    assert E >= 2048
    W = [lib.weights_to_device(synth.weights_D(w.dims, seed=31 + b, bias_scale=0.1)) for b in range(2)]
    m, gup = synth.edge_embeddings(E, w.dims.emb, seed=8)
    gb = lib.gp_basis_forward(ctx, w.dims, e, t)
    res = []
    try:
        for on in (True, False):
            lib.gp_set_side_stream(ctx, on)
            st = StackD(ctx, w.dims, W, t, gb)
            out = st.forward(H.to_dev(m, torch.float32)).clone()
            gm, gw = st.backward(H.to_dev(gup, torch.float32))
            torch.cuda.synchronize()
            res.append((out, gm.clone(), [{k: v.clone() for k, v in g.items()} for g in gw]))
    finally:
        lib.gp_set_side_stream(ctx, True)
    (o2, g2, w2), (o1, g1, w1) = res
    assert torch.equal(o2, o1)
    assert H.rel_l2(g2.cpu().numpy(), g1.cpu().numpy()) < 1e-6
    for b in range(2):
        for k in w1[b]:
            assert H.rel_l2(w2[b][k].cpu().numpy(), w1[b][k].cpu().numpy()) < 1e-6, (b, k)
