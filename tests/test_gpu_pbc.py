"""GPU parity for periodic structures: edge list with cell offsets and image-aware triplets bit-exact
against the oracle; geometry, a variant-D block, a variant-G block (matrix-core triplet kernels forced
on) and forces on a periodic graph against the fp64 oracle.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import basis as obasis
from oracle import energy as oenergy
from oracle import graph as ograph
from tests import helpers as H

pytestmark = pytest.mark.gpu
F64 = torch.float64


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _structures(seed, sizes=(9, 6), a=(4.2, 3.7)):
    """Two periodic structures with different triclinic cells; atoms at least 0.9 apart (minimum image)."""
    rng = np.random.default_rng(seed)
    pos, cells, gptr = [], [], [0]
    for n, a0 in zip(sizes, a):
        cell = np.array([[a0, 0.0, 0.0], [0.25 * a0 * rng.uniform(-1, 1), 1.1 * a0, 0.0],
                         [0.1, -0.3, 0.95 * a0]], dtype=np.float32)
        pts = []
        while len(pts) < n:
            p = rng.uniform(0, 1, 3) @ cell.astype(np.float64)
            ok = True
            for q in pts:
                for im in np.ndindex(3, 3, 3):
                    if np.linalg.norm(p - q - (np.array(im) - 1) @ cell.astype(np.float64)) < 0.9:
                        ok = False
            if ok:
                pts.append(p)
        pos.append(np.array(pts))
        cells.append(cell)
        gptr.append(gptr[-1] + n)
    return np.concatenate(pos).astype(np.float32), np.array(gptr, dtype=np.int32), np.stack(cells)


def _build(lib, ctx, pos, gptr, cells, cutoff, rep, cap=0):
    return lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), cutoff, cap,
                           cell=H.to_dev(cells, torch.float32), rep=rep)


@pytest.mark.parametrize("cutoff,rep,cap", [(3.0, (1, 1, 1), 0), (4.4, (2, 2, 2), 0), (4.4, (2, 2, 2), 10), (3.5, (1, 2, 1), 5)])
def test_periodic_graph_bit_exact(lib, ctx, cutoff, rep, cap):
    pos, gptr, cells = _structures(1)
    s, d, o, rp = ograph.edges_pbc(pos, gptr, cells, cutoff, rep, cap)
    kj, ji, seg = ograph.triplets(s, d, rp, o)
    e, t = _build(lib, ctx, pos, gptr, cells, cutoff, rep, cap)
    assert np.array_equal(e["src"].cpu().numpy(), s) and np.array_equal(e["dst"].cpu().numpy(), d)
    assert np.array_equal(e["offset"].cpu().numpy(), o) and np.array_equal(e["row_ptr"].cpu().numpy(), rp)
    assert np.array_equal(t["idx_kj"].cpu().numpy(), kj) and np.array_equal(t["idx_ji"].cpu().numpy(), ji)
    assert np.array_equal(t["seg_ptr_ji"].cpu().numpy(), seg)
    # kj-major view: a permutation of the triplets sorted by (idx_kj, idx_ji)
    order = np.lexsort((ji, kj))
    assert np.array_equal(t["perm_kj"].cpu().numpy(), order)
    assert np.array_equal(t["idx_ji_kj"].cpu().numpy(), ji[order])
    assert np.array_equal(t["id_swap"].cpu().numpy(), ograph.reverse_edges(s, d, o))
    # geometry of the shifted sources
    shift = ograph.edge_shifts(o, d, gptr, cells)
    dd, unit, ca = obasis.geometry(torch.tensor(pos, dtype=F64), s, d, kj, ji, shift)
    assert np.abs(e["dist"].cpu().numpy() - dd.numpy()).max() < 1e-5
    assert np.abs(e["unit"].cpu().numpy() - unit.numpy()).max() < 1e-5


def test_no_image_in_range_reproduces_open_boundaries(lib, ctx):
    pos, gptr, cells = _structures(2)
    e0, t0 = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), 3.0, 0)
    e1, t1 = _build(lib, ctx, pos, gptr, cells * 40.0, 3.0, (1, 1, 1))
    for k in ("src", "dst", "row_ptr", "dist", "unit"):
        assert torch.equal(e0[k], e1[k]), k
    assert not e1["offset"].any()
    for k in ("idx_kj", "idx_ji", "seg_ptr_ji", "perm_kj", "idx_ji_kj", "seg_ptr_kj", "id_swap"):
        assert torch.equal(t0[k], t1[k]), k


def _oracle_graph(pos, gptr, cells, cutoff, rep, cap=0):
    s, d, o, rp = ograph.edges_pbc(pos, gptr, cells, cutoff, rep, cap)
    kj, ji, seg = ograph.triplets(s, d, rp, o)
    return dict(src=s, dst=d, offset=o, row_ptr=rp, idx_kj=kj, idx_ji=ji, seg=seg, shift=ograph.edge_shifts(o, d, gptr, cells))


def test_block_D_on_a_periodic_graph(lib, ctx):
    from paper_2203_09697_amd.stack import StackD
    w = synth.get_workload("cfg1", cutoff=3.6)
    dims = w.dims
    pos, gptr, cells = _structures(3)
    ref = _oracle_graph(pos, gptr, cells, dims.cutoff, (1, 1, 1))
    e, t = _build(lib, ctx, pos, gptr, cells, dims.cutoff, (1, 1, 1))
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    E = len(ref["src"])
    pos64 = torch.tensor(pos, dtype=F64)
    d, unit, ca = obasis.geometry(pos64, ref["src"], ref["dst"], ref["idx_kj"], ref["idx_ji"], ref["shift"])
    ob = dict(rbf=obasis.rbf_bessel(d, dims.cutoff, dims.num_radial, dims.envelope_p),
              sbf=obasis.sbf(d, ca, ref["idx_kj"], dims.cutoff, dims.num_spherical, dims.num_radial, dims.envelope_p))
    W_list = [synth.weights_D(dims, seed=60 + b, bias_scale=0.1) for b in range(2)]
    m, gup = synth.edge_embeddings(E, dims.emb, seed=8)
    out_ref, gm_ref, gW_ref = H.oracle_stack_D(ref, ob, dims, W_list, m, gup)
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    assert np.abs(gb["cos_alpha"].cpu().numpy() - ca.numpy()).max() < 1e-5
    stack = StackD(ctx, dims, [lib.weights_to_device(W) for W in W_list], t, gb)
    out = stack.forward(H.to_dev(m, torch.float32))
    gm, gW = stack.backward(H.to_dev(gup, torch.float32))
    torch.cuda.synchronize()
    errs = {"m_out": H.rel_l2(out.cpu().numpy(), out_ref), "grad_m": H.rel_l2(gm.cpu().numpy(), gm_ref)}
    for b in range(2):
        for k in gW_ref[b]:
            errs[f"block{b}.{k}"] = H.rel_l2(gW[b][k].cpu().numpy(), gW_ref[b][k])
    bad = {k: v for k, v in errs.items() if not v <= 1e-4}
    assert not bad, bad


@pytest.mark.parametrize("dtype,tol,mfma", [("f32", 1e-4, -1), ("bf16", 2e-2, 1)])
def test_forces_G_on_a_periodic_graph(lib, ctx, dtype, tol, mfma):
    # variant G + energy head on a periodic graph; with bf16 the per-centre-atom matrix-core kernels are forced on
    from paper_2203_09697_amd.binding_e import ForceModelG
    w = synth.get_workload("cfg5", emb=64, int_emb=32, emb_rbf=8, emb_cbf=16, emb_bil=32, num_radial=16,
                           num_spherical=7, cutoff=3.8, dtype=dtype)
    dims = w.dims
    pos, gptr, cells = _structures(4)
    ref = _oracle_graph(pos, gptr, cells, dims.cutoff, (1, 1, 1))
    e, t = _build(lib, ctx, pos, gptr, cells, dims.cutoff, (1, 1, 1))
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    E = len(ref["src"])
    W_list = [synth.weights_G(dims, seed=70 + b) for b in range(2)]
    Wh = synth.weights_head(dims.emb, 16, seed=9, bias_scale=0.1)
    m0, _ = synth.edge_embeddings(E, dims.emb, seed=10)
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    lib.gp_set_triplet_mfma(ctx, mfma)
    try:
        model = ForceModelG(ctx, dims, [lib.weights_to_device(W) for W in W_list], lib.weights_to_device(Wh), 16, e, t, gb,
                            H.to_dev(gptr, torch.int32))
        energy, forces = model.energy_and_forces(H.to_dev(m0, torch.float32))
        torch.cuda.synchronize()
    finally:
        lib.gp_set_triplet_mfma(ctx, -1)
    E_ref, f_ref = oenergy.forces(oenergy.energy_G, pos, ref["src"], ref["dst"], ref["idx_kj"], ref["idx_ji"],
                                  torch.tensor(m0, dtype=F64), [H.t64(W) for W in W_list], H.t64(Wh), dims, ref["shift"])
    assert abs(float(energy.sum()) - E_ref) <= tol * max(1.0, abs(E_ref))
    assert H.rel_l2(forces.cpu().numpy(), f_ref) <= tol, H.rel_l2(forces.cpu().numpy(), f_ref)
    # a rigid translation leaves a periodic structure's energy unchanged: forces sum to zero per structure
    f = forces.cpu().numpy()
    for g in range(len(gptr) - 1):
        assert np.abs(f[gptr[g]:gptr[g + 1]].sum(axis=0)).max() <= 50 * tol * np.abs(f_ref).max()
