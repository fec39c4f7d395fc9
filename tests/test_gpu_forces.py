"""GPU parity: energy head and forces (f = -dE/dx through the Gaussian basis and the angle cosines)
of the variant-G stack against the fp64 oracle, plus the invariants forces must satisfy.

Bar: energy relative error <= 1e-4; forces relative L2 <= 1e-4 (fp32 path) and max-abs error
reported relative to max|f|.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import energy as oenergy
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _force_case(lib, ctx, workload, pos_gptr, seed, n_blocks, hidden):
    from paper_2203_09697_amd.binding_e import ForceModelG
    dims = workload.dims
    pos, gptr = pos_gptr
    ref = H.oracle_graph(pos, gptr, dims.cutoff, workload.max_neighbors)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), dims.cutoff,
                           workload.max_neighbors)
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    E = len(ref["src"])
    W_list = [synth.weights_G(dims, seed=300 + seed + b) for b in range(n_blocks)]
    Wh = synth.weights_head(dims.emb, hidden, seed=seed + 11, bias_scale=0.1)
    m0, _ = synth.edge_embeddings(E, dims.emb, seed=seed + 7)
    gb = lib.gp_basis_forward(ctx, dims, e, t)
    model = ForceModelG(ctx, dims, [lib.weights_to_device(W) for W in W_list], lib.weights_to_device(Wh), hidden, e, t,
                        gb, H.to_dev(gptr, torch.int32))
    energy, forces = model.energy_and_forces(H.to_dev(m0, torch.float32))
    torch.cuda.synchronize()
    E_ref, f_ref = oenergy.forces(oenergy.energy_G, pos, ref["src"], ref["dst"], ref["idx_kj"], ref["idx_ji"],
                                  torch.tensor(m0, dtype=torch.float64), [H.t64(W) for W in W_list], H.t64(Wh), dims)
    return pos, energy.cpu().numpy(), forces.cpu().numpy(), E_ref, f_ref, e


def test_out_edge_lists(lib, ctx):
    from paper_2203_09697_amd.binding_e import gp_edges_by_source
    pos, gptr = synth.slab_adsorbate_positions(2, 4, 3, 3, 7, seed=1)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), 5.0, 9)
    out_ptr, out_list = gp_edges_by_source(ctx, e)
    src = e["src"].cpu().numpy()
    order = np.lexsort((np.arange(len(src)), src))
    assert np.array_equal(out_list.cpu().numpy(), order)
    assert np.array_equal(np.diff(out_ptr.cpu().numpy()), np.bincount(src, minlength=len(pos)))


@pytest.mark.parametrize("seed", [0, 1])
def test_forces_small(lib, ctx, seed):
    w = synth.get_workload("cfg5", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0, dtype="f32")
    pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, synth.cube_positions(30, 6.0, 0.9, seed=seed), seed, 3, 7)
    assert abs(E_gpu.sum() - E_ref) <= 1e-4 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 1e-4, (H.rel_l2(f_gpu, f_ref), np.abs(f_gpu - f_ref).max(), np.abs(f_ref).max())
    scale = np.abs(f_ref).max()
    assert np.abs(f_gpu - f_ref).max() <= 1e-4 * scale
    # net force and net torque vanish (translation / rotation invariance of the energy)
    assert np.abs(f_gpu.sum(axis=0)).max() <= 1e-4 * scale * np.sqrt(len(pos))
    assert np.abs(np.cross(pos.astype(np.float64), f_gpu).sum(axis=0)).max() <= 1e-3 * scale * np.sqrt(len(pos))


def test_forces_two_structures_cfg3_widths(lib, ctx):
    # two structures in one batch, neighbour cap active (one-way edges), configuration-3 widths
    w = synth.get_workload("cfg3", dtype="f32")
    pos_gptr = synth.slab_adsorbate_positions(2, 4, 3, 3, 9, seed=4)
    pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, pos_gptr, 2, 2, 64)
    assert len(E_gpu) == 2
    assert abs(E_gpu.sum() - E_ref) <= 1e-4 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 1e-4, H.rel_l2(f_gpu, f_ref)


@pytest.mark.parametrize("mode", [1, 0], ids=["matrix-core triplets", "vector triplets"])
def test_forces_bf16_cfg3_widths(lib, ctx, mode):
    # bf16 GEMM operands (the precision of configuration 5), two blocks so that the basis gradients of the
    # second block accumulate onto the first; both forms of the triplet kernels.  Bar: the bf16 figure, 2e-2.
    w = synth.get_workload("cfg3")
    assert w.dims.dtype == "bf16"
    lib.gp_set_triplet_mfma(ctx, mode)
    try:
        pos_gptr = synth.slab_adsorbate_positions(2, 4, 3, 3, 9, seed=6)
        pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, pos_gptr, 4, 2, 64)
    finally:
        lib.gp_set_triplet_mfma(ctx, -1)
    assert abs(E_gpu.sum() - E_ref) <= 2e-2 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 2e-2, H.rel_l2(f_gpu, f_ref)


def test_forces_radial_at_target(lib, ctx):
    # the mirrored form: grad of cos(alpha) is produced in ji-major order and permuted; two blocks accumulate
    w = synth.get_workload("cfg5", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0, dtype="f32", radial_at_target=True)
    pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, synth.cube_positions(30, 6.0, 0.9, seed=2), 5, 2, 7)
    assert abs(E_gpu.sum() - E_ref) <= 1e-4 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 1e-4, H.rel_l2(f_gpu, f_ref)
    assert np.abs(f_gpu.sum(axis=0)).max() <= 1e-4 * np.abs(f_ref).max() * np.sqrt(len(pos))


def test_forces_symmetric(lib, ctx):
    w = synth.get_workload("cfg5", emb=32, int_emb=16, emb_rbf=4, emb_cbf=5, emb_bil=12, num_radial=9,
                           num_spherical=4, cutoff=4.0, dtype="f32", symmetric=True)
    pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, synth.cube_positions(30, 6.0, 0.9, seed=3), 6, 2, 7)
    assert abs(E_gpu.sum() - E_ref) <= 1e-4 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 1e-4, H.rel_l2(f_gpu, f_ref)


# ---- graphs whose atoms need several shares of the per-centre-atom kernels -------------------------
def _dense_box():
    # 90 atoms, cutoff 7: in-degrees from about 30 to 90; the backward matrix-core kernels cut the rows of an atom
    # into shares of 64, the forward ones its out-edges into shares of 32, so most atoms span 2-3 shares
    from dataclasses import replace
    return replace(synth.get_workload("cfg3", emb=64, emb_rbf=8, cutoff=7.0), max_neighbors=0), synth.box_positions(90, 0.08, 0.9, seed=6)


@pytest.mark.parametrize("mode", [1, 0], ids=["matrix-core triplets", "vector triplets"])
def test_forces_dense_box_bf16_several_shares(lib, ctx, mode):
    w, pos_gptr = _dense_box()
    lib.gp_set_triplet_mfma(ctx, mode)
    try:
        pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, pos_gptr, 8, 2, 32)
    finally:
        lib.gp_set_triplet_mfma(ctx, -1)
    deg = np.diff(e["row_ptr"].cpu().numpy())
    assert deg.max() > 64 and deg.min() < 64
    assert abs(E_gpu.sum() - E_ref) <= 2e-2 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 2e-2, H.rel_l2(f_gpu, f_ref)
    assert H.row_err(f_gpu, f_ref) <= 4 * 2e-2, H.row_err(f_gpu, f_ref)


def test_forces_dense_box_fp32(lib, ctx):
    from dataclasses import replace
    w, pos_gptr = _dense_box()
    w = replace(w, dims=replace(w.dims, dtype="f32"))
    pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, pos_gptr, 8, 2, 32)
    assert abs(E_gpu.sum() - E_ref) <= 1e-4 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 1e-4, H.rel_l2(f_gpu, f_ref)
    assert H.row_err(f_gpu, f_ref) <= 4e-4, H.row_err(f_gpu, f_ref)


@pytest.mark.timeout(900)
def test_forces_cfg5_model_on_a_box_the_oracle_can_follow(lib, ctx):
    """The whole force-training model of configuration 5 (3 bilinear blocks at its widths, bf16 GEMM operands, energy
    head of width 256, forces) on a box of the same density and cutoff that is small enough for the full oracle
    (which keeps every triplet's outer product for its reverse pass, 16 KB per triplet and block): 80 atoms,
    in-degrees up to 79, so two or three shares per atom in every per-centre-atom kernel.  The matrix-core triplet
    kernels are forced on, as the library picks them at full size (this box has 78 triplets per edge, below the
    96 from which it would choose them by itself)."""
    w = synth.get_workload("cfg5")
    pos_gptr = synth.box_positions(80, 0.08, 0.9, seed=2)
    lib.gp_set_triplet_mfma(ctx, 1)
    try:
        pos, E_gpu, f_gpu, E_ref, f_ref, e = _force_case(lib, ctx, w, pos_gptr, 0, w.n_blocks, w.head_hidden)
    finally:
        lib.gp_set_triplet_mfma(ctx, -1)
    deg = np.diff(e["row_ptr"].cpu().numpy())
    assert deg.max() > 64
    err = np.abs(f_gpu - f_ref).max()
    print("cfg5 model, 80-atom box: E=%d  max|f|=%.4e  max-abs force error=%.3e  rel-L2=%.2e" % (
        len(e["src"]), np.abs(f_ref).max(), err, H.rel_l2(f_gpu, f_ref)))
    assert abs(E_gpu.sum() - E_ref) <= 2e-2 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 2e-2, H.rel_l2(f_gpu, f_ref)
    assert err <= 4 * 2e-2 * np.abs(f_ref).max()


@pytest.mark.parametrize("triplet_mode", [-1, 0], ids=["library's choice of triplet kernels", "per-edge triplet kernels"])
def test_forces_variant_D(lib, ctx, triplet_mode):
    """Forces of the Hadamard (DimeNet++-style, energy-centric) model, Sec. 3.2/3.3: two blocks + head on two capped
    structures at configuration 2's widths, against automatic differentiation of the oracle's energy through the Bessel
    radial basis, the spherical basis and cos(alpha)."""
    from paper_2203_09697_amd.binding_e import ForceModelD
    w = synth.get_workload("cfg2")
    dims = w.dims
    pos, gptr = synth.slab_adsorbate_positions(2, 3, 3, 3, 8, seed=21)
    ref = H.oracle_graph(pos, gptr, dims.cutoff, w.max_neighbors)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), dims.cutoff, w.max_neighbors)
    assert np.array_equal(t["idx_kj"].cpu().numpy(), ref["idx_kj"])
    E, hidden = len(ref["src"]), 16
    W_list = [synth.weights_D(dims, seed=400 + b, bias_scale=0.1) for b in range(2)]
    Wh = synth.weights_head(dims.emb, hidden, seed=5, bias_scale=0.1)
    m0, _ = synth.edge_embeddings(E, dims.emb, seed=9)
    lib.gp_set_triplet_mfma(ctx, triplet_mode)
    try:
        gb = lib.gp_basis_forward(ctx, dims, e, t)
        model = ForceModelD(ctx, dims, [lib.weights_to_device(W) for W in W_list], lib.weights_to_device(Wh), hidden, e, t, gb,
                            H.to_dev(gptr, torch.int32))
        energy, forces = model.energy_and_forces(H.to_dev(m0, torch.float32))
        torch.cuda.synchronize()
    finally:
        lib.gp_set_triplet_mfma(ctx, -1)
    E_ref, f_ref = oenergy.forces(oenergy.energy_D, pos, ref["src"], ref["dst"], ref["idx_kj"], ref["idx_ji"],
                                  torch.tensor(m0, dtype=torch.float64), [H.t64(W) for W in W_list], H.t64(Wh), dims)
    f_gpu = forces.cpu().numpy()
    scale = np.abs(f_ref).max()
    print("variant D forces: E=%d max|f|=%.4e max-abs error=%.3e rel-L2=%.2e" % (E, scale, np.abs(f_gpu - f_ref).max(), H.rel_l2(f_gpu, f_ref)))
    assert abs(energy.cpu().numpy().sum() - E_ref) <= 1e-4 * max(1.0, abs(E_ref))
    assert H.rel_l2(f_gpu, f_ref) <= 1e-4
    assert np.abs(f_gpu - f_ref).max() <= 2e-4 * scale
    assert np.abs(f_gpu.sum(axis=0)).max() <= 1e-4 * scale * np.sqrt(len(pos))
