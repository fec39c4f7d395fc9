"""GPU parity: the output block (per-atom sum of radially weighted messages + node MLP) alone and
behind a variant-D block stack, forward and backward, against the fp64 oracle.

Tolerance: relative L2 error <= 1e-4 per tensor (fp32 path).
"""
import numpy as np
import pytest
import torch

import synth
from oracle import output as ooutput
from tests import helpers as H

pytestmark = pytest.mark.gpu
TOL = 1e-4
F64 = torch.float64


@pytest.fixture(scope="module")
def ctx(lib):
    return lib.Context(0)


def _graph(lib, ctx, pos, gptr, cutoff, cap):
    ref = H.oracle_graph(pos, gptr, cutoff, cap)
    e, t = lib.build_graph(ctx, H.to_dev(pos, torch.float32), H.to_dev(gptr, torch.int32), cutoff, cap)
    assert np.array_equal(e["dst"].cpu().numpy(), ref["dst"])
    return ref, e, t


def _oracle_out(m, rbf, dst, gptr, n_atoms, W, coef):
    Wt = {k: v.clone().requires_grad_(True) for k, v in H.t64(W).items()}
    mt = torch.tensor(m, dtype=F64, requires_grad=True)
    E = ooutput.structure_energies(ooutput.output_block(mt, torch.tensor(rbf, dtype=F64), dst, n_atoms, Wt), gptr)
    grads = torch.autograd.grad((E * torch.tensor(coef, dtype=F64)).sum(), [mt] + list(Wt.values()))
    return E.detach().numpy(), grads[0].numpy(), {k: grads[1 + i].numpy() for i, k in enumerate(Wt)}


@pytest.mark.parametrize("emb,out_emb,R,L,structures", [(32, 16, 6, 3, 1), (256, 256, 6, 3, 2), (40, 24, 5, 0, 3), (64, 48, 6, 4, 2)])
def test_output_block_alone(lib, ctx, emb, out_emb, R, L, structures):
    from paper_2203_09697_amd import binding_o as O
    pos, gptr = synth.slab_adsorbate_positions(structures, 4, 3, 3, 8, seed=emb)
    ref, e, t = _graph(lib, ctx, pos, gptr, 5.0, 12)
    E_, N = len(ref["src"]), len(pos)
    rng = np.random.default_rng(emb + 1)
    m = rng.standard_normal((E_, emb)).astype(np.float32)
    rbf = rng.standard_normal((E_, R)).astype(np.float32)
    coef = rng.standard_normal(structures).astype(np.float32)
    W = synth.weights_out(emb, out_emb, R, L, seed=3, bias_scale=0.2)
    E_ref, gm_ref, gW_ref = _oracle_out(m, rbf, ref["dst"], gptr, N, W, coef)

    Wd = lib.weights_to_device(W)
    gWd = {k: torch.empty_like(v) for k, v in Wd.items()}
    sb, cb = O.gp_output_workspace(emb, out_emb, R, L, N, E_)
    saved = torch.empty(max(sb, 8), dtype=torch.uint8, device="cuda:0")
    scratch = torch.empty(max(cb, 8), dtype=torch.uint8, device="cuda:0")
    dm, drbf, dgptr = H.to_dev(m, torch.float32), H.to_dev(rbf, torch.float32), H.to_dev(gptr, torch.int32)
    energy = torch.full((structures,), 7.0, dtype=torch.float32, device="cuda:0")
    O.gp_output_forward(ctx, Wd, dm, drbf, e["row_ptr"], dgptr, False, energy, saved, scratch)
    assert H.rel_l2(energy.cpu().numpy(), E_ref) <= TOL
    O.gp_output_forward(ctx, Wd, dm, drbf, e["row_ptr"], dgptr, True, energy, saved, scratch)   # accumulate
    assert H.rel_l2(energy.cpu().numpy(), 2 * E_ref) <= TOL

    gm = torch.empty_like(dm)
    O.gp_output_backward(ctx, Wd, dm, drbf, e["dst"], dgptr, N, H.to_dev(coef, torch.float32), saved, False, gm, gWd, scratch)
    torch.cuda.synchronize()
    errs = {"grad_m": H.rel_l2(gm.cpu().numpy(), gm_ref)}
    for k in gW_ref:
        errs[k] = H.rel_l2(gWd[k].cpu().numpy(), gW_ref[k])
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
    # accumulate onto an existing gradient; no weight gradients requested
    base = rng.standard_normal((E_, emb)).astype(np.float32)
    gm2 = H.to_dev(base, torch.float32)
    O.gp_output_backward(ctx, Wd, dm, drbf, e["dst"], dgptr, N, H.to_dev(coef, torch.float32), saved, True, gm2, None, scratch)
    assert H.rel_l2(gm2.cpu().numpy(), base.astype(np.float64) + gm_ref) <= TOL


def test_model_D_with_output_blocks(lib, ctx):
    from paper_2203_09697_amd.binding_o import ModelD
    w = synth.get_workload("cfg2", emb=64, int_emb=32, basis_emb=8)
    dims = w.dims
    pos, gptr = synth.slab_adsorbate_positions(2, 4, 3, 3, 8, seed=11)
    ref, e, t = _graph(lib, ctx, pos, gptr, dims.cutoff, 14)
    E_, N, nb = len(ref["src"]), len(pos), 2
    Wb = [synth.weights_D(dims, seed=40 + b, bias_scale=0.1) for b in range(nb)]
    Wo = [synth.weights_out(dims.emb, 48, dims.num_radial, 3, seed=50 + b, bias_scale=0.1) for b in range(nb)]
    m0, _ = synth.edge_embeddings(E_, dims.emb, seed=5)
    coef = np.array([1.0, -0.5], dtype=np.float32)
    ob = H.oracle_basis_D(pos, ref, dims)

    Wbt = [{k: v.clone().requires_grad_(True) for k, v in H.t64(W).items()} for W in Wb]
    Wot = [{k: v.clone().requires_grad_(True) for k, v in H.t64(W).items()} for W in Wo]
    mt = torch.tensor(m0, dtype=F64, requires_grad=True)
    E_ref = ooutput.model_D_energies(mt, ob["rbf"], ob["sbf"], ref["idx_kj"], ref["idx_ji"], ref["dst"], gptr, N, Wbt, Wot,
                                     dims.n_res_before, dims.n_res_after)
    leaves = [mt] + [W[k] for W in Wbt for k in W] + [W[k] for W in Wot for k in W]
    grads = torch.autograd.grad((E_ref * torch.tensor(coef, dtype=F64)).sum(), leaves)

    gb = lib.gp_basis_forward(ctx, dims, e, t)
    model = ModelD(ctx, dims, [lib.weights_to_device(W) for W in Wb], [lib.weights_to_device(W) for W in Wo], e, t, gb,
                   H.to_dev(gptr, torch.int32))
    energy = model.forward(H.to_dev(m0, torch.float32))
    gm, gWb, gWo = model.backward(H.to_dev(coef, torch.float32))
    torch.cuda.synchronize()
    errs = {"energy": H.rel_l2(energy.cpu().numpy(), E_ref.detach().numpy()), "grad_m0": H.rel_l2(gm.cpu().numpy(), grads[0].numpy())}
    i = 1
    for b, W in enumerate(Wbt):
        for k in W:
            errs[f"block{b}.{k}"] = H.rel_l2(gWb[b][k].cpu().numpy(), grads[i].numpy())
            i += 1
    for b, W in enumerate(Wot):
        for k in W:
            errs[f"out{b}.{k}"] = H.rel_l2(gWo[b][k].cpu().numpy(), grads[i].numpy())
            i += 1
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
