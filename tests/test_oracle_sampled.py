"""Pin for oracle/sampled.py (CPU only): the centre-atom sub-problem reproduces the full oracle's
output rows on Out(j) (both variants) and gradient rows on In(j) (bilinear variant) exactly, on a
capped (asymmetric) graph."""
import numpy as np
import pytest
import torch

import synth
from oracle import basis, block, graph, sampled

F64 = torch.float64


def _t64(w):
    return {k: torch.tensor(v, dtype=F64) for k, v in w.items()}


@pytest.mark.parametrize("variant", ["D", "G"])
def test_centre_subproblem_is_exact(variant):
    pos, gptr = synth.slab_adsorbate_positions(1, 3, 3, 3, 6, seed=3)
    cutoff, cap = 4.5, 7
    src, dst, row_ptr = graph.edges(pos, gptr, cutoff, cap)
    idx_kj, idx_ji, _ = graph.triplets(src, dst, row_ptr)
    E = len(src)
    if variant == "D":
        dims = synth.BlockDims(variant="D", dtype="f32", emb=8, int_emb=5, basis_emb=3, num_radial=4,
                               num_spherical=3, cutoff=cutoff)
        W = _t64(synth.weights_D(dims, seed=1, bias_scale=0.1))
    else:
        dims = synth.BlockDims(variant="G", dtype="f32", emb=8, int_emb=5, emb_rbf=3, emb_cbf=4, emb_bil=6,
                               num_radial=7, num_spherical=3, cutoff=cutoff)
        W = _t64(synth.weights_G(dims, seed=1))
    m_np, gup_np = synth.edge_embeddings(E, dims.emb, seed=2)
    pos64 = torch.tensor(pos, dtype=F64)

    def run(src_, dst_, kj_, ji_, m_, gup_):
        d, _, ca = basis.geometry(pos64, src_, dst_, kj_, ji_)
        m_ = m_.clone().requires_grad_(True)
        if variant == "D":
            rbf = basis.rbf_bessel(d, cutoff, dims.num_radial)
            sbf = basis.sbf(d, ca, kj_, cutoff, dims.num_spherical, dims.num_radial)
            out = block.block_D(m_, rbf, sbf, kj_, ji_, W)
        else:
            out = block.block_G(m_, basis.rbf_gauss(d, cutoff, dims.num_radial), basis.y_l0(ca, dims.num_spherical),
                                kj_, ji_, W)
        (gm,) = torch.autograd.grad((out * gup_).sum(), m_)
        return out.detach().numpy(), gm.numpy()

    m, gup = torch.tensor(m_np, dtype=F64), torch.tensor(gup_np, dtype=F64)
    out_full, gm_full = run(src, dst, idx_kj, idx_ji, m, gup)
    checked = 0
    for j in (0, 5, 17, len(pos) - 1):
        sp = sampled.centre_subproblem(src, dst, row_ptr, j)
        S = sp["edges"]
        out_s, gm_s = run(src[S], dst[S], sp["idx_kj"], sp["idx_ji"], m[S], gup[S])
        assert np.allclose(out_s[sp["out_local"]], out_full[S[sp["out_local"]]], rtol=1e-12, atol=1e-13)
        if variant == "G":
            assert np.allclose(gm_s[sp["in_local"]], gm_full[S[sp["in_local"]]], rtol=1e-12, atol=1e-13)
        checked += len(sp["out_local"]) + len(sp["in_local"])
    assert checked > 20


def test_masked_readout_equals_the_full_oracle_with_a_masked_upstream_gradient():
    """L_J and all its gradients (messages, weights, radial basis, cos alpha, forces) from the sum of centre-atom
    sub-problems against the full oracle run once with the upstream gradient zeroed outside Out(J)."""
    pos, gptr = synth.slab_adsorbate_positions(1, 3, 3, 3, 6, seed=4)
    cutoff, cap = 4.5, 8
    src, dst, row_ptr = graph.edges(pos, gptr, cutoff, cap)
    idx_kj, idx_ji, seg = graph.triplets(src, dst, row_ptr)
    E = len(src)
    dims = synth.BlockDims(variant="G", dtype="f32", emb=8, int_emb=5, emb_rbf=3, emb_cbf=4, emb_bil=6,
                           num_radial=7, num_spherical=3, cutoff=cutoff)
    W_np = synth.weights_G(dims, seed=1)
    m_np, gup_np = synth.edge_embeddings(E, dims.emb, seed=2)
    J = [1, 4, 11, len(pos) - 2]
    got = sampled.masked_readout_G(pos, src, dst, row_ptr, seg, J, m_np, gup_np, W_np, dims)
    # full oracle, masked upstream gradient
    mask = np.isin(src, J)
    assert 0 < mask.sum() < E
    pos_t = torch.tensor(pos.astype(np.float64), dtype=F64, requires_grad=True)
    d, _, ca = basis.geometry(pos_t, src, dst, idx_kj, idx_ji)
    g = basis.rbf_gauss(d, cutoff, dims.num_radial); g.retain_grad()
    ca.retain_grad()
    Wt = {k: v.clone().requires_grad_(True) for k, v in _t64(W_np).items()}
    mt = torch.tensor(m_np, dtype=F64, requires_grad=True)
    out = block.block_G(mt, g, basis.y_l0(ca, dims.num_spherical), idx_kj, idx_ji, Wt)
    L = (out * torch.tensor(gup_np * mask[:, None], dtype=F64)).sum()
    names = list(Wt)
    grads = torch.autograd.grad(L, [mt, pos_t, g, ca] + [Wt[k] for k in names])
    assert abs(got["loss"] - float(L)) < 1e-11 * max(1.0, abs(float(L)))
    for e_, row in got["out_rows"].items():
        assert np.allclose(row, out.detach().numpy()[e_], rtol=1e-12, atol=1e-13)
    assert sorted(got["out_rows"]) == np.nonzero(mask)[0].tolist()
    assert np.allclose(got["grad_m"], grads[0].numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(got["forces"], -grads[1].numpy(), rtol=1e-10, atol=1e-11)
    assert np.allclose(got["grad_rbf"], grads[2].numpy(), rtol=1e-11, atol=1e-12)
    gc = np.zeros(len(idx_kj))
    gc[got["trip_ids"]] = got["grad_cos"]
    assert len(np.unique(got["trip_ids"])) == len(got["trip_ids"])
    assert np.allclose(gc, grads[3].numpy(), rtol=1e-11, atol=1e-12)
    for k, gr in zip(names, grads[4:]):
        assert np.allclose(got["grad_W"][k], gr.numpy(), rtol=1e-11, atol=1e-12), k
    assert np.abs(grads[1].numpy()).max() > 1e-6 and np.abs(grads[3].numpy()).max() > 1e-8
