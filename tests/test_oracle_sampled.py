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
