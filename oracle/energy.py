"""Oracle: energy head and forces (test infrastructure only).

Per Sec. 3.3 the updated messages are summed per target atom, h_i = sum_j m'_ji,
and passed through an MLP; the structure energy is the sum of the per-atom
outputs.  Per Sec. 3.2 (energy-centric paradigm) the forces are the negative
gradient of that energy with respect to the atom positions, obtained here by
automatic differentiation through the basis functions (the graph itself and
the input messages m are held fixed).
"""
import numpy as np
import torch

from . import basis, block, graph

F64 = torch.float64


def energy_head(m, dst, n_atoms, Wh):
    """E = sum_i [ w2 . act(h_i W1 + b1) + b2 ],  h_i = sum_{e: dst[e]=i} m_e."""
    h = torch.zeros((n_atoms, m.shape[1]), dtype=F64)
    h = h.index_add(0, torch.as_tensor(np.asarray(dst), dtype=torch.long), m)
    e_atom = block.act(h @ Wh["W1"] + Wh["b1"]) @ Wh["w2"] + Wh["b2"]
    return e_atom.sum(), e_atom


def energy_G(pos, src, dst, idx_kj, idx_ji, m0, W_list, Wh, dims, shift=None):
    """Energy of the variant-G stack + head as a differentiable function of pos (torch fp64 [N,3]).
    shift [E,3]: constant image shifts of the edge sources (periodic structures)."""
    d, _unit, cos_alpha = basis.geometry(pos, src, dst, idx_kj, idx_ji, shift)
    g = basis.rbf_gauss(d, dims.cutoff, dims.num_radial, dims.envelope_p)
    Y = basis.y_l0(cos_alpha, dims.num_spherical)
    id_swap = graph.reverse_edges(src, dst) if getattr(dims, "symmetric", False) and shift is None else None
    assert not (getattr(dims, "symmetric", False) and shift is not None), "pass offsets to reverse_edges for periodic graphs"
    m = block.stack_G(m0, g, Y, idx_kj, idx_ji, W_list, getattr(dims, "radial_at_target", False), id_swap)
    E, _ = energy_head(m, dst, pos.shape[0], Wh)
    return E


def energy_D(pos, src, dst, idx_kj, idx_ji, m0, W_list, Wh, dims):
    """Energy of the variant-D stack + head as a differentiable function of pos."""
    d, _unit, cos_alpha = basis.geometry(pos, src, dst, idx_kj, idx_ji)
    rbf = basis.rbf_bessel(d, dims.cutoff, dims.num_radial, dims.envelope_p)
    sbf = basis.sbf(d, cos_alpha, idx_kj, dims.cutoff, dims.num_spherical, dims.num_radial, dims.envelope_p)
    m = block.stack_D(m0, rbf, sbf, idx_kj, idx_ji, W_list, dims.n_res_before, dims.n_res_after)
    E, _ = energy_head(m, dst, pos.shape[0], Wh)
    return E


def forces(energy_fn, pos_np, *args):
    """f = -dE/dx by automatic differentiation; returns (E float, f [N,3] numpy fp64)."""
    pos = torch.tensor(np.asarray(pos_np, dtype=np.float64), dtype=F64, requires_grad=True)
    E = energy_fn(pos, *args)
    (gpos,) = torch.autograd.grad(E, pos)
    return float(E.detach()), (-gpos).numpy()
