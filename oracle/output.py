"""Oracle: output block (test infrastructure only).

Sec. 3.3: the updated messages of an interaction block are fed to an output block that sums
them per target atom, h_i = sum_j m'_ji (EdgeAggr), and transforms the sum by an MLP
(NodeUpdate).  This build's reading of what the paper leaves open: each message is first
weighted by a learned linear function of the radial basis of its edge; the summed vector is
projected to the output width without bias, passed through n_layers dense layers with bias and
SiLU, and reduced to one scalar per atom by a final linear layer without bias; a structure's
energy is the sum over its atoms, and the model's energy the sum over all output blocks.
Plain fp64 torch ops, one statement per formula.
"""
import numpy as np
import torch

from . import block

F64 = torch.float64


def output_block(m, rbf, dst, n_atoms, W):
    """Per-atom scalar P_i of one output block.

    t_e = m_e * (rbf_e W_rbf);  h_i = sum_{e: dst[e]=i} t_e;  u = h W_up;
    u = act(u W_k + b_k), k = 0..n_layers-1;  P_i = u_i . w_final
    """
    t = m * (rbf @ W["W_rbf"])
    h = torch.zeros((n_atoms, m.shape[1]), dtype=F64)
    h = h.index_add(0, torch.as_tensor(np.asarray(dst), dtype=torch.long), t)
    u = h @ W["W_up"]
    k = 0
    while f"W{k}" in W:
        u = block.act(u @ W[f"W{k}"] + W[f"b{k}"])
        k += 1
    return u @ W["w_final"]


def structure_energies(p_atom, graph_ptr):
    """E_g = sum of the per-atom scalars of structure g."""
    gp = np.asarray(graph_ptr)
    return torch.stack([p_atom[gp[g]:gp[g + 1]].sum() for g in range(len(gp) - 1)])


def model_D_energies(m0, rbf, sbf, idx_kj, idx_ji, dst, graph_ptr, n_atoms, W_blocks, W_outs, n_res_before, n_res_after):
    """Energies of a variant-D stack with one output block after every interaction block."""
    m = m0
    E = torch.zeros(len(graph_ptr) - 1, dtype=F64)
    for Wb, Wo in zip(W_blocks, W_outs):
        m = block.block_D(m, rbf, sbf, idx_kj, idx_ji, Wb, n_res_before, n_res_after)
        E = E + structure_energies(output_block(m, rbf, dst, n_atoms, Wo), graph_ptr)
    return E
