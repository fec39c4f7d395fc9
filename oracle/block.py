"""Oracle: interaction blocks in fp64 (test infrastructure only).

One block is the message update of Sec. 3.3,
    m'_ji = f_update(m_ji, sum_{k in N_j \\ {i}} f_int(m_kj, e_RBF, a_SBF)),
with f_int the TripletUpdate, the sum the TripletAggr and f_update the
EdgeUpdate of the extended graph net (Sec. 2.1).  Variant D is the Hadamard
interaction with down/up projection (Sec. 3.3); variant G replaces the
Hadamard product by a bilinear layer (Sec. 3.4).  The paper gives the layer
structure in prose only; the exact layer list below is this build's reading
and is what the HIP library is checked against.  Gradients come from
automatic differentiation of these forward functions.
"""
import math

import numpy as np
import torch

F64 = torch.float64


def act(v):
    """SiLU."""
    return v * torch.sigmoid(v)


def to64(a):
    if isinstance(a, torch.Tensor):
        return a.to(F64)
    return torch.as_tensor(np.asarray(a), dtype=F64)


def _long(a):
    return torch.as_tensor(np.asarray(a), dtype=torch.long)


def triplet_aggregate_D(x_kj, s, idx_kj, idx_ji, n_edges):
    """TripletUpdate + TripletAggr, Hadamard form: a_e = sum_{t: ji(t)=e} x_kj[kj(t)] * s_t."""
    tau = x_kj[_long(idx_kj)] * s
    a = torch.zeros((n_edges, x_kj.shape[1]), dtype=F64)
    return a.index_add(0, _long(idx_ji), tau)


def triplet_aggregate_G(x_kj, y, idx_kj, idx_ji, n_edges):
    """Bilinear form: A_e[c, f] = sum_{t: ji(t)=e} y_t[c] * x_kj[kj(t), f]."""
    kj, ji = _long(idx_kj), _long(idx_ji)
    A = torch.zeros((n_edges, y.shape[1], x_kj.shape[1]), dtype=F64)
    step = 1 << 16                       # triplets per pass, only to bound the size of tau
    for lo in range(0, len(kj), step):
        sl = slice(lo, lo + step)
        tau = y[sl, :, None] * x_kj[kj[sl]][:, None, :]
        A.index_add_(0, ji[sl], tau)
    return A


def block_D(m, rbf, sbf, idx_kj, idx_ji, W, n_res_before=1, n_res_after=2):
    """Variant D.  m [E,emb], rbf [E,R], sbf [T,S*R]; W: dict of fp64 tensors W[in,out]."""
    E = m.shape[0]
    x_ji = act(m @ W["W_ji"] + W["b_ji"])
    x_kj = act(m @ W["W_kj"] + W["b_kj"])
    x_kj = x_kj * ((rbf @ W["W_rbf1"]) @ W["W_rbf2"])
    x_kj = act(x_kj @ W["W_down"])
    s = (sbf @ W["W_sbf1"]) @ W["W_sbf2"]
    a = triplet_aggregate_D(x_kj, s, idx_kj, idx_ji, E)
    h = x_ji + act(a @ W["W_up"])
    for r in range(n_res_before):
        h = h + act(act(h @ W[f"W_b{r}_1"] + W[f"b_b{r}_1"]) @ W[f"W_b{r}_2"] + W[f"b_b{r}_2"])
    h = act(h @ W["W_lin"] + W["b_lin"]) + m
    for r in range(n_res_after):
        h = h + act(act(h @ W[f"W_a{r}_1"] + W[f"b_a{r}_1"]) @ W[f"W_a{r}_2"] + W[f"b_a{r}_2"])
    return h


def block_G(m, g, Y, idx_kj, idx_ji, W, radial_at_target=False, id_swap=None):
    """Variant G.  m [E,emb], g [E,R] Gaussian rbf, Y [T,S] = Y_l0(cos alpha).

    The radial factor of the triplet basis is taken at the source edge k->j of the triplet, or,
    with radial_at_target, at its target edge j->i (the ordering of operations in which the
    radial factor leaves the sum over k; Sec. 3.4 speaks of choosing the order of operations of
    the bilinear layer).  Here the sum is written out per triplet in both cases.

    With id_swap (the opposite edge of every edge, -1 if absent) the two messages on a bond are
    coupled (Sec. 3.4, symmetric message passing): the triplet result z is up-projected twice and
    edge e receives (act(z_e W_up) + act(z_swap(e) W_up_ac)) / sqrt(2), the second term being
    zero where the opposite edge does not exist.
    """
    E = m.shape[0]
    x = act(m @ W["W_ba"])
    x = x * ((g @ W["W_rbfS"]) @ W["W_rbfB"])
    x = act(x @ W["W_down"])                                   # [E, emb_trip]
    Rad = torch.einsum("en,lnc->elc", g, W["W_c"])             # [E, S, emb_cbf]
    y = torch.einsum("tl,tlc->tc", Y, Rad[_long(idx_ji if radial_at_target else idx_kj)])      # [T, emb_cbf]
    A = triplet_aggregate_G(x, y, idx_kj, idx_ji, E)           # [E, emb_cbf, emb_trip]
    z = torch.einsum("ecf,cfo->eo", A, W["W_bil"])             # [E, emb_bil]
    x3 = act(z @ W["W_up"])
    if id_swap is not None:
        sw = _long(id_swap)
        x_ac = act(z @ W["W_up_ac"])
        has = (sw >= 0).to(F64)[:, None]
        x3 = (x3 + x_ac[sw.clamp(min=0)] * has) / math.sqrt(2.0)
    return (act(m @ W["W_skip"]) + x3) / math.sqrt(2.0)


def stack_D(m, rbf, sbf, idx_kj, idx_ji, W_list, n_res_before=1, n_res_after=2):
    for W in W_list:
        m = block_D(m, rbf, sbf, idx_kj, idx_ji, W, n_res_before, n_res_after)
    return m


def stack_G(m, g, Y, idx_kj, idx_ji, W_list, radial_at_target=False, id_swap=None):
    for W in W_list:
        m = block_G(m, g, Y, idx_kj, idx_ji, W, radial_at_target, id_swap)
    return m


def loss_and_grads(out, upstream, wrt):
    """L = sum(out * upstream); returns dL/d(each tensor in wrt) by automatic differentiation."""
    L = (out * upstream).sum()
    return torch.autograd.grad(L, wrt, allow_unused=True)
