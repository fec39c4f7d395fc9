"""Shared test plumbing: run the oracle and the HIP library on the same seeded inputs."""
import numpy as np
import torch

import synth
from oracle import basis as obasis
from oracle import block as oblock
from oracle import graph as ograph

F64 = torch.float64


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def row_err(got, ref):
    """Largest per-row relative L2 error: max_r |got_r - ref_r| / max(|ref_r|, rms row norm of ref).
    A whole-tensor norm hides a few corrupted rows among 1e5 good ones; this does not.  Rows whose own norm is
    below the tensor's rms row norm are measured against that rms (their own norm may be arbitrarily small)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    got = got.reshape(got.shape[0], -1) if got.ndim > 1 else got.reshape(-1, 1)
    ref = ref.reshape(got.shape)
    if ref.size == 0:
        return 0.0
    rn = np.sqrt((ref * ref).sum(axis=1))
    floor = np.sqrt((rn * rn).mean())
    if floor == 0:
        return float(np.sqrt(((got - ref) ** 2).sum(axis=1)).max())
    return float((np.sqrt(((got - ref) ** 2).sum(axis=1)) / np.maximum(rn, floor)).max())


def t64(w):
    return {k: torch.tensor(np.asarray(v), dtype=F64) for k, v in w.items()}


def oracle_graph(pos, gptr, cutoff, max_nb):
    src, dst, row_ptr = ograph.edges(pos, gptr, cutoff, max_nb)
    idx_kj, idx_ji, seg = ograph.triplets(src, dst, row_ptr)
    return dict(src=src, dst=dst, row_ptr=row_ptr, idx_kj=idx_kj, idx_ji=idx_ji, seg=seg)


def oracle_basis_D(pos, g, dims):
    pos64 = torch.tensor(pos, dtype=F64)
    d, unit, ca = obasis.geometry(pos64, g["src"], g["dst"], g["idx_kj"], g["idx_ji"])
    rbf = obasis.rbf_bessel(d, dims.cutoff, dims.num_radial, dims.envelope_p)
    rad = obasis.sbf_radial(d, dims.cutoff, dims.num_spherical, dims.num_radial, dims.envelope_p)
    Y = obasis.y_l0(ca, dims.num_spherical)
    kj = torch.as_tensor(g["idx_kj"], dtype=torch.long)
    sbf = (rad[kj] * Y[:, :, None]).reshape(len(kj), rad.shape[1] * rad.shape[2])   # explicit width: also for 0 triplets
    return dict(d=d, unit=unit, cos_alpha=ca, rbf=rbf, rad=rad.reshape(rad.shape[0], -1), sbf=sbf)


def oracle_stack_D(g, ob, dims, W_list, m, gup):
    """Forward + gradients of L = sum(out * gup) w.r.t. m and every weight."""
    Wt = [{k: v.clone().requires_grad_(True) for k, v in t64(W).items()} for W in W_list]
    mt = torch.tensor(m, dtype=F64, requires_grad=True)
    out = oblock.stack_D(mt, ob["rbf"], ob["sbf"], g["idx_kj"], g["idx_ji"], Wt, dims.n_res_before, dims.n_res_after)
    leaves = [mt] + [W[k] for W in Wt for k in W]
    grads = oblock.loss_and_grads(out, torch.tensor(gup, dtype=F64), leaves)
    grads = [torch.zeros_like(l) if gr is None else gr for gr, l in zip(grads, leaves)]   # a leaf the output does not depend on
    gm = grads[0].numpy()
    gW, i = [], 1
    for W in Wt:
        gW.append({k: grads[i + j].numpy() for j, k in enumerate(W)})
        i += len(W)
    return out.detach().numpy(), gm, gW


def oracle_basis_G(pos, g, dims):
    pos64 = torch.tensor(pos, dtype=F64)
    d, unit, ca = obasis.geometry(pos64, g["src"], g["dst"], g["idx_kj"], g["idx_ji"])
    rbf = obasis.rbf_gauss(d, dims.cutoff, dims.num_radial, dims.envelope_p)
    Y = obasis.y_l0(ca, dims.num_spherical)
    return dict(d=d, unit=unit, cos_alpha=ca, rbf=rbf, Y=Y)


def oracle_stack_G(g, ob, dims, W_list, m, gup, want_grad_rbf=False, want_grad_cos=False):
    """Forward + gradients of L = sum(out * gup) w.r.t. m, every weight and the radial basis; with want_grad_cos
    also w.r.t. cos(alpha) of every triplet, returned in kj-major order (sorted by (idx_kj, idx_ji))."""
    Wt = [{k: v.clone().requires_grad_(True) for k, v in t64(W).items()} for W in W_list]
    mt = torch.tensor(m, dtype=F64, requires_grad=True)
    rbf = ob["rbf"].detach().clone().requires_grad_(True)
    id_swap = ograph.reverse_edges(g["src"], g["dst"]) if getattr(dims, "symmetric", False) else None
    cos = ob["cos_alpha"].detach().clone().requires_grad_(True)
    Y = obasis.y_l0(cos, dims.num_spherical) if want_grad_cos else ob["Y"]
    out = oblock.stack_G(mt, rbf, Y, g["idx_kj"], g["idx_ji"], Wt, getattr(dims, "radial_at_target", False), id_swap)
    leaves = [mt, rbf] + [W[k] for W in Wt for k in W] + ([cos] if want_grad_cos else [])
    grads = oblock.loss_and_grads(out, torch.tensor(gup, dtype=F64), leaves)
    grads = [torch.zeros_like(l) if gr is None else gr for gr, l in zip(grads, leaves)]   # a leaf the output does not depend on
    gm, grbf = grads[0].numpy(), grads[1].numpy()
    gW, i = [], 2
    for W in Wt:
        gW.append({k: grads[i + j].numpy() for j, k in enumerate(W)})
        i += len(W)
    if want_grad_cos:
        order = np.lexsort((np.asarray(g["idx_ji"]), np.asarray(g["idx_kj"])))
        return out.detach().numpy(), gm, gW, grbf, grads[-1].numpy()[order]
    return out.detach().numpy(), gm, gW, grbf


def to_dev(a, dtype, device="cuda:0"):
    return torch.as_tensor(np.ascontiguousarray(a), dtype=dtype).to(device)


def graph_from_oracle(g, device="cuda:0"):
    """Device-side gp_graph dict built from oracle index lists (for kernel tests that must
    not depend on the library's own graph construction)."""
    idx_kj, idx_ji = np.asarray(g["idx_kj"]), np.asarray(g["idx_ji"])
    E, T = len(g["src"]), len(idx_kj)
    order = np.lexsort((idx_ji, idx_kj))             # kj-major, then ji
    seg_kj = np.zeros(E + 1, dtype=np.int64)
    np.add.at(seg_kj, idx_kj + 1, 1)
    seg_kj = np.cumsum(seg_kj)
    return dict(n_edges=E, n_triplets=T,
                idx_kj=to_dev(idx_kj, torch.int32, device), idx_ji=to_dev(idx_ji, torch.int32, device),
                seg_ptr_ji=to_dev(g["seg"], torch.int32, device),
                perm_kj=to_dev(order, torch.int32, device), idx_ji_kj=to_dev(idx_ji[order], torch.int32, device),
                seg_ptr_kj=to_dev(seg_kj, torch.int32, device))
