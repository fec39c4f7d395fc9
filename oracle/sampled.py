"""Oracle: exact sub-problems for sampled checks at sizes the full oracle cannot run
(test infrastructure only).

For a centre atom j, let In(j) be the edges k->j and Out(j) the edges j->i.  Every triplet
whose target edge lies in Out(j) has its source edge in In(j), and every triplet whose source
edge lies in In(j) has its target edge in Out(j) (definition of a triplet, Sec. 3.1).  Hence a
block evaluated on the edge subset S = In(j) u Out(j) with exactly the triplets between them
reproduces, exactly,
  * the block output rows m'_e for e in Out(j)  (their aggregation is complete), and
  * for the bilinear variant (Sec. 3.4), the gradient rows dL/dm_e' for e' in In(j) of
    L = sum_e <m'_e, upstream_e>: every path from m_e' to the loss runs through a triplet into
    Out(j) or through the skip term of its own row, and in that variant the own row is a SUM of
    the skip term and the aggregated term, so its derivative w.r.t. m_e' does not depend on the
    (incomplete) aggregation of row e'.  For the Hadamard variant the own row is a nonlinear
    function of that sum, so only the output rows are exact,
whatever the rest of the graph looks like.
"""
import numpy as np


def centre_subproblem(src, dst, row_ptr, j):
    """Edge subset and local triplet lists of centre atom j.

    Returns dict(edges=S (global ids, ascending), out_local, in_local (positions in S),
    idx_kj, idx_ji (local ids, ordered by (ji, kj)))."""
    src = np.asarray(src)
    dst = np.asarray(dst)
    in_e = np.arange(row_ptr[j], row_ptr[j + 1], dtype=np.int64)
    out_e = np.nonzero(src == j)[0].astype(np.int64)
    S = np.unique(np.concatenate([in_e, out_e]))
    loc = {int(e): n for n, e in enumerate(S)}
    kj, ji = [], []
    for e in out_e:                      # ascending global id == ascending local id
        i = dst[e]
        for ep in in_e:
            if src[ep] != i:
                kj.append(loc[int(ep)])
                ji.append(loc[int(e)])
    return dict(edges=S, out_local=np.array([loc[int(e)] for e in out_e], dtype=np.int64),
                in_local=np.array([loc[int(e)] for e in in_e], dtype=np.int64),
                idx_kj=np.asarray(kj, dtype=np.int64), idx_ji=np.asarray(ji, dtype=np.int64))


def masked_readout_G(pos, src, dst, row_ptr, seg_ptr_ji, atoms, m, upstream, W, dims):
    """Bilinear block (Sec. 3.4) under the loss L_J = sum over the out-edges e of the atoms j in `atoms`
    of <m'_e, upstream_e>, i.e. with an upstream gradient that vanishes outside Out(J).

    Every m'_e with e in Out(j) is reproduced exactly by the sub-problem of centre atom j (see the module
    header), as a function of the messages, the weights and the positions alike.  Hence L_J is the sum of
    the sub-problems' losses, and so is every gradient of it: dL/dm (rows outside the sub-problems are
    zero), dL/dW for every weight, dL/dg for the radial basis rows, dL/dcos(alpha) of the triplets of
    Out(J) and the forces -dL/dx (graph and messages held fixed, Sec. 3.2).  Each sub-problem is small
    enough for the fp64 oracle even when the whole graph is not.

    Returns dict(loss, out_rows {edge id: m'_e}, grad_m [E, emb], grad_W {name: array}, grad_rbf [E, R],
    grad_cos (values) with trip_ids (their ji-major triplet ids, from seg_ptr_ji), forces [N, 3])."""
    import torch

    from . import basis, block
    F64 = torch.float64
    src, dst = np.asarray(src), np.asarray(dst)
    E = len(src)
    pos_t = torch.tensor(np.asarray(pos, dtype=np.float64), dtype=F64, requires_grad=True)
    Wt = {k: torch.tensor(np.asarray(v), dtype=F64, requires_grad=True) for k, v in W.items()}
    names = list(Wt)
    res = dict(loss=0.0, out_rows={}, grad_m=np.zeros((E, m.shape[1])), grad_W={k: np.zeros(tuple(v.shape)) for k, v in Wt.items()},
               grad_rbf=np.zeros((E, dims.num_radial)), grad_cos=[], trip_ids=[], forces=np.zeros((len(pos), 3)))
    for j in atoms:
        sp = centre_subproblem(src, dst, row_ptr, int(j))
        S, ol = sp["edges"], sp["out_local"]
        d, _unit, ca = basis.geometry(pos_t, src[S], dst[S], sp["idx_kj"], sp["idx_ji"])
        g = basis.rbf_gauss(d, dims.cutoff, dims.num_radial, dims.envelope_p)
        g.retain_grad()
        ca.retain_grad()
        Y = basis.y_l0(ca, dims.num_spherical)
        ms = torch.tensor(np.asarray(m)[S], dtype=F64, requires_grad=True)
        o = block.block_G(ms, g, Y, sp["idx_kj"], sp["idx_ji"], Wt)
        up = torch.zeros_like(o)
        up[ol] = torch.tensor(np.asarray(upstream)[S[ol]], dtype=F64)
        L = (o * up).sum()
        grads = torch.autograd.grad(L, [ms, pos_t, g, ca] + [Wt[k] for k in names], allow_unused=True)
        res["loss"] += float(L.detach())
        for n_, e_ in zip(ol, S[ol]):
            res["out_rows"][int(e_)] = o.detach().numpy()[n_]
        res["grad_m"][S] += grads[0].numpy()
        res["forces"] -= grads[1].numpy()
        res["grad_rbf"][S] += grads[2].numpy()
        res["grad_cos"].append(grads[3].numpy())
        # the sub-problem lists its triplets by (target edge, source edge) ascending, as the whole list does
        res["trip_ids"].append(np.concatenate([np.arange(seg_ptr_ji[e_], seg_ptr_ji[e_ + 1]) for e_ in S[ol]]))
        for k, gr in zip(names, grads[4:]):
            if gr is not None:
                res["grad_W"][k] += gr.numpy()
    res["grad_cos"] = np.concatenate(res["grad_cos"]) if res["grad_cos"] else np.zeros(0)
    res["trip_ids"] = np.concatenate(res["trip_ids"]) if res["trip_ids"] else np.zeros(0, dtype=np.int64)
    return res
