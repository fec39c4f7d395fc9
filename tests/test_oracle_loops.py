"""Second layer of pins for the oracle (CPU only): the blocks written out as nested scalar
loops, hand-written reverse passes of the two aggregation forms, and a routed closed form of
the energy head.

The oracle's forward functions are vectorised torch statements and its gradients come from
automatic differentiation.  Everything here re-derives the same quantities without torch ops
on tensors: Python loops over edges, triplets and features on numpy scalars, following the
update equation of Sec. 3.3 (sum over k in N_j without i of f_int(m_kj, e_RBF, a_SBF), then
f_update), the bilinear form of Sec. 3.4 and the output step of Sec. 3.3 (messages summed per
target atom, then an MLP).  A transposed weight, a swapped gather index, a dropped bias or a
scatter by the wrong end of an edge fails one of them.
"""
import math

import numpy as np
import torch

import synth
from oracle import basis, block, energy, graph

F64 = torch.float64


def _silu(v):
    return v / (1.0 + math.exp(-v))


def _dsilu(v):
    s = 1.0 / (1.0 + math.exp(-v))
    return s * (1.0 + v * (1.0 - s))


def _dense(x, W, b=None):
    """y[o] = sum_i x[i] W[i, o] (+ b[o]) with scalar loops."""
    n_in, n_out = W.shape
    assert len(x) == n_in
    y = []
    for o in range(n_out):
        acc = 0.0 if b is None else float(b[o])
        for i in range(n_in):
            acc += float(x[i]) * float(W[i, o])
        y.append(acc)
    return y


def _tiny(variant, seed, n_atoms=8, cutoff=3.0, bias_scale=0.3):
    pos, gptr = synth.cube_positions(n_atoms, 3.8, 0.9, seed=seed)
    src, dst, row_ptr = graph.edges(pos, gptr, cutoff)
    idx_kj, idx_ji, seg = graph.triplets(src, dst, row_ptr)
    if variant == "D":
        dims = synth.BlockDims(variant="D", dtype="f32", emb=5, int_emb=3, basis_emb=2,
                               num_radial=3, num_spherical=3, cutoff=cutoff, n_res_before=1, n_res_after=1)
        W = synth.weights_D(dims, seed=seed + 1, bias_scale=bias_scale)
    else:
        dims = synth.BlockDims(variant="G", dtype="f32", emb=5, int_emb=3, emb_rbf=2, emb_cbf=3,
                               emb_bil=4, num_radial=5, num_spherical=3, cutoff=cutoff)
        W = synth.weights_G(dims, seed=seed + 1)
    W = {k: np.asarray(v, dtype=np.float64) for k, v in W.items()}
    m, gup = synth.edge_embeddings(len(src), dims.emb, seed=seed + 2)
    pos64 = torch.tensor(pos, dtype=F64)
    d, _unit, ca = basis.geometry(pos64, src, dst, idx_kj, idx_ji)
    return dict(pos=pos, src=np.asarray(src), dst=np.asarray(dst), idx_kj=np.asarray(idx_kj), idx_ji=np.asarray(idx_ji),
                dims=dims, W=W, m=m.astype(np.float64), gup=gup.astype(np.float64), d=d, cos_alpha=ca)


def _t(w):
    return {k: torch.tensor(v, dtype=F64) for k, v in w.items()}


# ---- variant D, every layer including the residual layers and every bias ---------------------------
def _block_D_loops(m, rbf, sbf, idx_kj, idx_ji, W, n_res_before, n_res_after):
    E = len(m)
    x_ji, x_kj = [], []
    for e in range(E):
        x_ji.append([_silu(v) for v in _dense(m[e], W["W_ji"], W["b_ji"])])
        xk = [_silu(v) for v in _dense(m[e], W["W_kj"], W["b_kj"])]
        gate = _dense(_dense(rbf[e], W["W_rbf1"]), W["W_rbf2"])
        xk = [a * b for a, b in zip(xk, gate)]
        x_kj.append([_silu(v) for v in _dense(xk, W["W_down"])])
    F = W["W_down"].shape[1]
    a = [[0.0] * F for _ in range(E)]
    for t in range(len(idx_kj)):                       # TripletUpdate, then TripletAggr in triplet order
        s_t = _dense(_dense(sbf[t], W["W_sbf1"]), W["W_sbf2"])
        for f in range(F):
            a[idx_ji[t]][f] += x_kj[idx_kj[t]][f] * s_t[f]
    out = []
    for e in range(E):
        h = [p + _silu(q) for p, q in zip(x_ji[e], _dense(a[e], W["W_up"]))]
        for r in range(n_res_before):
            u = [_silu(v) for v in _dense(h, W[f"W_b{r}_1"], W[f"b_b{r}_1"])]
            u = [_silu(v) for v in _dense(u, W[f"W_b{r}_2"], W[f"b_b{r}_2"])]
            h = [p + q for p, q in zip(h, u)]
        h = [_silu(v) + float(m[e][i]) for i, v in enumerate(_dense(h, W["W_lin"], W["b_lin"]))]
        for r in range(n_res_after):
            u = [_silu(v) for v in _dense(h, W[f"W_a{r}_1"], W[f"b_a{r}_1"])]
            u = [_silu(v) for v in _dense(u, W[f"W_a{r}_2"], W[f"b_a{r}_2"])]
            h = [p + q for p, q in zip(h, u)]
        out.append(h)
    return np.asarray(out)


def test_block_D_matches_scalar_loops_with_residual_layers_and_biases():
    s = _tiny("D", seed=11)
    dims = s["dims"]
    assert len(s["idx_kj"]) > 30
    rbf = basis.rbf_bessel(s["d"], dims.cutoff, dims.num_radial)
    sbf = basis.sbf(s["d"], s["cos_alpha"], s["idx_kj"], dims.cutoff, dims.num_spherical, dims.num_radial)
    for k in ("b_kj", "b_lin", "b_ji", "b_b0_1", "b_b0_2", "b_a0_1", "b_a0_2"):
        assert np.abs(s["W"][k]).max() > 0.01, k
    out = block.block_D(torch.tensor(s["m"], dtype=F64), rbf, sbf, s["idx_kj"], s["idx_ji"], _t(s["W"]),
                        dims.n_res_before, dims.n_res_after).numpy()
    ref = _block_D_loops(s["m"], rbf.numpy(), sbf.numpy(), s["idx_kj"], s["idx_ji"], s["W"], dims.n_res_before, dims.n_res_after)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_block_D_routes_b_kj_b_lin_and_one_residual_layer():
    """Single non-zero entries: b_kj alone drives the triplet path; b_lin and the residual layer before
    the skip act on fixed features."""
    s = _tiny("D", seed=12)
    dims = s["dims"]
    E, R = len(s["src"]), dims.num_radial
    rbf = basis.rbf_bessel(s["d"], dims.cutoff, dims.num_radial)
    sbf = basis.sbf(s["d"], s["cos_alpha"], s["idx_kj"], dims.cutoff, dims.num_spherical, dims.num_radial)
    Z = {k: np.zeros_like(v) for k, v in s["W"].items()}
    W = {k: v.copy() for k, v in Z.items()}
    # triplet path fed by the bias of the k->j projection only (m does not enter it)
    W["b_kj"][1] = 0.8
    W["W_rbf1"][2, 1] = 1.3
    W["W_rbf2"][1, 1] = 0.7
    W["W_down"][1, 2] = 1.1
    W["W_sbf1"][2 * R + 0, 0] = 0.9
    W["W_sbf2"][0, 2] = 1.2
    W["W_up"][2, 3] = 0.6
    # residual layer before the skip: feature 3 -> hidden 0 (bias 0.2) -> feature 4 (bias -0.1)
    W["W_b0_1"][3, 0] = 1.4; W["b_b0_1"][0] = 0.2
    W["W_b0_2"][0, 4] = 0.5; W["b_b0_2"][4] = -0.1
    # skip layer: feature 4 -> feature 0, bias on feature 2
    W["W_lin"][4, 0] = 1.5; W["b_lin"][2] = 0.35
    out = block.block_D(torch.tensor(s["m"], dtype=F64), rbf, sbf, s["idx_kj"], s["idx_ji"], _t(W),
                        dims.n_res_before, dims.n_res_after).numpy()
    rn, sn = rbf.numpy(), sbf.numpy()
    ref = s["m"].copy()
    for e in range(E):
        a = 0.0
        for t in range(len(s["idx_kj"])):
            if s["idx_ji"][t] == e:
                k = s["idx_kj"][t]
                xk = _silu(1.1 * (_silu(0.8) * (1.3 * 0.7 * rn[k, 2])))
                a += xk * (0.9 * 1.2 * sn[t, 2 * R + 0])
        h3 = _silu(0.6 * a)                                     # x_ji is act(0) = 0 everywhere
        # residual layer: every output feature o gets act(b_b0_2[o] + ...) added, here only feature 4 is non-zero
        h4 = _silu(0.5 * _silu(1.4 * h3 + 0.2) - 0.1)
        other = _silu(0.5 * _silu(1.4 * h3 + 0.2) * 0.0)        # = act(0) = 0 for the other features
        assert other == 0.0
        ref[e, 0] += _silu(1.5 * h4)
        ref[e, 2] += _silu(0.35)
        # features 1, 3, 4 receive act(0) = 0 from the skip layer
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)


# ---- variant G, default form (radial factor at the source edge) ------------------------------------
def _block_G_loops(m, g, Y, idx_kj, idx_ji, W):
    E = len(m)
    S, R, C = W["W_c"].shape
    F = W["W_down"].shape[1]
    O = W["W_bil"].shape[2]
    x = []
    for e in range(E):
        v = [_silu(q) for q in _dense(m[e], W["W_ba"])]
        gate = _dense(_dense(g[e], W["W_rbfS"]), W["W_rbfB"])
        v = [p * q for p, q in zip(v, gate)]
        x.append([_silu(q) for q in _dense(v, W["W_down"])])
    A = np.zeros((E, C, F))
    for t in range(len(idx_kj)):
        k, e = idx_kj[t], idx_ji[t]
        for c in range(C):
            y = 0.0
            for l in range(S):
                rad = 0.0
                for n in range(R):
                    rad += float(g[k, n]) * float(W["W_c"][l, n, c])    # radial factor of the SOURCE edge k->j
                y += float(Y[t, l]) * rad
            for f in range(F):
                A[e, c, f] += y * x[k][f]
    out = []
    for e in range(E):
        z = [0.0] * O
        for o in range(O):
            for c in range(C):
                for f in range(F):
                    z[o] += A[e, c, f] * float(W["W_bil"][c, f, o])
        up = [_silu(q) for q in _dense(z, W["W_up"])]
        sk = [_silu(q) for q in _dense(m[e], W["W_skip"])]
        out.append([(p + q) / math.sqrt(2.0) for p, q in zip(sk, up)])
    return np.asarray(out)


def test_block_G_source_edge_form_matches_scalar_loops():
    s = _tiny("G", seed=13)
    dims = s["dims"]
    assert len(s["idx_kj"]) > 30
    g = basis.rbf_gauss(s["d"], dims.cutoff, dims.num_radial)
    Y = basis.y_l0(s["cos_alpha"], dims.num_spherical)
    out = block.block_G(torch.tensor(s["m"], dtype=F64), g, Y, s["idx_kj"], s["idx_ji"], _t(s["W"])).numpy()
    ref = _block_G_loops(s["m"], g.numpy(), Y.numpy(), s["idx_kj"], s["idx_ji"], s["W"])
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    # the loops above are not the target-edge form: that one differs on this input
    out_t = block.block_G(torch.tensor(s["m"], dtype=F64), g, Y, s["idx_kj"], s["idx_ji"], _t(s["W"]), radial_at_target=True).numpy()
    assert not np.allclose(out_t, ref, rtol=1e-4, atol=1e-7)


# ---- hand-written reverse passes of the two aggregation forms --------------------------------------
def test_aggregate_D_backward_by_loops_matches_autograd():
    """a_e[f] = sum_{t in e} x[kj(t), f] s[t, f]  =>  dL/dx[k, f] = sum_{t: kj(t)=k} G[ji(t), f] s[t, f],
    dL/ds[t, f] = G[ji(t), f] x[kj(t), f] (gather and scatter exchange roles)."""
    s = _tiny("D", seed=14)
    E, T, F = len(s["src"]), len(s["idx_kj"]), 4
    rng = np.random.default_rng(5)
    x = rng.standard_normal((E, F)); sv = rng.standard_normal((T, F)); G = rng.standard_normal((E, F))
    xt = torch.tensor(x, dtype=F64, requires_grad=True)
    st = torch.tensor(sv, dtype=F64, requires_grad=True)
    a = block.triplet_aggregate_D(xt, st, s["idx_kj"], s["idx_ji"], E)
    gx, gs = torch.autograd.grad((a * torch.tensor(G, dtype=F64)).sum(), [xt, st])
    gx_ref, gs_ref = np.zeros((E, F)), np.zeros((T, F))
    for t in range(T):
        k, e = s["idx_kj"][t], s["idx_ji"][t]
        for f in range(F):
            gx_ref[k, f] += G[e, f] * sv[t, f]
            gs_ref[t, f] = G[e, f] * x[k, f]
    assert np.allclose(gx.numpy(), gx_ref, rtol=1e-13, atol=1e-13)
    assert np.allclose(gs.numpy(), gs_ref, rtol=1e-13, atol=1e-13)


def test_aggregate_G_backward_by_loops_matches_autograd():
    """A_e[c, f] = sum_{t in e} y[t, c] x[kj(t), f]  =>  dL/dx[k, f] = sum_{t: kj(t)=k} sum_c G[ji(t), c, f] y[t, c],
    dL/dy[t, c] = sum_f G[ji(t), c, f] x[kj(t), f]."""
    s = _tiny("G", seed=15)
    E, T, C, F = len(s["src"]), len(s["idx_kj"]), 3, 4
    rng = np.random.default_rng(6)
    x = rng.standard_normal((E, F)); y = rng.standard_normal((T, C)); G = rng.standard_normal((E, C, F))
    xt = torch.tensor(x, dtype=F64, requires_grad=True)
    yt = torch.tensor(y, dtype=F64, requires_grad=True)
    A = block.triplet_aggregate_G(xt, yt, s["idx_kj"], s["idx_ji"], E)
    gx, gy = torch.autograd.grad((A * torch.tensor(G, dtype=F64)).sum(), [xt, yt])
    gx_ref, gy_ref = np.zeros((E, F)), np.zeros((T, C))
    for t in range(T):
        k, e = s["idx_kj"][t], s["idx_ji"][t]
        for c in range(C):
            for f in range(F):
                gx_ref[k, f] += G[e, c, f] * y[t, c]
                gy_ref[t, c] += G[e, c, f] * x[k, f]
    assert np.allclose(gx.numpy(), gx_ref, rtol=1e-13, atol=1e-13)
    assert np.allclose(gy.numpy(), gy_ref, rtol=1e-13, atol=1e-13)


def test_block_G_hand_written_backward_matches_autograd():
    """The whole reverse pass of the source-edge bilinear block, layer by layer with explicit
    loops over triplets for the gather/scatter transposition, against automatic differentiation:
    gradients w.r.t. the messages, every weight, the radial basis and the angular basis."""
    s = _tiny("G", seed=16)
    dims = s["dims"]
    E, T = len(s["src"]), len(s["idx_kj"])
    W = s["W"]
    g = basis.rbf_gauss(s["d"], dims.cutoff, dims.num_radial).numpy()
    Y = basis.y_l0(s["cos_alpha"], dims.num_spherical).numpy()
    m, Gup = s["m"], s["gup"]
    kj, ji = s["idx_kj"], s["idx_ji"]
    vs, vd = np.vectorize(_silu), np.vectorize(_dsilu)
    # forward, keeping what the reverse pass needs
    z_ba = m @ W["W_ba"]; gate = (g @ W["W_rbfS"]) @ W["W_rbfB"]
    xg = vs(z_ba) * gate
    z_dn = xg @ W["W_down"]; x = vs(z_dn)
    Rad = np.einsum("en,lnc->elc", g, W["W_c"])
    y = np.einsum("tl,tlc->tc", Y, Rad[kj])
    A = np.zeros((E, y.shape[1], x.shape[1]))
    for t in range(T):
        A[ji[t]] += np.outer(y[t], x[kj[t]])
    z = np.einsum("ecf,cfo->eo", A, W["W_bil"])
    z_up = z @ W["W_up"]; z_sk = m @ W["W_skip"]
    # reverse
    r2 = 1.0 / math.sqrt(2.0)
    d_up = Gup * r2 * vd(z_up); d_sk = Gup * r2 * vd(z_sk)
    gW = {"W_up": z.T @ d_up, "W_skip": m.T @ d_sk}
    dz = d_up @ W["W_up"].T
    gW["W_bil"] = np.einsum("ecf,eo->cfo", A, dz)
    dA = np.einsum("eo,cfo->ecf", dz, W["W_bil"])
    dx, dy = np.zeros_like(x), np.zeros_like(y)
    for t in range(T):
        dx[kj[t]] += dA[ji[t]].T @ y[t]
        dy[t] = dA[ji[t]] @ x[kj[t]]
    dY = np.einsum("tc,tlc->tl", dy, Rad[kj])
    dRad = np.zeros_like(Rad)
    for t in range(T):
        dRad[kj[t]] += np.outer(Y[t], dy[t])
    gW["W_c"] = np.einsum("en,elc->lnc", g, dRad)
    dg = np.einsum("elc,lnc->en", dRad, W["W_c"])
    d_dn = dx * vd(z_dn)
    gW["W_down"] = xg.T @ d_dn
    dxg = d_dn @ W["W_down"].T
    dgate = dxg * vs(z_ba)
    gW["W_rbfB"] = (g @ W["W_rbfS"]).T @ dgate
    gW["W_rbfS"] = g.T @ (dgate @ W["W_rbfB"].T)
    dg += (dgate @ W["W_rbfB"].T) @ W["W_rbfS"].T
    d_ba = dxg * gate * vd(z_ba)
    gW["W_ba"] = m.T @ d_ba
    dm = d_ba @ W["W_ba"].T + d_sk @ W["W_skip"].T
    # automatic differentiation of the oracle
    Wt = {k: torch.tensor(v, dtype=F64, requires_grad=True) for k, v in W.items()}
    mt = torch.tensor(m, dtype=F64, requires_grad=True)
    gt = torch.tensor(g, dtype=F64, requires_grad=True)
    Yt = torch.tensor(Y, dtype=F64, requires_grad=True)
    out = block.block_G(mt, gt, Yt, kj, ji, Wt)
    names = list(Wt)
    grads = block.loss_and_grads(out, torch.tensor(Gup, dtype=F64), [mt, gt, Yt] + [Wt[k] for k in names])
    assert np.allclose(grads[0].numpy(), dm, rtol=1e-11, atol=1e-12)
    assert np.allclose(grads[1].numpy(), dg, rtol=1e-11, atol=1e-12)
    assert np.allclose(grads[2].numpy(), dY, rtol=1e-11, atol=1e-12)
    for k, gr in zip(names, grads[3:]):
        assert np.allclose(gr.numpy(), gW[k], rtol=1e-11, atol=1e-12), k


def test_block_D_hand_written_backward_matches_autograd():
    """Reverse pass of the Hadamard block (one residual layer on each side of the skip) by hand."""
    s = _tiny("D", seed=17)
    dims = s["dims"]
    E, T = len(s["src"]), len(s["idx_kj"])
    W = s["W"]
    rbf = basis.rbf_bessel(s["d"], dims.cutoff, dims.num_radial).numpy()
    sbf = basis.sbf(s["d"], s["cos_alpha"], s["idx_kj"], dims.cutoff, dims.num_spherical, dims.num_radial).numpy()
    m, Gup = s["m"], s["gup"]
    kj, ji = s["idx_kj"], s["idx_ji"]
    vs, vd = np.vectorize(_silu), np.vectorize(_dsilu)
    z_ji = m @ W["W_ji"] + W["b_ji"]; z_kj = m @ W["W_kj"] + W["b_kj"]
    r1 = rbf @ W["W_rbf1"]; gate = r1 @ W["W_rbf2"]
    xg = vs(z_kj) * gate
    z_dn = xg @ W["W_down"]; x = vs(z_dn)
    s1 = sbf @ W["W_sbf1"]; sp = s1 @ W["W_sbf2"]
    a = np.zeros((E, x.shape[1]))
    for t in range(T):
        a[ji[t]] += x[kj[t]] * sp[t]
    z_up = a @ W["W_up"]
    h0 = vs(z_ji) + vs(z_up)
    zb1 = h0 @ W["W_b0_1"] + W["b_b0_1"]; ub1 = vs(zb1)
    zb2 = ub1 @ W["W_b0_2"] + W["b_b0_2"]
    h1 = h0 + vs(zb2)
    z_lin = h1 @ W["W_lin"] + W["b_lin"]
    h2 = vs(z_lin) + m
    za1 = h2 @ W["W_a0_1"] + W["b_a0_1"]; ua1 = vs(za1)
    za2 = ua1 @ W["W_a0_2"] + W["b_a0_2"]
    # reverse
    gW = {}
    dh2 = Gup.copy()
    d = Gup * vd(za2); gW["W_a0_2"] = ua1.T @ d; gW["b_a0_2"] = d.sum(0)
    d = (d @ W["W_a0_2"].T) * vd(za1); gW["W_a0_1"] = h2.T @ d; gW["b_a0_1"] = d.sum(0)
    dh2 += d @ W["W_a0_1"].T
    dm = dh2.copy()
    d = dh2 * vd(z_lin); gW["W_lin"] = h1.T @ d; gW["b_lin"] = d.sum(0)
    dh1 = d @ W["W_lin"].T
    dh0 = dh1.copy()
    d = dh1 * vd(zb2); gW["W_b0_2"] = ub1.T @ d; gW["b_b0_2"] = d.sum(0)
    d = (d @ W["W_b0_2"].T) * vd(zb1); gW["W_b0_1"] = h0.T @ d; gW["b_b0_1"] = d.sum(0)
    dh0 += d @ W["W_b0_1"].T
    d = dh0 * vd(z_ji); gW["W_ji"] = m.T @ d; gW["b_ji"] = d.sum(0); dm += d @ W["W_ji"].T
    d = dh0 * vd(z_up); gW["W_up"] = a.T @ d
    da = d @ W["W_up"].T
    dx, dsp = np.zeros_like(x), np.zeros_like(sp)
    for t in range(T):
        dx[kj[t]] += da[ji[t]] * sp[t]
        dsp[t] = da[ji[t]] * x[kj[t]]
    gW["W_sbf2"] = s1.T @ dsp; gW["W_sbf1"] = sbf.T @ (dsp @ W["W_sbf2"].T)
    d = dx * vd(z_dn); gW["W_down"] = xg.T @ d
    dxg = d @ W["W_down"].T
    dgate = dxg * vs(z_kj)
    gW["W_rbf2"] = r1.T @ dgate; gW["W_rbf1"] = rbf.T @ (dgate @ W["W_rbf2"].T)
    d = dxg * gate * vd(z_kj); gW["W_kj"] = m.T @ d; gW["b_kj"] = d.sum(0); dm += d @ W["W_kj"].T
    Wt = {k: torch.tensor(v, dtype=F64, requires_grad=True) for k, v in W.items()}
    mt = torch.tensor(m, dtype=F64, requires_grad=True)
    out = block.block_D(mt, torch.tensor(rbf, dtype=F64), torch.tensor(sbf, dtype=F64), kj, ji, Wt, 1, 1)
    names = list(Wt)
    grads = block.loss_and_grads(out, torch.tensor(Gup, dtype=F64), [mt] + [Wt[k] for k in names])
    assert np.allclose(grads[0].numpy(), dm, rtol=1e-11, atol=1e-12)
    for k, gr in zip(names, grads[1:]):
        assert np.allclose(gr.numpy(), gW[k], rtol=1e-11, atol=1e-12), k


# ---- energy head (output step of Sec. 3.3): routed closed form ---------------------------------------
def test_energy_head_routed_closed_form():
    """Three atoms with different in- and out-degrees, hand-set head weights, every E_i written out.
    Edges (source -> target): 1->0, 2->0, 0->1, 0->2, 1->2, 0->2 is listed once; in-degrees 2, 1, 2,
    out-degrees 2, 2, 1.  Messages differ per edge so that summing by the source instead of the target,
    dropping b2 or b1, or applying w2 before the activation changes the result."""
    src = np.array([1, 2, 0, 0, 1])
    dst = np.array([0, 0, 1, 2, 2])                    # sorted by target as the graph builder emits them
    m = np.array([[0.5, -1.0], [2.0, 0.25], [-0.75, 1.5], [1.25, 0.5], [-0.5, -0.25]])
    W1 = np.array([[0.8, -0.6, 0.3], [0.2, 0.9, -1.1]])
    b1 = np.array([0.1, -0.2, 0.3])
    w2 = np.array([1.5, -0.7, 0.4])
    b2 = np.array([0.25])
    Wh = _t(dict(W1=W1, b1=b1, w2=w2, b2=b2))
    E, e_atom = energy.energy_head(torch.tensor(m, dtype=F64), dst, 3, Wh)
    h = {0: m[0] + m[1], 1: m[2], 2: m[3] + m[4]}        # messages ARRIVING at each atom
    ref = []
    for i in range(3):
        acc = float(b2[0])
        for o in range(3):
            pre = b1[o] + h[i][0] * W1[0, o] + h[i][1] * W1[1, o]
            acc += w2[o] * _silu(pre)
        ref.append(acc)
    assert np.allclose(e_atom.numpy(), ref, rtol=1e-14, atol=1e-14)
    assert abs(float(E) - sum(ref)) < 1e-13
    # the value a source-side sum would give is different on this input
    h_src = {0: m[2] + m[3], 1: m[0] + m[4], 2: m[1]}
    wrong = [float(b2[0]) + sum(w2[o] * _silu(b1[o] + h_src[i] @ W1[:, o]) for o in range(3)) for i in range(3)]
    assert not np.allclose(wrong, ref, rtol=1e-3)
    # an atom without in-edges contributes w2 . act(b1) + b2
    E4, e4 = energy.energy_head(torch.tensor(m, dtype=F64), dst, 4, Wh)
    lone = float(b2[0]) + sum(w2[o] * _silu(b1[o]) for o in range(3))
    assert abs(float(e4[3]) - lone) < 1e-14 and abs(float(E4) - sum(ref) - lone) < 1e-13


def test_energy_G_is_head_of_stack_on_recomputed_geometry():
    """energy_G = head(stack(features(pos))): compare with the pieces called one by one, and check that the
    force on an isolated-from-triplets coordinate comes out of the explicit chain rule through d only."""
    s = _tiny("G", seed=18)
    dims = s["dims"]
    W = _t(s["W"])
    Wh = _t({k: np.asarray(v, dtype=np.float64) for k, v in synth.weights_head(dims.emb, 4, seed=3, bias_scale=0.2).items()})
    m = torch.tensor(s["m"], dtype=F64)
    pos64 = torch.tensor(s["pos"], dtype=F64)
    E = energy.energy_G(pos64, s["src"], s["dst"], s["idx_kj"], s["idx_ji"], m, [W], Wh, dims)
    g = basis.rbf_gauss(s["d"], dims.cutoff, dims.num_radial)
    Y = basis.y_l0(s["cos_alpha"], dims.num_spherical)
    out = _block_G_loops(s["m"], g.numpy(), Y.numpy(), s["idx_kj"], s["idx_ji"], s["W"])
    n = len(s["pos"])
    ref = 0.0
    for i in range(n):
        h = np.zeros(dims.emb)
        for e in range(len(s["src"])):
            if s["dst"][e] == i:
                h += out[e]
        pre = h @ Wh["W1"].numpy() + Wh["b1"].numpy()
        ref += float(sum(Wh["w2"].numpy()[o] * _silu(pre[o]) for o in range(len(pre))) + Wh["b2"].numpy()[0])
    assert abs(float(E) - ref) < 1e-11 * max(1.0, abs(ref))
