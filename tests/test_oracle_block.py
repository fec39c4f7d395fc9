"""Pins for the oracle's interaction blocks, energy and forces (CPU only).

Finite differences, physical invariances (Sec. 3.1: the block sees geometry only
through distances and angles), the partition property behind graph parallelism
(Sec. 2.2: local aggregates summed over processing units equal the global
aggregate), counting special cases and weight-routing special cases.
"""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import basis, block, energy, graph

F64 = torch.float64


def _t64(w):
    return {k: torch.tensor(v, dtype=F64) for k, v in w.items()}


def _tiny(variant="D", seed=0, cutoff=3.2, n_atoms=12):
    pos, gptr = synth.cube_positions(n_atoms, 4.5, 0.9, seed=seed)
    src, dst, row_ptr = graph.edges(pos, gptr, cutoff)
    idx_kj, idx_ji, seg = graph.triplets(src, dst, row_ptr)
    if variant == "D":
        dims = synth.BlockDims(variant="D", dtype="f32", emb=8, int_emb=5, basis_emb=3,
                               num_radial=4, num_spherical=3, cutoff=cutoff)
        W = _t64(synth.weights_D(dims, seed=seed + 1, bias_scale=0.2))
    else:
        dims = synth.BlockDims(variant="G", dtype="f32", emb=8, int_emb=5, emb_rbf=3, emb_cbf=4,
                               emb_bil=6, num_radial=7, num_spherical=3, cutoff=cutoff)
        W = _t64(synth.weights_G(dims, seed=seed + 1))
    m, gup = synth.edge_embeddings(len(src), dims.emb, seed=seed + 2)
    return dict(pos=pos, gptr=gptr, src=src, dst=dst, row_ptr=row_ptr, idx_kj=idx_kj, idx_ji=idx_ji,
                seg=seg, dims=dims, W=W, m=torch.tensor(m, dtype=F64), gup=torch.tensor(gup, dtype=F64))


def _features(s, pos64):
    dims = s["dims"]
    d, unit, ca = basis.geometry(pos64, s["src"], s["dst"], s["idx_kj"], s["idx_ji"])
    if dims.variant == "D":
        rbf = basis.rbf_bessel(d, dims.cutoff, dims.num_radial)
        sbf = basis.sbf(d, ca, s["idx_kj"], dims.cutoff, dims.num_spherical, dims.num_radial)
        return rbf, sbf
    return basis.rbf_gauss(d, dims.cutoff, dims.num_radial), basis.y_l0(ca, dims.num_spherical)


def _run(s, pos64, m=None, W=None):
    f1, f2 = _features(s, pos64)
    m = s["m"] if m is None else m
    W = s["W"] if W is None else W
    fn = block.block_D if s["dims"].variant == "D" else block.block_G
    return fn(m, f1, f2, s["idx_kj"], s["idx_ji"], W)


@pytest.mark.parametrize("variant", ["D", "G"])
def test_gradients_match_central_differences(variant):
    s = _tiny(variant)
    assert len(s["idx_kj"]) > 50
    pos64 = torch.tensor(s["pos"], dtype=F64)
    f1, f2 = _features(s, pos64)
    fn = block.block_D if variant == "D" else block.block_G
    leaves = {"m": s["m"].clone().requires_grad_(True), "f1": f1.clone().requires_grad_(True),
              "f2": f2.clone().requires_grad_(True)}
    for k, v in s["W"].items():
        leaves[k] = v.clone().requires_grad_(True)

    def loss():
        W = {k: leaves[k] for k in s["W"]}
        out = fn(leaves["m"], leaves["f1"], leaves["f2"], s["idx_kj"], s["idx_ji"], W)
        return (out * s["gup"]).sum()

    names = list(leaves)
    grads = torch.autograd.grad(loss(), [leaves[n] for n in names])
    rng = np.random.default_rng(0)
    h = 1e-6
    for name, g in zip(names, grads):
        t = leaves[name]
        flat = t.detach().view(-1)
        for idx in rng.choice(flat.numel(), size=min(64, flat.numel()), replace=False):
            old = float(flat[idx])
            with torch.no_grad():
                flat[idx] = old + h; lp = float(loss())
                flat[idx] = old - h; lm = float(loss())
                flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = float(g.reshape(-1)[idx])
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (name, int(idx), fd, an)


def _random_rotation(rng):
    q, r = np.linalg.qr(rng.standard_normal((3, 3)))
    q = q * np.sign(np.diag(r))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    return q


@pytest.mark.parametrize("variant", ["D", "G"])
def test_rotation_translation_invariance(variant):
    s = _tiny(variant, seed=1)
    rng = np.random.default_rng(3)
    pos64 = torch.tensor(s["pos"], dtype=F64)
    out = _run(s, pos64)
    Q = torch.tensor(_random_rotation(rng), dtype=F64)
    shift = torch.tensor(rng.uniform(-5, 5, 3), dtype=F64)
    out2 = _run(s, pos64 @ Q.T + shift)
    assert float((out - out2).abs().max()) < 1e-11 * float(out.abs().max())
    # a reflection must also leave it unchanged (only distances and cos(angle) enter)
    out3 = _run(s, pos64 * torch.tensor([1.0, -1.0, 1.0], dtype=F64))
    assert float((out - out3).abs().max()) < 1e-11 * float(out.abs().max())


@pytest.mark.parametrize("variant", ["D", "G"])
def test_atom_permutation_equivariance(variant):
    s = _tiny(variant, seed=2)
    rng = np.random.default_rng(4)
    n = len(s["pos"])
    perm = rng.permutation(n)                   # new atom a is old atom perm[a]
    inv = np.argsort(perm)
    pos2 = s["pos"][perm]
    src2, dst2, row2 = graph.edges(pos2, s["gptr"], s["dims"].cutoff)
    kj2, ji2, _ = graph.triplets(src2, dst2, row2)
    old_id = {(a, b): e for e, (a, b) in enumerate(zip(s["src"].tolist(), s["dst"].tolist()))}
    emap = np.array([old_id[(perm[a], perm[b])] for a, b in zip(src2.tolist(), dst2.tolist())])
    assert sorted(emap.tolist()) == list(range(len(s["src"])))
    s2 = dict(s, pos=pos2, src=src2, dst=dst2, idx_kj=kj2, idx_ji=ji2)
    out = _run(s, torch.tensor(s["pos"], dtype=F64))
    out2 = _run(s2, torch.tensor(pos2, dtype=F64), m=s["m"][emap])
    assert float((out[emap] - out2).abs().max()) < 1e-11 * float(out.abs().max())
    assert inv is not None


def test_aggregate_counts_and_linearity():
    s = _tiny("D", seed=3)
    E, T = len(s["src"]), len(s["idx_kj"])
    ones_x = torch.ones((E, 5), dtype=F64)
    ones_s = torch.ones((T, 5), dtype=F64)
    a = block.triplet_aggregate_D(ones_x, ones_s, s["idx_kj"], s["idx_ji"], E)
    assert torch.equal(a[:, 0], torch.tensor(np.diff(s["seg"]), dtype=F64))
    rng = np.random.default_rng(0)
    x = torch.tensor(rng.standard_normal((E, 5)), dtype=F64)
    sv = torch.tensor(rng.standard_normal((T, 5)), dtype=F64)
    a1 = block.triplet_aggregate_D(x, sv, s["idx_kj"], s["idx_ji"], E)
    a2 = block.triplet_aggregate_D(x, 2 * sv, s["idx_kj"], s["idx_ji"], E)
    assert torch.allclose(a2, 2 * a1, rtol=1e-14)
    # brute-force definition on a few edges
    for e in rng.choice(E, 5, replace=False):
        ref = np.zeros(5)
        for t in range(T):
            if s["idx_ji"][t] == e:
                ref += x[s["idx_kj"][t]].numpy() * sv[t].numpy()
        assert np.allclose(a1[e].numpy(), ref, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("variant", ["D", "G"])
def test_partition_property(variant):
    # Sec. 2.2: each unit aggregates its own triplet subset; the sum over units is the full aggregate
    s = _tiny(variant, seed=4)
    E, T = len(s["src"]), len(s["idx_kj"])
    rng = np.random.default_rng(1)
    x = torch.tensor(rng.standard_normal((E, 5)), dtype=F64)
    width = 5 if variant == "D" else 4
    f = torch.tensor(rng.standard_normal((T, width)), dtype=F64)
    agg = block.triplet_aggregate_D if variant == "D" else block.triplet_aggregate_G
    full = agg(x, f, s["idx_kj"], s["idx_ji"], E)
    owner = rng.integers(0, 3, size=T)
    parts = sum(agg(x, f[owner == p], s["idx_kj"][owner == p], s["idx_ji"][owner == p], E) for p in range(3))
    assert torch.allclose(full, parts, rtol=1e-13, atol=1e-13)


def test_variant_G_reduces_to_segment_sum():
    s = _tiny("G", seed=5)
    E, T = len(s["src"]), len(s["idx_kj"])
    rng = np.random.default_rng(2)
    x = rng.standard_normal((E, 5))
    Y00 = 1.0 / (2.0 * math.sqrt(math.pi))
    y = torch.full((T, 1), Y00, dtype=F64)
    A = block.triplet_aggregate_G(torch.tensor(x, dtype=F64), y, s["idx_kj"], s["idx_ji"], E)
    ref = np.zeros((E, 5))
    np.add.at(ref, s["idx_ji"], x[s["idx_kj"]])
    assert np.allclose(A[:, 0, :].numpy(), Y00 * ref, rtol=1e-13, atol=1e-13)
    # outer-product structure: A[e, c, f] for two different c differ only by the y factor
    y2 = torch.tensor(rng.standard_normal((T, 2)), dtype=F64)
    A2 = block.triplet_aggregate_G(torch.tensor(x, dtype=F64), y2, s["idx_kj"], s["idx_ji"], E)
    for c in range(2):
        ref = np.zeros((E, 5))
        np.add.at(ref, s["idx_ji"], y2[:, c:c + 1].numpy() * x[s["idx_kj"]])
        assert np.allclose(A2[:, c, :].numpy(), ref, rtol=1e-13, atol=1e-13)


def _silu(v):
    return v / (1.0 + np.exp(-v))


def test_block_D_weight_routing():
    """All weights zero except single entries: the output must be the closed form
    that follows from y = x @ W with W[in, out], SiLU activations and the skip."""
    s = _tiny("D", seed=6)
    dims = s["dims"]
    E = len(s["src"])
    pos64 = torch.tensor(s["pos"], dtype=F64)
    rbf, sbf = _features(s, pos64)
    Z = {k: torch.zeros_like(v) for k, v in s["W"].items()}
    m = s["m"]
    out = block.block_D(m, rbf, sbf, s["idx_kj"], s["idx_ji"], Z)
    assert torch.allclose(out, m, atol=1e-15)          # everything off: only the skip survives
    # route input feature 2 -> x_ji feature 5 (weight 0.7), then feature 5 -> lin output 1
    W = {k: v.clone() for k, v in Z.items()}
    W["W_ji"][2, 5] = 0.7
    W["b_ji"][5] = 0.1
    W["W_lin"][5, 1] = 1.3
    out = block.block_D(m, rbf, sbf, s["idx_kj"], s["idx_ji"], W).numpy()
    mn = m.numpy()
    ref = mn.copy()
    ref[:, 1] += _silu(1.3 * _silu(0.7 * mn[:, 2] + 0.1))
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-13)
    # triplet path: m feature 0 -> x_kj feature 3, gate from rbf channel 1, down to int feature 4,
    # sbf channel (l=1, n=2) -> basis 2 -> int feature 4, up to emb feature 6, lin 6 -> 7
    W = {k: v.clone() for k, v in Z.items()}
    W["W_kj"][0, 3] = 0.9
    W["W_rbf1"][1, 0] = 1.1
    W["W_rbf2"][0, 3] = 0.8
    W["W_down"][3, 4] = 1.2
    R = dims.num_radial
    W["W_sbf1"][1 * R + 1, 2] = 0.6
    W["W_sbf2"][2, 4] = 1.5
    W["W_up"][4, 6] = 0.5
    W["W_lin"][6, 7] = 1.0
    out = block.block_D(m, rbf, sbf, s["idx_kj"], s["idx_ji"], W).numpy()
    xk = _silu(1.2 * (_silu(0.9 * mn[:, 0]) * (1.1 * 0.8 * rbf[:, 1].numpy())))
    a = np.zeros(E)
    np.add.at(a, s["idx_ji"], xk[s["idx_kj"]] * (0.6 * 1.5 * sbf[:, 1 * R + 1].numpy()))
    ref = mn.copy()
    ref[:, 7] += _silu(1.0 * _silu(0.5 * a))
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)


def test_block_G_weight_routing():
    s = _tiny("G", seed=7)
    dims = s["dims"]
    E = len(s["src"])
    pos64 = torch.tensor(s["pos"], dtype=F64)
    g, Y = _features(s, pos64)
    Z = {k: torch.zeros_like(v) for k, v in s["W"].items()}
    m = s["m"]
    mn = m.numpy()
    W = {k: v.clone() for k, v in Z.items()}
    W["W_skip"][1, 2] = 0.4
    out = block.block_G(m, g, Y, s["idx_kj"], s["idx_ji"], W).numpy()
    ref = np.zeros_like(mn)
    ref[:, 2] = _silu(0.4 * mn[:, 1])
    assert np.allclose(out, ref / math.sqrt(2.0), rtol=1e-13, atol=1e-14)
    # triplet path
    W = {k: v.clone() for k, v in Z.items()}
    W["W_ba"][0, 3] = 0.9
    W["W_rbfS"][2, 1] = 1.1
    W["W_rbfB"][1, 3] = 0.8
    W["W_down"][3, 4] = 1.2
    W["W_c"][2, 5, 1] = 0.7          # l = 2, radial channel 5 -> cbf channel 1
    W["W_bil"][1, 4, 2] = 1.4        # (cbf 1, trip 4) -> bil 2
    W["W_up"][2, 6] = 0.5
    out = block.block_G(m, g, Y, s["idx_kj"], s["idx_ji"], W).numpy()
    gn, Yn = g.numpy(), Y.numpy()
    x = _silu(1.2 * (_silu(0.9 * mn[:, 0]) * (1.1 * 0.8 * gn[:, 2])))
    yt = Yn[:, 2] * (0.7 * gn[s["idx_kj"], 5])
    A = np.zeros(E)
    np.add.at(A, s["idx_ji"], yt * x[s["idx_kj"]])
    ref = np.zeros_like(mn)
    ref[:, 6] = _silu(0.5 * 1.4 * A)
    assert np.allclose(out, ref / math.sqrt(2.0), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("variant", ["D", "G"])
def test_forces_are_negative_energy_gradient(variant):
    # Sec. 3.2: f = -grad_x E
    s = _tiny(variant, seed=8)
    dims = s["dims"]
    Wh = _t64(synth.weights_head(dims.emb, 7, seed=11, bias_scale=0.1))
    W2 = _t64(synth.weights_D(dims, 21, 0.1) if variant == "D" else synth.weights_G(dims, 21))
    efn = energy.energy_D if variant == "D" else energy.energy_G
    args = (s["src"], s["dst"], s["idx_kj"], s["idx_ji"], s["m"], [s["W"], W2], Wh, dims)
    E0, f = energy.forces(efn, s["pos"], *args)
    pos = s["pos"].astype(np.float64)
    h = 1e-4
    rng = np.random.default_rng(0)
    for a, c in [(a, c) for a in range(len(pos)) for c in range(3)]:      # every coordinate
        pp, pm = pos.copy(), pos.copy()
        pp[a, c] += h; pm[a, c] -= h
        with torch.no_grad():
            ep = float(efn(torch.tensor(pp, dtype=F64), *args))
            em = float(efn(torch.tensor(pm, dtype=F64), *args))
        fd = -(ep - em) / (2 * h)
        assert abs(fd - f[a, c]) <= 1e-6 * max(np.abs(f).max(), 1e-3), (a, c, fd, f[a, c])
    scale = np.abs(f).max()
    assert scale > 1e-6
    assert np.abs(f.sum(axis=0)).max() < 1e-12 * max(1, scale) * len(pos)
    assert np.abs(np.cross(pos, f).sum(axis=0)).max() < 1e-11 * max(1, scale) * len(pos)
    # forces rotate with the frame
    Q = _random_rotation(rng)
    E1, f1 = energy.forces(efn, pos @ Q.T, *args)
    assert abs(E1 - E0) < 1e-11 * max(1, abs(E0))
    assert np.abs(f1 - f @ Q.T).max() < 1e-10 * max(1, scale)


# ---- variant G with the radial factor at the target edge ---------------------------------------
def test_radial_at_target_matches_brute_force_loops():
    # the defining sum written as explicit loops over edges, their triplets, l, c and f
    s = _tiny("G", seed=4, n_atoms=9)
    E = len(s["src"])
    pos64 = torch.tensor(s["pos"], dtype=F64)
    g, Y = _features(s, pos64)
    W = s["W"]
    out = block.block_G(s["m"], g, Y, s["idx_kj"], s["idx_ji"], W, radial_at_target=True).numpy()
    m, gn, Yn = s["m"].numpy(), g.numpy(), Y.numpy()
    Wn = {k: v.numpy() for k, v in W.items()}
    x = _silu(m @ Wn["W_ba"]) * ((gn @ Wn["W_rbfS"]) @ Wn["W_rbfB"])
    x = _silu(x @ Wn["W_down"])
    S, R, C = Wn["W_c"].shape
    F = x.shape[1]
    z = np.zeros((E, Wn["W_bil"].shape[2]))
    for e in range(E):
        Rad_e = np.array([[sum(gn[e, n] * Wn["W_c"][l, n, c] for n in range(R)) for c in range(C)] for l in range(S)])
        A = np.zeros((C, F))
        for t in np.nonzero(np.asarray(s["idx_ji"]) == e)[0]:
            y = np.array([sum(Yn[t, l] * Rad_e[l, c] for l in range(S)) for c in range(C)])
            A += np.outer(y, x[s["idx_kj"][t]])
        z[e] = np.einsum("cf,cfo->o", A, Wn["W_bil"])
    ref = (_silu(m @ Wn["W_skip"]) + _silu(z @ Wn["W_up"])) / math.sqrt(2.0)
    assert np.allclose(out, ref, rtol=1e-11, atol=1e-12)


def test_radial_at_target_equals_source_form_when_all_edges_share_a_length():
    # if every edge carries the same radial basis row, it does not matter which edge of a triplet supplies it
    s = _tiny("G", seed=5)
    pos64 = torch.tensor(s["pos"], dtype=F64)
    g, Y = _features(s, pos64)
    g_same = g[3].expand_as(g).clone()
    a = block.block_G(s["m"], g_same, Y, s["idx_kj"], s["idx_ji"], s["W"], radial_at_target=False)
    b = block.block_G(s["m"], g_same, Y, s["idx_kj"], s["idx_ji"], s["W"], radial_at_target=True)
    assert torch.allclose(a, b, rtol=1e-12, atol=1e-13)
    # and with the real basis the two readings differ
    c = block.block_G(s["m"], g, Y, s["idx_kj"], s["idx_ji"], s["W"], radial_at_target=True)
    d = block.block_G(s["m"], g, Y, s["idx_kj"], s["idx_ji"], s["W"], radial_at_target=False)
    assert not torch.allclose(c, d, rtol=1e-3, atol=1e-6)


def test_radial_at_target_factorises_and_differentiates():
    # the radial factor leaves the sum over k: A_e = Rad_e^T (sum_t Y(t) (x) x_kj), the re-association
    # the fast path uses; plus central differences of the gradient w.r.t. the radial basis
    s = _tiny("G", seed=6)
    E = len(s["src"])
    pos64 = torch.tensor(s["pos"], dtype=F64)
    g, Y = _features(s, pos64)
    W = s["W"]
    x = block.act(block.act(s["m"] @ W["W_ba"]) * ((g @ W["W_rbfS"]) @ W["W_rbfB"]) @ W["W_down"])
    Rad = torch.einsum("en,lnc->elc", g, W["W_c"])
    B1 = torch.zeros((E, Y.shape[1], x.shape[1]), dtype=F64)
    B1.index_add_(0, torch.as_tensor(np.asarray(s["idx_ji"]), dtype=torch.long),
                  Y[:, :, None] * x[torch.as_tensor(np.asarray(s["idx_kj"]), dtype=torch.long)][:, None, :])
    A = torch.einsum("elc,elf->ecf", Rad, B1)
    z = torch.einsum("ecf,cfo->eo", A, W["W_bil"])
    ref = (block.act(s["m"] @ W["W_skip"]) + block.act(z @ W["W_up"])) / math.sqrt(2.0)
    out = block.block_G(s["m"], g, Y, s["idx_kj"], s["idx_ji"], W, radial_at_target=True)
    assert torch.allclose(out, ref, rtol=1e-12, atol=1e-13)
    gq = g.clone().requires_grad_(True)
    L = (block.block_G(s["m"], gq, Y, s["idx_kj"], s["idx_ji"], W, radial_at_target=True) * s["gup"]).sum()
    (grad,) = torch.autograd.grad(L, gq)
    rng = np.random.default_rng(2)
    for idx in rng.choice(g.numel(), size=64, replace=False):
        h = 1e-6
        def at(delta):
            y = g.clone().reshape(-1)
            y[idx] += delta
            return float((block.block_G(s["m"], y.reshape(g.shape), Y, s["idx_kj"], s["idx_ji"], W, radial_at_target=True) * s["gup"]).sum())
        fd = (at(h) - at(-h)) / (2 * h)
        assert abs(fd - float(grad.reshape(-1)[idx])) <= 1e-6 * max(1.0, abs(fd))


# ---- symmetric message passing ------------------------------------------------------------------
def test_reverse_edges_is_an_involution_and_respects_the_cap():
    pos, gptr = synth.cube_positions(14, 4.5, 0.9, seed=8)
    src, dst, _ = graph.edges(pos, gptr, 3.2)                 # no cap: every edge has its opposite
    sw = graph.reverse_edges(src, dst)
    assert (sw >= 0).all() and np.array_equal(sw[sw], np.arange(len(src)))
    assert np.array_equal(np.asarray(src)[sw], dst) and np.array_equal(np.asarray(dst)[sw], src)
    src, dst, _ = graph.edges(pos, gptr, 3.2, 3)              # cap 3: some edges lose their opposite
    sw = graph.reverse_edges(src, dst)
    pairs = set(zip(map(int, src), map(int, dst)))
    for e in range(len(src)):
        has = (int(dst[e]), int(src[e])) in pairs
        assert (sw[e] >= 0) == has
        if has:
            assert src[sw[e]] == dst[e] and dst[sw[e]] == src[e] and sw[sw[e]] == e
    assert (sw < 0).any()


def test_symmetric_block_matches_explicit_loops_and_gradients():
    s = _tiny("G", seed=9, n_atoms=10)
    E = len(s["src"])
    pos64 = torch.tensor(s["pos"], dtype=F64)
    g, Y = _features(s, pos64)
    rng = np.random.default_rng(3)
    W = dict(s["W"])
    W["W_up_ac"] = torch.tensor(rng.uniform(-0.4, 0.4, tuple(W["W_up"].shape)), dtype=F64)
    # drop the opposite of a few edges by hand to exercise the "absent" branch
    sw = graph.reverse_edges(s["src"], s["dst"])
    sw[[0, 5, 7]] = -1
    out = block.block_G(s["m"], g, Y, s["idx_kj"], s["idx_ji"], W, id_swap=sw).numpy()
    # explicit: recompute z exactly as the non-symmetric block does, then couple edge by edge
    Wz = {k: v for k, v in W.items() if k != "W_up_ac"}
    Wz = dict(Wz)
    x = block.act(block.act(s["m"] @ W["W_ba"]) * ((g @ W["W_rbfS"]) @ W["W_rbfB"]) @ W["W_down"])
    Rad = torch.einsum("en,lnc->elc", g, W["W_c"])
    kj = torch.as_tensor(np.asarray(s["idx_kj"]), dtype=torch.long)
    y = torch.einsum("tl,tlc->tc", Y, Rad[kj])
    A = block.triplet_aggregate_G(x, y, s["idx_kj"], s["idx_ji"], E)
    z = torch.einsum("ecf,cfo->eo", A, W["W_bil"]).numpy()
    mn = s["m"].numpy()
    ref = np.zeros_like(mn)
    for e in range(E):
        x3 = _silu(z[e] @ W["W_up"].numpy())
        if sw[e] >= 0:
            x3 = x3 + _silu(z[sw[e]] @ W["W_up_ac"].numpy())
        x3 = x3 / math.sqrt(2.0)
        ref[e] = (_silu(mn[e] @ W["W_skip"].numpy()) + x3) / math.sqrt(2.0)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    # central differences w.r.t. the new weight and the input messages
    def loss(m_, Wac):
        W2 = dict(W)
        W2["W_up_ac"] = Wac
        return (block.block_G(m_, g, Y, s["idx_kj"], s["idx_ji"], W2, id_swap=sw) * s["gup"]).sum()
    mq, wq = s["m"].clone().requires_grad_(True), W["W_up_ac"].clone().requires_grad_(True)
    gm, gw = torch.autograd.grad(loss(mq, wq), [mq, wq])
    for name, x0, gr in (("m", s["m"], gm), ("W_up_ac", W["W_up_ac"], gw)):
        for idx in rng.choice(x0.numel(), size=min(64, x0.numel()), replace=False):
            h = 1e-6
            def at(delta):
                yv = x0.clone().reshape(-1)
                yv[idx] += delta
                yv = yv.reshape(x0.shape)
                return float(loss(yv, W["W_up_ac"]) if name == "m" else loss(s["m"], yv))
            fd = (at(h) - at(-h)) / (2 * h)
            assert abs(fd - float(gr.reshape(-1)[idx])) <= 1e-6 * max(1.0, abs(fd)), name
