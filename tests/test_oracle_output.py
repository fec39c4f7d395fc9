"""Pins for the oracle's output block (CPU only): special cases that reduce to a plain segment
sum computed independently with numpy, linearity, atom-permutation behaviour, central finite
differences of the gradient, and agreement of the stacked model with its parts.
"""
import numpy as np
import torch

import synth
from oracle import block, graph, output

F64 = torch.float64


def _t64(w):
    return {k: torch.tensor(v, dtype=F64) for k, v in w.items()}


def _case(seed=0, n_atoms=14, emb=6, out_emb=5, R=4, n_layers=2):
    pos, gptr = synth.cube_positions(n_atoms, 4.5, 0.9, seed=seed)
    src, dst, row_ptr = graph.edges(pos, gptr, 3.0)
    rng = np.random.default_rng(seed + 5)
    E = len(src)
    m = torch.tensor(rng.standard_normal((E, emb)), dtype=F64)
    rbf = torch.tensor(rng.standard_normal((E, R)), dtype=F64)
    W = _t64(synth.weights_out(emb, out_emb, R, n_layers, seed=seed + 1, bias_scale=0.3))
    return dict(pos=pos, src=src, dst=dst, m=m, rbf=rbf, W=W, n_atoms=n_atoms, E=E, emb=emb, out_emb=out_emb, R=R)


def test_reduces_to_a_weighted_segment_sum():
    # no dense layers, gate identically one (rbf = first unit vector, W_rbf row 0 = ones), W_up = identity:
    # P_i = sum over in-edges of m_e . w_final, checked against numpy's unbuffered add
    c = _case(n_layers=0, out_emb=6)
    W = dict(c["W"])
    W["W_rbf"] = torch.zeros((c["R"], c["emb"]), dtype=F64)
    W["W_rbf"][0] = 1.0
    W["W_up"] = torch.eye(c["emb"], dtype=F64)
    rbf = torch.zeros((c["E"], c["R"]), dtype=F64)
    rbf[:, 0] = 1.0
    got = output.output_block(c["m"], rbf, c["dst"], c["n_atoms"], W).numpy()
    ref = np.zeros(c["n_atoms"])
    np.add.at(ref, np.asarray(c["dst"]), c["m"].numpy() @ W["w_final"].numpy())
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)
    # atoms without in-edges contribute exactly zero
    deg = np.bincount(np.asarray(c["dst"]), minlength=c["n_atoms"])
    assert np.all(got[deg == 0] == 0.0)


def test_radial_gate_is_per_edge_and_per_feature():
    # one dense-free block: scaling column n of rbf scales the contribution routed through row n of W_rbf only
    c = _case(n_layers=0, out_emb=6)
    W = dict(c["W"])
    W["W_up"] = torch.eye(c["emb"], dtype=F64)
    base = output.output_block(c["m"], c["rbf"], c["dst"], c["n_atoms"], W)
    parts = []
    for n in range(c["R"]):
        Wn = dict(W)
        Wn["W_rbf"] = torch.zeros_like(W["W_rbf"])
        Wn["W_rbf"][n] = W["W_rbf"][n]
        parts.append(output.output_block(c["m"], c["rbf"], c["dst"], c["n_atoms"], Wn))
    assert torch.allclose(sum(parts), base, rtol=1e-12, atol=1e-12)
    # and the explicit double loop over edges and features
    ref = np.zeros(c["n_atoms"])
    m, rbf, Wr, wf = c["m"].numpy(), c["rbf"].numpy(), W["W_rbf"].numpy(), W["w_final"].numpy()
    for e in range(c["E"]):
        for f in range(c["emb"]):
            ref[c["dst"][e]] += m[e, f] * float(rbf[e] @ Wr[:, f]) * wf[f]
    assert np.allclose(base.numpy(), ref, rtol=1e-12, atol=1e-12)


def test_linear_in_final_vector_and_bias_path():
    c = _case()
    W2 = dict(c["W"])
    W2["w_final"] = 2.5 * c["W"]["w_final"]
    a = output.output_block(c["m"], c["rbf"], c["dst"], c["n_atoms"], c["W"])
    b = output.output_block(c["m"], c["rbf"], c["dst"], c["n_atoms"], W2)
    assert torch.allclose(b, 2.5 * a, rtol=1e-13, atol=1e-13)
    # zero messages: every atom gets the same bias-only value act(...act(b_0) W_1 + b_1...) . w_final
    z = output.output_block(torch.zeros_like(c["m"]), c["rbf"], c["dst"], c["n_atoms"], c["W"])
    u = block.act(c["W"]["b0"])
    u = block.act(u @ c["W"]["W1"] + c["W"]["b1"])
    assert torch.allclose(z, (u @ c["W"]["w_final"]).expand(c["n_atoms"]), rtol=1e-13, atol=1e-13)


def test_edge_order_does_not_matter_and_atoms_permute():
    c = _case(seed=3)
    rng = np.random.default_rng(0)
    pe = rng.permutation(c["E"])
    a = output.output_block(c["m"], c["rbf"], c["dst"], c["n_atoms"], c["W"])
    b = output.output_block(c["m"][pe], c["rbf"][pe], np.asarray(c["dst"])[pe], c["n_atoms"], c["W"])
    assert torch.allclose(a, b, rtol=1e-12, atol=1e-12)
    pa = rng.permutation(c["n_atoms"])           # atom i becomes atom pa[i]
    d2 = pa[np.asarray(c["dst"])]
    b = output.output_block(c["m"], c["rbf"], d2, c["n_atoms"], c["W"])
    assert torch.allclose(b[pa], a, rtol=1e-12, atol=1e-12)


def test_gradients_match_central_differences():
    c = _case(seed=2)
    gptr = np.array([0, 6, c["n_atoms"]])
    coef = torch.tensor([0.7, -1.3], dtype=F64)

    def loss(m, W):
        return (output.structure_energies(output.output_block(m, c["rbf"], c["dst"], c["n_atoms"], W), gptr) * coef).sum()

    m = c["m"].clone().requires_grad_(True)
    W = {k: v.clone().requires_grad_(True) for k, v in c["W"].items()}
    L = loss(m, W)
    grads = torch.autograd.grad(L, [m] + list(W.values()))
    rng = np.random.default_rng(1)
    for name, x, g in [("m", m, grads[0])] + [(k, W[k], grads[1 + i]) for i, k in enumerate(W)]:
        flat = x.detach().reshape(-1)
        for idx in rng.choice(flat.numel(), size=min(6, flat.numel()), replace=False):
            h = 1e-6
            def at(delta):
                y = flat.clone()
                y[idx] += delta
                if name == "m":
                    return float(loss(y.reshape(x.shape), c["W"]))
                W2 = dict(c["W"])
                W2[name] = y.reshape(x.shape)
                return float(loss(c["m"], W2))
            fd = (at(h) - at(-h)) / (2 * h)
            assert abs(fd - float(g.reshape(-1)[idx])) <= 1e-6 * max(1.0, abs(fd)), (name, idx)


def test_structure_energies_partition_the_atoms():
    p = torch.arange(10, dtype=F64)
    e = output.structure_energies(p, [0, 3, 3, 10])
    assert e.tolist() == [3.0, 0.0, 42.0]
