"""Pins for the oracle's geometry and basis functions (CPU only).

Closed forms, library routines (scipy.special), orthonormality integrals and
textbook constants stored in tests/golden/constants.txt.
"""
import math
import os

import numpy as np
import pytest
import scipy.special as sp
import torch

from oracle import basis

F64 = torch.float64
GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "constants.txt")) as fh:
    for line in fh:
        if line.strip() and not line.startswith("#"):
            name, val = line.split()[:2]
            GOLD[name] = float(val)


def test_envelope_closed_forms():
    x = torch.linspace(0, 1, 101, dtype=F64, requires_grad=True)
    u = basis.envelope(x, 5)
    assert abs(float(u[0].detach()) - 1) < 1e-15 and abs(float(u[-1].detach())) < 1e-13
    (du,) = torch.autograd.grad(u.sum(), x, create_graph=True)
    xd = x.detach()
    assert torch.allclose(du, -105 * xd ** 4 * (1 - xd) ** 2, atol=1e-12)
    (d2u,) = torch.autograd.grad(du.sum(), x)
    assert abs(float(du[-1])) < 1e-12 and abs(float(d2u[-1])) < 1e-11
    # explicit polynomial for p = 5
    assert torch.allclose(u.detach(), 1 - 21 * xd ** 5 + 35 * xd ** 6 - 15 * xd ** 7, atol=1e-14)


def test_spherical_bessel_vs_scipy():
    x = np.concatenate([np.linspace(0.02, 9.0, 400), np.linspace(9.0, 45.0, 400)])
    ours = basis.sph_jl(torch.tensor(x, dtype=F64), 8)
    for l in range(9):
        ref = sp.spherical_jn(l, x)
        err = np.abs(ours[l].numpy() - ref)
        scale = np.maximum(np.abs(ref), 1e-3 * np.abs(ref).max())
        assert (err / scale).max() < 1e-10, (l, (err / scale).max())
    # relative accuracy also where j_l is tiny (small argument, high order)
    xs = np.array([0.05, 0.2, 0.79, 1.5])
    ours = basis.sph_jl(torch.tensor(xs, dtype=F64), 6)
    for l in range(7):
        ref = sp.spherical_jn(l, xs)
        assert np.allclose(ours[l].numpy(), ref, rtol=1e-11, atol=0)
    assert np.allclose(ours[0].numpy(), np.sin(xs) / xs, rtol=1e-15)


def test_bessel_zeros():
    z = basis.bessel_zeros(7, 6)
    assert np.allclose(z[0], np.pi * np.arange(1, 7), rtol=1e-14)
    assert abs(z[1, 0] - GOLD["z_1_1"]) < 1e-12
    assert abs(z[1, 1] - GOLD["z_1_2"]) < 1e-12
    assert abs(z[1, 2] - GOLD["z_1_3"]) < 1e-12
    assert abs(z[2, 0] - GOLD["z_2_1"]) < 1e-12
    assert abs(z[2, 1] - GOLD["z_2_2"]) < 1e-12
    assert np.allclose(np.tan(z[1]), z[1], rtol=1e-9)
    for l in range(7):
        assert np.all(np.diff(z[l]) > 0)
        assert np.abs(sp.spherical_jn(l, z[l])).max() < 1e-12
        # n-th zero: exactly n-1 sign changes of j_l strictly inside (0, z_ln)
        for n in range(6):
            xs = np.linspace(1e-3, z[l, n] - 1e-6, 20000)
            sign_changes = int((np.diff(np.sign(sp.spherical_jn(l, xs))) != 0).sum())
            assert sign_changes == n


def test_y_l0_constants_and_scipy():
    c = torch.linspace(-1, 1, 41, dtype=F64)
    Y = basis.y_l0(c, 7).numpy()
    cn = c.numpy()
    assert np.allclose(Y[:, 0], GOLD["Y00"], rtol=1e-14)
    assert np.allclose(Y[:, 1], GOLD["Y10"] * cn, rtol=1e-14, atol=1e-16)
    assert np.allclose(Y[:, 2], GOLD["Y20"] * (3 * cn ** 2 - 1), rtol=1e-13, atol=1e-15)
    for l in range(7):
        ref = math.sqrt((2 * l + 1) / (4 * math.pi)) * sp.eval_legendre(l, cn)
        assert np.allclose(Y[:, l], ref, rtol=1e-12, atol=1e-14)


def test_y_l0_orthonormal_on_sphere():
    # 2 pi int_0^pi Y_l0 Y_l'0 sin(a) da = delta, by Gauss-Legendre quadrature in cos(a)
    nodes, wts = np.polynomial.legendre.leggauss(32)
    Y = basis.y_l0(torch.tensor(nodes, dtype=F64), 7).numpy()
    G = 2 * math.pi * (Y * wts[:, None]).T @ Y
    assert np.allclose(G, np.eye(7), atol=1e-12)


def _radial_quadrature(c, n=400):
    nodes, wts = np.polynomial.legendre.leggauss(n)
    d = 0.5 * c * (nodes + 1)
    return d, 0.5 * c * wts


@pytest.mark.parametrize("c", [5.0, 12.0])
def test_rbf_orthonormal(c):
    d, w = _radial_quadrature(c)
    dt = torch.tensor(d, dtype=F64)
    rbf = basis.rbf_bessel(dt, c, 6).numpy() / basis.envelope(dt / c).numpy()[:, None]
    G = (rbf * (w * d * d)[:, None]).T @ rbf
    assert np.allclose(G, np.eye(6), atol=1e-10)


@pytest.mark.parametrize("c", [5.0, 6.0])
def test_sbf_radial_orthonormal_and_cutoff(c):
    d, w = _radial_quadrature(c)
    dt = torch.tensor(d, dtype=F64)
    rad = basis.sbf_radial(dt, c, 7, 6).numpy() / basis.envelope(dt / c).numpy()[:, None, None]
    for l in range(7):
        G = (rad[:, l] * (w * d * d)[:, None]).T @ rad[:, l]
        assert np.allclose(G, np.eye(6), atol=1e-9), l
    edge = basis.sbf_radial(torch.tensor([c * (1 - 1e-9)], dtype=F64), c, 7, 6)
    assert float(edge.abs().max()) < 1e-12
    # explicit value against the library routine, l = 3, n = 2, with the envelope
    z = basis.bessel_zeros(7, 6)
    dd = 0.37 * c
    ref = (basis.envelope(torch.tensor(dd / c, dtype=F64)).item()
           * math.sqrt(2.0 / (c ** 3 * sp.spherical_jn(4, z[3, 1]) ** 2))
           * sp.spherical_jn(3, z[3, 1] * dd / c))
    got = basis.sbf_radial(torch.tensor([dd], dtype=F64), c, 7, 6)[0, 3, 1].item()
    assert abs(got - ref) < 1e-12 * max(1, abs(ref))


def test_sbf_layout_and_source_edge_distance():
    # sbf[t, l*R + n] = radial(d of edge kj)[l, n] * Y_l0(cos alpha_t)
    d = torch.tensor([1.0, 2.0, 3.5], dtype=F64)
    cosa = torch.tensor([0.3, -0.8], dtype=F64)
    idx_kj = np.array([2, 0])
    out = basis.sbf(d, cosa, idx_kj, 5.0, 7, 6).numpy()
    assert out.shape == (2, 42)
    z = basis.bessel_zeros(7, 6)
    for t, (e, ca) in enumerate(zip(idx_kj, cosa.numpy())):
        dd = float(d[e])
        for l in (0, 2, 6):
            for n in (0, 5):
                rad = (1 - 21 * (dd / 5) ** 5 + 35 * (dd / 5) ** 6 - 15 * (dd / 5) ** 7) \
                    * math.sqrt(2.0 / (125 * sp.spherical_jn(l + 1, z[l, n]) ** 2)) \
                    * sp.spherical_jn(l, z[l, n] * dd / 5)
                ang = math.sqrt((2 * l + 1) / (4 * math.pi)) * sp.eval_legendre(l, ca)
                assert abs(out[t, l * 6 + n] - rad * ang) < 1e-12


def test_gaussian_rbf():
    c, R = 6.0, 128
    mu = np.arange(R) / (R - 1)
    d = torch.tensor(mu[1:-1] * c, dtype=F64)
    g = basis.rbf_gauss(d, c, R).numpy()
    u = basis.envelope(torch.tensor(mu[1:-1], dtype=F64)).numpy()
    assert np.allclose(np.diag(g[:, 1:-1]), u, rtol=1e-13)
    # one grid step away: exp(-1/2)
    assert np.allclose(np.diag(g[:, 2:]), u * math.exp(-0.5), rtol=1e-10)
    assert g.shape == (R - 2, R)


def test_geometry_known_angles():
    # atoms: j at origin, i on +x, k on +y (right angle), k2 on -x (straight line)
    pos = torch.tensor([[0, 0, 0], [2, 0, 0], [0, 3, 0], [-1.5, 0, 0]], dtype=F64)
    # edges: 0: j->i (0->1), 1: k->j (2->0), 2: k2->j (3->0)
    src = np.array([0, 2, 3]); dst = np.array([1, 0, 0])
    d, unit, ca = basis.geometry(pos, src, dst, np.array([1, 2]), np.array([0, 0]))
    assert np.allclose(d.numpy(), [2, 3, 1.5])
    assert np.allclose(unit.numpy()[0], [1, 0, 0])
    assert np.allclose(ca.numpy(), [0.0, -1.0], atol=1e-15)
    # 60 degrees
    pos = torch.tensor([[0, 0, 0], [1, 0, 0], [0.5, math.sqrt(3) / 2, 0]], dtype=F64)
    _, _, ca = basis.geometry(pos, np.array([0, 2]), np.array([1, 0]), np.array([1]), np.array([0]))
    assert abs(float(ca[0]) - 0.5) < 1e-15
