"""Oracle: geometry and basis functions in fp64 (test infrastructure only).

The paper (Sec. 3.3) names a radial basis representation of the edge length
and a spherical basis representation of (d_kj, angle alpha_(kj,ji)) without
printing formulas; the functions here are the standard definitions of the
objects the workloads name:

  envelope  u(x) = 1 - (p+1)(p+2)/2 x^p + p(p+2) x^(p+1) - p(p+1)/2 x^(p+2)
  rbf_n(d)  = u(d/c) sqrt(2/c) sin(n pi d/c) / d,                 n = 1..R
  sbf_ln    = u(d/c) N_ln j_l(z_ln d/c) Y_l0(alpha),   l = 0..S-1, n = 1..R,
              z_ln the n-th positive zero of j_l,
              N_ln = sqrt(2 / (c^3 j_{l+1}(z_ln)^2)),
              Y_l0 = sqrt((2l+1)/(4 pi)) P_l(cos alpha),  flat index l*R + (n-1)
  g_n(d)    = u(d/c) exp(-((d/c - mu_n)/Delta)^2 / 2),  mu_n = n/(R-1), Delta = 1/(R-1)

alpha is the interior angle at atom j between the bonds j-i and j-k.
All torch functions are differentiable so that forces can be obtained by
automatic differentiation of the energy.
"""
import functools
import math

import numpy as np
import torch

F64 = torch.float64


# ----------------------------------------------------------------------------- geometry
def geometry(pos, src, dst, idx_kj, idx_ji, shift=None):
    """Edge lengths, unit vectors and triplet cosines.

    pos: torch [N,3] fp64.  Edge e runs src[e] -> dst[e]; unit[e] = (x_dst - x_src)/d_e.
    cos_alpha[t] = u_ji . u_jk with u_jk = (x_k - x_j)/d_kj = -unit[idx_kj[t]].
    shift [E,3] (periodic structures): the source atom of edge e sits at x_src + shift[e].
    """
    src = torch.as_tensor(np.asarray(src), dtype=torch.long)
    dst = torch.as_tensor(np.asarray(dst), dtype=torch.long)
    vec = pos[dst] - pos[src]
    if shift is not None:
        vec = vec - torch.as_tensor(np.asarray(shift), dtype=pos.dtype)
    d = torch.sqrt((vec * vec).sum(dim=1))
    unit = vec / d[:, None]
    kj = torch.as_tensor(np.asarray(idx_kj), dtype=torch.long)
    ji = torch.as_tensor(np.asarray(idx_ji), dtype=torch.long)
    cos_alpha = -(unit[ji] * unit[kj]).sum(dim=1)
    cos_alpha = torch.clamp(cos_alpha, -1.0, 1.0)
    return d, unit, cos_alpha


# ----------------------------------------------------------------------------- envelope
def envelope(x, p=5):
    a = -(p + 1) * (p + 2) / 2.0
    b = p * (p + 2) * 1.0
    c = -p * (p + 1) / 2.0
    return 1.0 + a * x ** p + b * x ** (p + 1) + c * x ** (p + 2)


# ----------------------------------------------------------------------------- spherical Bessel
def _double_factorial(n):
    r = 1.0
    while n > 1:
        r *= n
        n -= 2
    return r


def sph_jl(x, l_max):
    """Spherical Bessel functions j_0..j_lmax of a torch fp64 tensor x > 0.

    j_0 and j_1 in closed form.  For l >= 2: the ascending power series
        j_l(x) = x^l/(2l+1)!! * sum_k (-x^2/2)^k / (k! (2l+3)(2l+5)...(2l+2k+1))
    where x < l + 1 (upward recurrence loses accuracy there), otherwise the
    upward recurrence j_{l+1} = (2l+1)/x j_l - j_{l-1}.
    """
    out = [torch.sin(x) / x]
    if l_max >= 1:
        out.append(torch.sin(x) / (x * x) - torch.cos(x) / x)
    up_prev, up = out[0], out[-1]
    for l in range(2, l_max + 1):
        up_prev, up = up, (2 * l - 1) / x * up - up_prev
        # power series
        q = -0.5 * x * x
        term = torch.ones_like(x)
        ser = torch.ones_like(x)
        for k in range(1, 60):
            term = term * q / (k * (2 * l + 2 * k + 1))
            ser = ser + term
        ser = ser * x ** l / _double_factorial(2 * l + 1)
        out.append(torch.where(x < l + 1.0, ser, up))
    return out


def _jl_scalar(l, x):
    return float(sph_jl(torch.tensor([x], dtype=F64), l)[l][0])


@functools.lru_cache(maxsize=None)
def bessel_zeros(num_spherical, num_radial):
    """z[l][n-1] = n-th positive zero of j_l, by bisection between the zeros of
    j_{l-1}, which interlace them (z_{0,n} = n pi)."""
    n0 = num_radial + num_spherical
    prev = [math.pi * (n + 1) for n in range(n0)]
    zeros = [prev[:num_radial]]
    for l in range(1, num_spherical):
        cur = []
        for n in range(len(prev) - 1):
            a, b = prev[n], prev[n + 1]
            fa = _jl_scalar(l, a)
            for _ in range(200):
                mid = 0.5 * (a + b)
                fm = _jl_scalar(l, mid)
                if (fm > 0) == (fa > 0):
                    a, fa = mid, fm
                else:
                    b = mid
                if b - a < 1e-15 * b:
                    break
            cur.append(0.5 * (a + b))
        zeros.append(cur[:num_radial])
        prev = cur
    return np.asarray(zeros, dtype=np.float64)


def sbf_normalizer(zeros, cutoff):
    """N[l][n] = sqrt(2 / (c^3 j_{l+1}(z_ln)^2))."""
    return _sbf_normalizer_cached(zeros.shape[0], zeros.shape[1], float(cutoff))


@functools.lru_cache(maxsize=None)
def _sbf_normalizer_cached(num_spherical, num_radial, cutoff):
    zeros = bessel_zeros(num_spherical, num_radial)
    S, R = zeros.shape
    out = np.zeros_like(zeros)
    for l in range(S):
        for n in range(R):
            out[l, n] = math.sqrt(2.0 / (cutoff ** 3 * _jl_scalar(l + 1, float(zeros[l, n])) ** 2))
    return out


# ----------------------------------------------------------------------------- Legendre / Y_l0
def legendre(c, l_max):
    """P_0..P_lmax(c) by (l+1) P_{l+1} = (2l+1) c P_l - l P_{l-1}."""
    out = [torch.ones_like(c)]
    if l_max >= 1:
        out.append(c)
    for l in range(1, l_max):
        out.append(((2 * l + 1) * c * out[l] - l * out[l - 1]) / (l + 1))
    return out


def y_l0(cos_alpha, num_spherical):
    """[T, S] real spherical harmonics with m = 0."""
    P = legendre(cos_alpha, num_spherical - 1)
    cols = [math.sqrt((2 * l + 1) / (4 * math.pi)) * P[l] for l in range(num_spherical)]
    return torch.stack(cols, dim=1)


# ----------------------------------------------------------------------------- bases
def rbf_bessel(d, cutoff, num_radial, p=5):
    """[E, R]"""
    x = d / cutoff
    n = torch.arange(1, num_radial + 1, dtype=F64)
    return (envelope(x, p) * math.sqrt(2.0 / cutoff))[:, None] * torch.sin(n[None, :] * math.pi * x[:, None]) / d[:, None]


def sbf_radial(d, cutoff, num_spherical, num_radial, p=5):
    """Radial factor of the spherical basis per edge: [E, S, R] = u(d/c) N_ln j_l(z_ln d/c)."""
    zeros = bessel_zeros(num_spherical, num_radial)
    norm = sbf_normalizer(zeros, cutoff)
    x = d / cutoff
    u = envelope(x, p)
    rows = []
    for l in range(num_spherical):
        cols = []
        for n in range(num_radial):
            jl = sph_jl(float(zeros[l, n]) * x, l)[l]
            cols.append(u * float(norm[l, n]) * jl)
        rows.append(torch.stack(cols, dim=1))
    return torch.stack(rows, dim=1)


def sbf(d, cos_alpha, idx_kj, cutoff, num_spherical, num_radial, p=5):
    """[T, S*R]: radial factor taken at the source edge k->j, angular factor Y_l0(alpha_kji)."""
    rad = sbf_radial(d, cutoff, num_spherical, num_radial, p)          # [E,S,R]
    kj = torch.as_tensor(np.asarray(idx_kj), dtype=torch.long)
    Y = y_l0(cos_alpha, num_spherical)                                  # [T,S]
    out = rad[kj] * Y[:, :, None]
    return out.reshape(out.shape[0], num_spherical * num_radial)


def rbf_gauss(d, cutoff, num_radial, p=5):
    """[E, R] Gaussian radial basis with envelope."""
    x = d / cutoff
    mu = torch.arange(num_radial, dtype=F64) / (num_radial - 1)
    delta = 1.0 / (num_radial - 1)
    return envelope(x, p)[:, None] * torch.exp(-0.5 * ((x[:, None] - mu[None, :]) / delta) ** 2)
