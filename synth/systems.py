"""Seeded atom-position generators (fp32 output, open boundaries).

These stand in for OC20 structures: a metal slab with adsorbate atoms on top,
a dense box of atoms for the large-cutoff regime, and a small cube for the
tiny correctness case.  Each returns (pos[N,3] float32, graph_ptr[G+1] int32).
"""
import numpy as np


def _rejection_fill(rng, existing, n_new, draw, min_dist, max_tries=200000):
    """Sequentially draw points with draw(rng) and keep those at least
    min_dist away from every point kept so far (and from `existing`)."""
    pts = [np.asarray(p, dtype=np.float64) for p in existing]
    out = []
    tries = 0
    while len(out) < n_new:
        tries += 1
        if tries > max_tries:
            raise RuntimeError("rejection sampling did not converge")
        p = draw(rng)
        if pts:
            d = np.sqrt(((np.asarray(pts) - p) ** 2).sum(axis=1))
            if d.min() < min_dist:
                continue
        pts.append(p)
        out.append(p)
    return np.asarray(out, dtype=np.float64).reshape(n_new, 3)


def cube_positions(n_atoms=24, side=6.0, min_dist=0.9, seed=0):
    rng = np.random.default_rng(seed)
    pos = _rejection_fill(rng, [], n_atoms, lambda r: r.uniform(0.0, side, size=3), min_dist)
    return pos.astype(np.float32), np.array([0, n_atoms], dtype=np.int32)


def box_positions(n_atoms=1000, density=0.08, min_dist=0.9, seed=0):
    side = (n_atoms / density) ** (1.0 / 3.0)
    return cube_positions(n_atoms, side, min_dist, seed)


def _one_slab(rng, nx, ny, n_layers, n_ads, spacing=2.5, jitter=0.1, min_dist=0.9):
    """fcc (100) slab: square in-plane lattice of nearest-neighbour spacing
    `spacing`, layers spacing/sqrt(2) apart, every other layer shifted by half a
    cell; positions jittered uniformly; adsorbate atoms 1-3 A above the top layer."""
    dz = spacing / np.sqrt(2.0)
    slab = []
    for l in range(n_layers):
        shift = 0.5 * spacing * (l % 2)
        for a in range(nx):
            for b in range(ny):
                slab.append([a * spacing + shift, b * spacing + shift, l * dz])
    slab = np.asarray(slab, dtype=np.float64)
    slab += rng.uniform(-jitter, jitter, size=slab.shape)
    z_top = (n_layers - 1) * dz
    lx, ly = nx * spacing, ny * spacing

    def draw(r):
        return np.array([r.uniform(0.0, lx), r.uniform(0.0, ly), r.uniform(z_top + 1.0, z_top + 3.0)])

    ads = _rejection_fill(rng, list(slab), n_ads, draw, min_dist)
    return np.concatenate([slab, ads], axis=0)


def slab_adsorbate_positions(n_graphs=16, nx=4, ny=4, n_layers=4, n_ads=16, seed=0):
    rng = np.random.default_rng(seed)
    parts, ptr = [], [0]
    for _ in range(n_graphs):
        p = _one_slab(rng, nx, ny, n_layers, n_ads)
        parts.append(p)
        ptr.append(ptr[-1] + len(p))
    return np.concatenate(parts, axis=0).astype(np.float32), np.asarray(ptr, dtype=np.int32)


def make_positions(workload, seed=0):
    if workload.system == "cube":
        return cube_positions(*workload.system_args, seed=seed)
    if workload.system == "slab":
        return slab_adsorbate_positions(*workload.system_args, seed=seed)
    if workload.system == "box":
        return box_positions(*workload.system_args, seed=seed)
    raise ValueError(workload.system)
