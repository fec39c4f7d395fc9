"""Pins for the oracle's periodic radius graph (CPU only): a cell too large for any image reduces to
the open-boundary graph; an explicit replicated supercell with open boundaries gives the same
neighbourhoods; counting identities; the opposite-edge map negates offsets; the triplet exclusion
removes exactly the image that coincides with the target atom.
"""
import numpy as np
import torch

from oracle import basis, graph


def _cell_case(seed=0, n=7, a=4.0):
    rng = np.random.default_rng(seed)
    cell = np.array([[a, 0.0, 0.0], [0.3, a * 1.1, 0.0], [0.2, -0.4, a * 0.9]], dtype=np.float32)
    frac = rng.uniform(0, 1, (n, 3))
    pos = (frac @ cell.astype(np.float64)).astype(np.float32)
    return pos, np.array([0, n], dtype=np.int32), cell[None]


def test_huge_cell_reduces_to_open_boundaries():
    pos, gptr, cells = _cell_case(1)
    big = cells * 50.0
    s0, d0, r0 = graph.edges(pos, gptr, 3.0)
    s1, d1, o1, r1 = graph.edges_pbc(pos, gptr, big, 3.0, (1, 1, 1))
    assert np.array_equal(s0, s1) and np.array_equal(d0, d1) and np.array_equal(r0, r1) and not o1.any()
    k0 = graph.triplets(s0, d0, r0)
    k1 = graph.triplets(s1, d1, r1, o1)
    assert all(np.array_equal(a, b) for a, b in zip(k0, k1))


def test_matches_an_explicit_supercell():
    # replicate the cell 5x5x5 with open boundaries; the neighbourhood of every atom of the central copy
    # (as a set of (source atom, image) pairs) must be what edges_pbc finds
    pos, gptr, cells = _cell_case(2, n=5, a=3.4)
    cutoff, rep = 3.9, (2, 2, 2)
    s, d, o, rp = graph.edges_pbc(pos, gptr, cells, cutoff, rep)
    n = len(pos)
    images = [(a, b, c) for a in range(-2, 3) for b in range(-2, 3) for c in range(-2, 3)]
    cell64 = cells[0].astype(np.float64)
    big = np.concatenate([pos.astype(np.float64) + np.array(im) @ cell64 for im in images])
    centre = images.index((0, 0, 0))
    got = {(int(d[e]), int(s[e]), tuple(map(int, o[e]))) for e in range(len(s))}
    want = set()
    for i in range(n):
        dist = np.linalg.norm(big - big[centre * n + i], axis=1)
        assert np.abs(dist[dist > 0] - cutoff).min() > 1e-4          # no near-tie in this seed
        for q in np.nonzero(dist < cutoff)[0]:
            if q == centre * n + i:
                continue
            want.add((i, int(q % n), images[q // n]))
    assert got == want
    assert any(a == b for a, b, _ in got)                            # an atom sees its own image
    # edge vectors computed with the shifts have the same lengths as in the supercell
    shift = graph.edge_shifts(o, d, gptr, cells)
    dd, _, _ = basis.geometry(torch.tensor(pos, dtype=torch.float64), s, d, [], [], shift)
    for e in range(len(s)):
        im = images.index(tuple(map(int, o[e])))
        ref = np.linalg.norm(big[centre * n + d[e]] - big[im * n + s[e]])
        assert abs(float(dd[e]) - ref) < 1e-5      # positions are fp32


def test_ordering_counting_and_opposite_edges():
    pos, gptr, cells = _cell_case(3, n=6, a=3.6)
    s, d, o, rp = graph.edges_pbc(pos, gptr, cells, 3.8, (2, 2, 2))
    keys = [(int(d[e]), int(s[e]), *map(int, o[e])) for e in range(len(s))]
    assert keys == sorted(keys) and len(set(keys)) == len(keys)
    assert np.array_equal(np.diff(rp), np.bincount(d, minlength=len(pos)))
    sw = graph.reverse_edges(s, d, o)
    assert (sw >= 0).all() and np.array_equal(sw[sw], np.arange(len(s)))
    assert np.array_equal(o[sw], -o) and np.array_equal(s[sw], d)
    kj, ji, seg = graph.triplets(s, d, rp, o)
    deg = np.diff(rp).astype(np.int64)
    assert len(kj) == int((deg * (deg - 1)).sum())                   # symmetric graph: every edge loses exactly one
    # the excluded candidate is the opposite edge, nothing else
    for e in range(len(s)):
        j = s[e]
        cand = set(range(rp[j], rp[j + 1]))
        assert cand - set(kj[seg[e]:seg[e + 1]].tolist()) == {int(sw[e])}
    # open-boundary rule (atom index only) would remove more: images of atom i other than i itself stay in
    kj0, _, _ = graph.triplets(s, d, rp)
    assert len(kj0) < len(kj)


def test_cap_keeps_the_nearest_images():
    pos, gptr, cells = _cell_case(4, n=4, a=3.0)
    s, d, o, rp = graph.edges_pbc(pos, gptr, cells, 4.5, (2, 2, 2), max_neighbors=6)
    assert (np.diff(rp) == 6).all()
    sa, da, oa, rpa = graph.edges_pbc(pos, gptr, cells, 4.5, (2, 2, 2))
    shift = graph.edge_shifts(oa, da, gptr, cells)
    dist, _, _ = basis.geometry(torch.tensor(pos, dtype=torch.float64), sa, da, [], [], shift)
    dist = dist.numpy()
    for i in range(len(pos)):
        allr = np.sort(dist[rpa[i]:rpa[i + 1]])
        kept = {(int(s[e]), tuple(map(int, o[e]))) for e in range(rp[i], rp[i + 1])}
        full = {(int(sa[e]), tuple(map(int, oa[e]))): dist[e] for e in range(rpa[i], rpa[i + 1])}
        assert max(full[k] for k in kept) <= allr[5] + 1e-5
