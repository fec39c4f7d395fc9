"""Pins for the oracle's edge and triplet lists (CPU only).

Each check ties oracle/graph.py to something other than itself: a library
neighbour search in fp64, counting identities, brute force from the
definition, and symmetry properties of the definition (Sec. 3.1).
"""
import numpy as np
import pytest
from scipy.spatial import cKDTree

import synth
from oracle import graph


def _cfg1(seed=0):
    w = synth.get_workload("cfg1")
    pos, gptr = synth.make_positions(w, seed)
    return w, pos, gptr


def _small_slab(seed=0, n_graphs=2):
    pos, gptr = synth.slab_adsorbate_positions(n_graphs, 3, 3, 3, 5, seed=seed)
    return pos, gptr


def _pairs(src, dst):
    return set(zip(src.tolist(), dst.tolist()))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_edges_match_kdtree_fp64(seed):
    w, pos, gptr = _cfg1(seed)
    c = w.dims.cutoff
    src, dst, row_ptr = graph.edges(pos, gptr, c)
    p64 = pos.astype(np.float64)
    dall = np.sqrt(((p64[:, None] - p64[None]) ** 2).sum(-1))
    margin = np.abs(dall - c).min()
    assert margin > 1e-4, "generator produced a near-tie at the cutoff"
    tree = cKDTree(p64)
    ref = set()
    for i, nb in enumerate(tree.query_ball_point(p64, c)):
        for j in nb:
            if j != i:
                ref.add((j, i))
    assert _pairs(src, dst) == ref
    # order: by target, then source
    key = dst.astype(np.int64) * len(pos) + src
    assert np.all(np.diff(key) > 0)
    assert np.array_equal(np.bincount(dst, minlength=len(pos)), np.diff(row_ptr))


def test_edges_symmetric_without_cap_and_within_graph():
    pos, gptr = _small_slab()
    src, dst, _ = graph.edges(pos, gptr, 4.0)
    P = _pairs(src, dst)
    assert all((i, j) in P for (j, i) in P)
    gid = np.searchsorted(gptr, np.arange(len(pos)), side="right") - 1
    assert np.all(gid[src] == gid[dst])
    assert np.all(src != dst)


def test_edges_vectorised_equals_pair_loops():
    pos, gptr = _small_slab(seed=3)
    for cap in (0, 7):
        src, dst, _ = graph.edges(pos, gptr, 4.5, cap)
        assert list(zip(src.tolist(), dst.tolist())) == graph.edges_loops(pos, gptr, 4.5, cap)


def test_cap_keeps_nearest():
    pos, gptr = _small_slab(seed=1)
    c, M = 5.0, 6
    src, dst, row_ptr = graph.edges(pos, gptr, c, M)
    src0, dst0, row_ptr0 = graph.edges(pos, gptr, c, 0)
    p64 = pos.astype(np.float64)
    assert np.array_equal(np.diff(row_ptr), np.minimum(np.diff(row_ptr0), M))
    asym = 0
    for i in range(len(pos)):
        kept = src[row_ptr[i]:row_ptr[i + 1]]
        allc = src0[row_ptr0[i]:row_ptr0[i + 1]]
        assert set(kept) <= set(allc)
        dropped = np.setdiff1d(allc, kept)
        if len(dropped):
            dk = np.linalg.norm(p64[kept] - p64[i], axis=1).max()
            dd = np.linalg.norm(p64[dropped] - p64[i], axis=1).min()
            assert dk <= dd + 1e-6
    P = _pairs(src, dst)
    asym = sum((i, j) not in P for (j, i) in P)
    assert asym > 0, "the capped graph is expected to contain one-way edges"


def test_translation_and_permutation():
    rng = np.random.default_rng(5)
    pos, gptr = _small_slab(seed=2, n_graphs=1)
    pos = (np.round(pos * 1024) / 1024).astype(np.float32)       # exactly representable grid
    src, dst, _ = graph.edges(pos, gptr, 4.0, 5)
    shift = np.array([8.0, -16.0, 4.0], dtype=np.float32)         # keeps every coordinate exact
    src2, dst2, _ = graph.edges(pos + shift, gptr, 4.0, 5)
    assert np.array_equal(src, src2) and np.array_equal(dst, dst2)
    # uncapped: permuting atoms permutes the pair set (the cap's tie-break uses the index)
    perm = rng.permutation(len(pos))
    src3, dst3, _ = graph.edges(pos[perm], gptr, 4.0, 0)
    src4, dst4, _ = graph.edges(pos, gptr, 4.0, 0)
    assert {(perm[a], perm[b]) for a, b in _pairs(src3, dst3)} == _pairs(src4, dst4)


def test_triplets_against_definition_loops():
    w, pos, gptr = _cfg1()
    src, dst, row_ptr = graph.edges(pos, gptr, 3.0)
    idx_kj, idx_ji, seg = graph.triplets(src, dst, row_ptr)
    ref = graph.triplets_loops(list(zip(src.tolist(), dst.tolist())))
    assert sorted(zip(idx_kj.tolist(), idx_ji.tolist()), key=lambda p: (p[1], p[0])) == \
        sorted(ref, key=lambda p: (p[1], p[0]))
    assert list(zip(idx_kj.tolist(), idx_ji.tolist())) == sorted(ref, key=lambda p: (p[1], p[0]))


@pytest.mark.parametrize("cap", [0, 6])
def test_triplet_count_identities(cap):
    pos, gptr = _small_slab(seed=4)
    src, dst, row_ptr = graph.edges(pos, gptr, 5.0, cap)
    idx_kj, idx_ji, seg = graph.triplets(src, dst, row_ptr)
    T = len(idx_kj)
    P = _pairs(src, dst)
    indeg = np.diff(row_ptr)
    expect = sum(int(indeg[j]) - ((i, j) in P) for j, i in zip(src.tolist(), dst.tolist()))
    assert T == expect == seg[-1]
    if cap == 0:
        assert T == int((indeg * (indeg - 1)).sum())
    # validity and uniqueness
    assert np.all(dst[idx_kj] == src[idx_ji])
    assert np.all(src[idx_kj] != dst[idx_ji])
    assert len(set(zip(idx_kj.tolist(), idx_ji.tolist()))) == T
    assert np.array_equal(np.bincount(idx_ji, minlength=len(src)), np.diff(seg))


def test_triplets_complete_graph():
    n = 7
    rng = np.random.default_rng(0)
    pos = rng.uniform(0, 1, size=(n, 3)).astype(np.float32)
    src, dst, row_ptr = graph.edges(pos, np.array([0, n], dtype=np.int32), 10.0)
    assert len(src) == n * (n - 1)
    idx_kj, _, _ = graph.triplets(src, dst, row_ptr)
    assert len(idx_kj) == n * (n - 1) * (n - 2)


def test_workload_scale_orders_of_magnitude():
    # Sec. 2.2: edges are 1-2 orders above nodes, triplets 1-2 orders above edges
    w = synth.get_workload("cfg2")
    pos, gptr = synth.slab_adsorbate_positions(2, 4, 4, 4, 16, seed=0)
    src, dst, row_ptr = graph.edges(pos, gptr, w.dims.cutoff, w.max_neighbors)
    idx_kj, _, _ = graph.triplets(src, dst, row_ptr)
    assert 10 <= len(src) / len(pos) <= 100
    assert 10 <= len(idx_kj) / len(src) <= 100
