"""Oracle: radius graph and triplet enumeration (test infrastructure only).

Edges follow the paper's graph definition (Sec. 3.1, "Inputs and Outputs"):
each target atom t receives an edge from every source atom s of the same
structure within the cutoff distance.  Triplets follow the same section and
the sum in the message-update equation of Sec. 3.3: for an edge j->i, every
edge k->j with k != i.

Readings where the paper is silent:
  * "within a distance" is taken as strictly less than the cutoff;
  * the distance test is the fp32 expression
        d2 = fl(fl(fl(dx*dx) + fl(dy*dy)) + fl(dz*dz)),  dx = fl(x_i - x_j)
    compared with fl(c*c), so that any implementation can reproduce the edge
    set bit for bit;
  * an optional neighbour cap keeps, per target atom, the M sources with the
    smallest key (bit pattern of d2, source index);
  * open boundaries (no periodic images) unless the *_pbc functions are used;
  * output order: edges by (target, source); triplets by (edge j->i, edge k->j).

Periodic structures (edges_pbc): the source of an edge may be a periodic image of an atom,
x_src + n0 a0 + n1 a1 + n2 a2 with integer n (the edge's cell offset) and lattice vectors a
(rows of the structure's cell).  Every image with |n_a| <= rep[a] is tested with the same fp32
predicate on the shifted source position, shift component = fl(fl(fl(n0 a0) + fl(n1 a1)) + fl(n2 a2));
the atom itself (n = 0) is excluded, its own images are not.  Edges are ordered by (target,
source, n0, n1, n2); the cap key is (bit pattern of d2, source, n0, n1, n2).  A triplet
k->j->i is excluded only if k's image coincides with atom i: same atom and opposite offsets.
"""
import numpy as np


def pair_d2_f32(pos, i, js):
    """fp32 squared distance between atom i and atoms js, each operation rounded to fp32."""
    p = pos.astype(np.float32, copy=False)
    dx = p[i, 0] - p[js, 0]
    dy = p[i, 1] - p[js, 1]
    dz = p[i, 2] - p[js, 2]
    # numpy evaluates float32 arrays op by op, so no fused multiply-add can occur
    return (dx * dx + dy * dy) + dz * dz


def edges(pos, graph_ptr, cutoff, max_neighbors=0):
    """Directed edge list of the radius graph.

    Returns src[E], dst[E] (int32, edge e goes src[e] -> dst[e]) sorted by
    (dst, src), and row_ptr[N+1] (int32) with the in-edges of atom i at
    row_ptr[i]:row_ptr[i+1].
    """
    pos = np.ascontiguousarray(pos, dtype=np.float32)
    n = pos.shape[0]
    c = np.float32(cutoff)
    c2 = np.float32(c * c)
    src_l, dst_l = [], []
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    for g in range(len(graph_ptr) - 1):
        lo, hi = int(graph_ptr[g]), int(graph_ptr[g + 1])
        for i in range(lo, hi):
            js = np.arange(lo, hi, dtype=np.int64)
            js = js[js != i]
            d2 = pair_d2_f32(pos, i, js)
            keep = d2 < c2
            js, d2 = js[keep], d2[keep]
            if max_neighbors > 0 and len(js) > max_neighbors:
                bits = d2.view(np.uint32).astype(np.uint64)
                key = (bits << np.uint64(32)) | js.astype(np.uint64)
                order = np.argsort(key, kind="stable")[:max_neighbors]
                js = np.sort(js[order])
            src_l.append(js)
            dst_l.append(np.full(len(js), i, dtype=np.int64))
            row_ptr[i + 1] = len(js)
    row_ptr = np.cumsum(row_ptr)
    src = np.concatenate(src_l) if src_l else np.zeros(0, dtype=np.int64)
    dst = np.concatenate(dst_l) if dst_l else np.zeros(0, dtype=np.int64)
    return src.astype(np.int32), dst.astype(np.int32), row_ptr.astype(np.int32)


def triplets(src, dst, row_ptr, offset=None):
    """Triplet list k->j->i, k != i.

    Returns idx_kj[T], idx_ji[T] (edge ids, int32) ordered by (idx_ji, idx_kj)
    and seg_ptr[E+1] (int64) with the triplets of target edge e at
    seg_ptr[e]:seg_ptr[e+1].  offset [E,3] (periodic structures): k != i then means that
    the image of k is not atom i itself, i.e. not (same atom and offset_kj = -offset_ji).
    """
    n_edges = len(src)
    kj_l, ji_l = [], []
    seg = np.zeros(n_edges + 1, dtype=np.int64)
    for e in range(n_edges):
        j, i = int(src[e]), int(dst[e])
        cand = np.arange(row_ptr[j], row_ptr[j + 1], dtype=np.int64)  # in-edges k->j
        if offset is None:
            cand = cand[src[cand] != i]
        else:
            same = (src[cand] == i) & np.all(np.asarray(offset)[cand] == -np.asarray(offset)[e], axis=1)
            cand = cand[~same]
        kj_l.append(cand)
        ji_l.append(np.full(len(cand), e, dtype=np.int64))
        seg[e + 1] = len(cand)
    seg = np.cumsum(seg)
    idx_kj = np.concatenate(kj_l) if kj_l else np.zeros(0, dtype=np.int64)
    idx_ji = np.concatenate(ji_l) if ji_l else np.zeros(0, dtype=np.int64)
    return idx_kj.astype(np.int32), idx_ji.astype(np.int32), seg


def edges_loops(pos, graph_ptr, cutoff, max_neighbors=0):
    """Same edge list by explicit Python loops over ordered pairs (small inputs only)."""
    pos = np.ascontiguousarray(pos, dtype=np.float32)
    c = np.float32(cutoff)
    c2 = np.float32(c * c)
    out = []
    for g in range(len(graph_ptr) - 1):
        lo, hi = int(graph_ptr[g]), int(graph_ptr[g + 1])
        for i in range(lo, hi):
            cand = []
            for j in range(lo, hi):
                if j == i:
                    continue
                dx = np.float32(pos[i, 0] - pos[j, 0])
                dy = np.float32(pos[i, 1] - pos[j, 1])
                dz = np.float32(pos[i, 2] - pos[j, 2])
                d2 = np.float32(np.float32(np.float32(dx * dx) + np.float32(dy * dy)) + np.float32(dz * dz))
                if d2 < c2:
                    cand.append((int(d2.view(np.uint32)), j))
            if max_neighbors > 0 and len(cand) > max_neighbors:
                cand = sorted(cand)[:max_neighbors]
            for j in sorted(j for _, j in cand):
                out.append((j, i))
    return out


def triplets_loops(edge_pairs):
    """Triplets by the nested loop of the definition over an edge list of (src, dst) pairs."""
    out = []
    for e, (j, i) in enumerate(edge_pairs):
        for e2, (k, j2) in enumerate(edge_pairs):
            if j2 == j and k != i:
                out.append((e2, e))
    return out


def reverse_edges(src, dst, offset=None):
    """id_swap[e] = id of the edge running opposite to edge e (dst[e] -> src[e]), or -1 if the edge
    list has none (a neighbour cap can keep j->i and drop i->j).  Needed to couple the two
    messages on the same bond (Sec. 3.4, symmetric message passing).  With cell offsets the
    opposite edge carries the negated offset."""
    if offset is None:
        offset = np.zeros((len(src), 3), dtype=np.int64)
    off = np.asarray(offset)
    where = {(int(s), int(d), *map(int, o)): e for e, (s, d, o) in enumerate(zip(src, dst, off))}
    return np.array([where.get((int(d), int(s), *map(int, -o)), -1) for s, d, o in zip(src, dst, off)], dtype=np.int64)


def image_shift_f32(cell, n):
    """fp32 shift vector n0 a0 + n1 a1 + n2 a2, products and sums rounded one by one."""
    c = np.asarray(cell, dtype=np.float32)
    f = np.float32
    return np.array([f(f(f(f(n[0]) * c[0, k]) + f(f(n[1]) * c[1, k])) + f(f(n[2]) * c[2, k])) for k in range(3)], dtype=np.float32)


def edges_pbc(pos, graph_ptr, cells, cutoff, rep, max_neighbors=0):
    """Directed edge list of the radius graph of periodic structures.

    cells [G,3,3] (rows = lattice vectors), rep = (r0, r1, r2): images with |n_a| <= r_a are tested.
    Returns src, dst (int32), offset [E,3] (int32, the image of the source), row_ptr (int32),
    sorted by (dst, src, n0, n1, n2).
    """
    pos = np.ascontiguousarray(pos, dtype=np.float32)
    n = pos.shape[0]
    c = np.float32(cutoff)
    c2 = np.float32(c * c)
    images = [(a, b, d) for a in range(-rep[0], rep[0] + 1) for b in range(-rep[1], rep[1] + 1)
              for d in range(-rep[2], rep[2] + 1)]
    src_l, dst_l, off_l = [], [], []
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    for g in range(len(graph_ptr) - 1):
        lo, hi = int(graph_ptr[g]), int(graph_ptr[g + 1])
        shifts = np.stack([image_shift_f32(cells[g], im) for im in images])          # [NI,3] fp32
        for i in range(lo, hi):
            cand = []
            for j in range(lo, hi):
                ps = pos[j][None, :] + shifts                                        # fp32, one rounding
                dx = pos[i, 0] - ps[:, 0]
                dy = pos[i, 1] - ps[:, 1]
                dz = pos[i, 2] - ps[:, 2]
                d2 = (dx * dx + dy * dy) + dz * dz
                for q, im in enumerate(images):
                    if j == i and im == (0, 0, 0):
                        continue
                    if d2[q] < c2:
                        cand.append((int(d2[q].view(np.uint32)), j, im))
            if max_neighbors > 0 and len(cand) > max_neighbors:
                cand = sorted(cand)[:max_neighbors]
            kept = sorted((j, im) for _, j, im in cand)
            src_l += [j for j, _ in kept]
            off_l += [im for _, im in kept]
            dst_l += [i] * len(kept)
            row_ptr[i + 1] = len(kept)
    row_ptr = np.cumsum(row_ptr)
    return (np.array(src_l, dtype=np.int32), np.array(dst_l, dtype=np.int32),
            np.array(off_l, dtype=np.int32).reshape(-1, 3), row_ptr.astype(np.int32))


def edge_shifts(offset, dst, graph_ptr, cells):
    """fp64 shift vector of every edge: offset[e] . cell of the structure of the edge."""
    gp = np.asarray(graph_ptr)
    g_of = np.searchsorted(gp, np.asarray(dst), side="right") - 1
    return np.einsum("ea,eak->ek", np.asarray(offset, dtype=np.float64), np.asarray(cells, dtype=np.float64)[g_of])
