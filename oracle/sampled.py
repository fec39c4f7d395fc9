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
