"""Oracle for the exact Word Mover's Distance, the Word Centroid Distance and RWMD-based pruning.
TEST INFRASTRUCTURE ONLY: numpy / scipy on the host, fp64, never on the product path.

* `emd`   — Sec. II: the transport problem written out as a linear programme (minimise sum y[p,q] c[p,q] with
            non-negative flows whose row sums are x1 and whose column sums are x2) and handed to a library LP solver.
* `wmd_pairs` — Sec. III, "Solving the WMD problem": C = T1 o T2 (Euclidean distances between the words of the two
            histograms), F1, F2 the stored weights, EMD on them.
* `wcd`   — Sec. III, "Word Centroid Distance": centroids X·E, Euclidean distance between centroids.
* `wmd_topk_pruned` — Sec. III, "Speeding-up WMD using RWMD": RWMD to every database histogram, the k nearest by RWMD,
            WMD on those, the largest of these WMDs as cut-off L, WMD on the remaining histograms whose RWMD is below L.

Reading of the paper where it is silent: the stored fp32 weights of an L1-normalised histogram sum to 1 only up to
rounding, and the programme needs equal masses, so each histogram's weights are divided by their fp64 sum first.
"""
from __future__ import annotations

import numpy as np
import scipy.optimize
import scipy.sparse


def _doc(csr, i):
    ptr, col, val = csr
    a, b = int(ptr[i]), int(ptr[i + 1])
    if a == b:
        raise ValueError("empty histogram: its distance to anything is undefined")
    return np.asarray(col[a:b], dtype=np.int64), np.asarray(val[a:b], dtype=np.float64)


def cost_matrix(T1, T2):
    """C = T1 o T2: C[p, q] = Euclidean distance between row p of T1 and row q of T2 (Sec. III)."""
    T1 = np.asarray(T1, dtype=np.float64)
    T2 = np.asarray(T2, dtype=np.float64)
    diff = T1[:, None, :] - T2[None, :, :]
    return np.sqrt(np.sum(diff * diff, axis=2))


def emd(x1, x2, c):
    """Sec. II: min sum_{p,q} y[p,q] c[p,q]  s.t.  y >= 0,  sum_q y[p,q] = x1[p],  sum_p y[p,q] = x2[q]."""
    x1 = np.asarray(x1, dtype=np.float64)
    x2 = np.asarray(x2, dtype=np.float64)
    c = np.asarray(c, dtype=np.float64)
    h1, h2 = c.shape
    if x1.shape != (h1,) or x2.shape != (h2,):
        raise ValueError("shape mismatch")
    x1 = x1 / x1.sum()
    x2 = x2 / x2.sum()
    # y flattened row-major: variable p * h2 + q
    rows = scipy.sparse.kron(scipy.sparse.identity(h1), np.ones((1, h2)))
    cols = scipy.sparse.kron(np.ones((1, h1)), scipy.sparse.identity(h2))
    res = scipy.optimize.linprog(c.ravel(), A_eq=scipy.sparse.vstack([rows, cols]).tocsr(),
                                 b_eq=np.concatenate([x1, x2]), bounds=(0, None), method="highs")
    if res.status != 0:
        raise RuntimeError(f"LP solver: {res.message}")
    return float(res.fun)


def wmd_pair(E, db, queries, i, j):
    p, f1 = _doc(db, i)
    q, f2 = _doc(queries, j)
    return emd(f1, f2, cost_matrix(np.asarray(E)[p], np.asarray(E)[q]))


def wmd_pairs(E, db, queries, pi, pj):
    """WMD(X1[pi[t]], X2[pj[t]]) for a list of pairs."""
    return np.array([wmd_pair(E, db, queries, int(i), int(j)) for i, j in zip(pi, pj)], dtype=np.float64)


def centroids(E, csr):
    """X·E: the weighted average of a histogram's word vectors (weights as stored)."""
    E = np.asarray(E, dtype=np.float64)
    n = len(csr[0]) - 1
    out = np.zeros((n, E.shape[1]))
    for i in range(n):
        w, f = _doc(csr, i)
        out[i] = f @ E[w]
    return out


def wcd(E, db, queries):
    """WCD[i, j] = Euclidean distance between the centroids of database histogram i and query j."""
    return cost_matrix(centroids(E, db), centroids(E, queries))


def _smallest(values, ids, k):
    order = np.lexsort((ids, values))[:k]
    return ids[order], values[order]


def wmd_topk_pruned(E, db, queries, k, rwmd):
    """The k database histograms nearest to every query by WMD, found with the RWMD cut-off.

    `rwmd` is the n x q matrix of RWMD lower bounds (from the RWMD oracle).  Returns (idx, dist, evaluated):
    idx/dist are q x k ordered by (distance, index), evaluated[j] counts the WMD evaluations query j needed.
    """
    n = len(db[0]) - 1
    q = len(queries[0]) - 1
    k = min(k, n)
    idx = np.empty((q, k), dtype=np.int64)
    dist = np.empty((q, k), dtype=np.float64)
    evaluated = np.zeros(q, dtype=np.int64)
    for j in range(q):
        lower = np.asarray(rwmd[:, j], dtype=np.float64)
        first, _ = _smallest(lower, np.arange(n), k)
        d_first = wmd_pairs(E, db, queries, first, np.full(k, j))
        L = d_first.max()
        rest = np.setdiff1d(np.nonzero(lower < L)[0], first)
        d_rest = wmd_pairs(E, db, queries, rest, np.full(len(rest), j))
        ids = np.concatenate([first, rest])
        idx[j], dist[j] = _smallest(np.concatenate([d_first, d_rest]), ids, k)
        evaluated[j] = len(ids)
    return idx, dist, evaluated
