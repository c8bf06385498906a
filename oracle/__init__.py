"""ctypes front end of the C oracle (`rwmd_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It never touches the HIP library.  All arrays are host numpy
arrays; results are fp64.
"""
from __future__ import annotations

import ctypes
import pathlib

import numpy as np

_HERE = pathlib.Path(__file__).resolve().parent
_LIB_PATH = _HERE / "liblcrwmd_oracle.so"
_lib = None

_i64 = ctypes.c_int64
_pf = ctypes.POINTER(ctypes.c_float)
_pd = ctypes.POINTER(ctypes.c_double)
_pi64 = ctypes.POINTER(ctypes.c_int64)
_pi32 = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            from .build import build
            build()
        _lib = ctypes.CDLL(str(_LIB_PATH))
        _lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_rwmd_bruteforce", "oracle_rwmd_table", "oracle_rwmd_pairs",
                     "oracle_phase1", "oracle_phase2", "oracle_topk"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_pf)


def _csr(csr):
    ptr, col, val = csr
    ptr = np.ascontiguousarray(ptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    if ptr[0] != 0 or ptr[-1] != col.shape[0] or col.shape[0] != val.shape[0]:
        raise ValueError("malformed CSR")
    return (ptr, col, val), (ptr.ctypes.data_as(_pi64), col.ctypes.data_as(_pi32), val.ctypes.data_as(_pf),
                             _i64(ptr.shape[0] - 1))


def _check(rc):
    if rc == -1:
        raise ValueError("empty histogram: the minimum over an empty word set is undefined")
    if rc != 0:
        raise RuntimeError(f"oracle failed with code {rc}")


def _check_cols(v, *csrs):
    for (_, col, _) in csrs:
        if col.size and (col.min() < 0 or col.max() >= v):
            raise ValueError("word id outside the vocabulary")


def _full(fn_name, E, db, queries, parts):
    lib = _load()
    E, pE = _f32(E)
    v, m = E.shape
    dbk, dba = _csr(db)
    qk, qa = _csr(queries)
    _check_cols(v, dbk, qk)
    n, q = dbk[0].shape[0] - 1, qk[0].shape[0] - 1
    D = np.empty((n, q), dtype=np.float64)
    D12 = np.empty((n, q), dtype=np.float64) if parts else None
    D21 = np.empty((n, q), dtype=np.float64) if parts else None
    rc = getattr(lib, fn_name)(pE, _i64(v), _i64(m), _i64(m), *dba, *qa,
                               D.ctypes.data_as(_pd),
                               D12.ctypes.data_as(_pd) if parts else None,
                               D21.ctypes.data_as(_pd) if parts else None)
    _check(rc)
    return (D, D12, D21) if parts else D


def rwmd_bruteforce(E, db, queries, parts=False):
    """D[i, j] = max of the two one-directional RWMD bounds, pair by pair from the definition.

    With parts=True returns (D, D12, D21): D12[i, j] moves database doc i onto query j.
    """
    return _full("oracle_rwmd_bruteforce", E, db, queries, parts)


def rwmd_table(E, db, queries, parts=False):
    """Same values as rwmd_bruteforce, evaluated with one word-distance table per query."""
    return _full("oracle_rwmd_table", E, db, queries, parts)


def rwmd_pairs(E, db, queries, pi, pj):
    """Brute-force D[pi[t], pj[t]] for a list of pairs."""
    lib = _load()
    E, pE = _f32(E)
    v, m = E.shape
    dbk, dba = _csr(db)
    qk, qa = _csr(queries)
    _check_cols(v, dbk, qk)
    pi = np.ascontiguousarray(pi, dtype=np.int64)
    pj = np.ascontiguousarray(pj, dtype=np.int64)
    out = np.empty(pi.shape[0], dtype=np.float64)
    rc = lib.oracle_rwmd_pairs(pE, _i64(v), _i64(m), _i64(m), *dba, *qa,
                               pi.ctypes.data_as(_pi64), pj.ctypes.data_as(_pi64), _i64(pi.shape[0]),
                               out.ctypes.data_as(_pd))
    _check(rc)
    return out


def phase1(E, queries):
    """Z[w, j] = min over the words a of query j of ||E[w] - E[a]||, for every vocabulary word w."""
    lib = _load()
    E, pE = _f32(E)
    v, m = E.shape
    qk, qa = _csr(queries)
    _check_cols(v, qk)
    q = qk[0].shape[0] - 1
    Z = np.empty((v, q), dtype=np.float64)
    rc = lib.oracle_phase1(pE, _i64(v), _i64(m), _i64(m), qa[0], qa[1], qa[3], Z.ctypes.data_as(_pd))
    _check(rc)
    return Z


def phase2(X, Z):
    """D = X @ Z for CSR X (rows x v) and dense Z (v x ncols)."""
    lib = _load()
    Xk, Xa = _csr(X)
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    _check_cols(Z.shape[0], Xk)
    rows, ncols = Xk[0].shape[0] - 1, Z.shape[1]
    D = np.empty((rows, ncols), dtype=np.float64)
    rc = lib.oracle_phase2(Xa[0], Xa[1], Xa[2], Xa[3], Z.ctypes.data_as(_pd), _i64(ncols), D.ctypes.data_as(_pd))
    _check(rc)
    return D


def topk(D, k):
    """Per query column of D (n x q): indices and values of the k smallest, ordered by (value, index)."""
    lib = _load()
    D = np.ascontiguousarray(D, dtype=np.float64)
    n, q = D.shape
    idx = np.empty((q, k), dtype=np.int64)
    dist = np.empty((q, k), dtype=np.float64)
    rc = lib.oracle_topk(D.ctypes.data_as(_pd), _i64(n), _i64(q), _i64(k),
                         idx.ctypes.data_as(_pi64), dist.ctypes.data_as(_pd))
    _check(rc)
    return idx, dist


from .wmd import cost_matrix, emd, wmd_pair, wmd_pairs, centroids, wcd, wmd_topk_pruned  # noqa: E402,F401
