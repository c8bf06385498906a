"""Seeded synthetic inputs shaped like the paper's workloads (Sec. VI, Table IV).

The paper's corpora are proprietary and its embeddings are the word2vec
Google-News vectors; neither is available, so every test and benchmark runs on
synthetic stand-ins: unit-norm Gaussian embeddings of dimension m = 300 and
bag-of-words histograms whose word ids follow a Zipf law over a
frequency-ordered vocabulary.

This module only draws random inputs.  It contains none of the method's
arithmetic (no distances, minima, products) and is the only code shared by the
CPU oracle's tests and the HIP path's tests.
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 171107227


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload: vocabulary, database and query generators."""
    name: str
    index: int            # used to derive the seed streams
    v: int
    m: int
    n: int
    q: int
    h_lo: int
    h_hi: int
    zipf_s: float
    precision: str        # "f32" or "bf16" (storage type of E on the device)
    queries_from_db: bool = False   # all-pairs: the queries are database rows
    topk: int = 0


CONFIGS = {
    "tiny":   Config("tiny",   1, 5_000,     300, 1_000,     10,    20,  80,  1.1, "f32"),
    "medium": Config("medium", 2, 100_000,   300, 100_000,   1_000, 50,  150, 1.1, "f32"),
    "long":   Config("long",   3, 200_000,   300, 50_000,    512,   300, 700, 1.0, "f32"),
    "short":  Config("short",  4, 500_000,   300, 1_000_000, 4_096, 5,   40,  1.2, "bf16",
                     queries_from_db=True),
    "knn":    Config("knn",    5, 1_000_000, 300, 1_000_000, 2_048, 20,  200, 1.1, "bf16",
                     topk=16),
}


def seed_for(cfg_index: int, stream: int) -> int:
    """stream 0 = embeddings, 1 = database, 2 = queries."""
    return BASE_SEED + 1000 * cfg_index + stream


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def embeddings(v: int, m: int, seed: int, bf16_valued: bool = False) -> np.ndarray:
    """v x m float32, rows i.i.d. N(0,1) scaled to unit L2 norm.

    With bf16_valued the entries are afterwards rounded to the nearest bfloat16,
    so the same values can be handed to the device as bf16 without further loss.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty((v, m), dtype=np.float32)
    step = max(1, (1 << 22) // max(m, 1))
    for a in range(0, v, step):
        b = min(v, a + step)
        g = rng.standard_normal((b - a, m))
        g /= np.sqrt((g * g).sum(axis=1, keepdims=True))
        out[a:b] = g.astype(np.float32)
    if bf16_valued:
        out = bf16_bits_to_f32(to_bf16_bits(out))
    return out


def _zipf_cdf(v: int, s: float) -> np.ndarray:
    w = np.arange(1, v + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    c /= c[-1]
    return c


def corpus(n: int, v: int, h_lo: int, h_hi: int, zipf_s: float, seed: int):
    """n histograms in CSR form.

    Document i has h_i ~ UniformInt[h_lo, h_hi] distinct words: word ranks are
    drawn from P(r) ~ r^-s (r = 1..v, word id = r-1, i.e. the vocabulary is
    frequency ordered) until h_i distinct ids have been seen.  Each word gets a
    count 1 + Poisson(1); the stored weight is count / sum(count) in float32.
    Column ids are sorted inside each row.

    Returns (row_ptr int64[n+1], col_idx int32[nnz], val float32[nnz]).
    """
    if h_hi > v:
        raise ValueError("a document cannot have more distinct words than the vocabulary")
    rng = np.random.Generator(np.random.PCG64(seed))
    cdf = _zipf_cdf(v, zipf_s)
    h = rng.integers(h_lo, h_hi + 1, size=n, dtype=np.int64)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(h, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    col_idx = np.empty(nnz, dtype=np.int32)

    draws_per_doc = 3 * h_hi + 32
    chunk = max(1, (1 << 23) // draws_per_doc)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        hb = h[a:b]
        u = rng.random((b - a, draws_per_doc))
        d = np.searchsorted(cdf, u, side="right").astype(np.int32)
        np.minimum(d, v - 1, out=d)
        order = np.argsort(d, axis=1, kind="stable")
        ds = np.take_along_axis(d, order, axis=1)
        first_sorted = np.ones(ds.shape, dtype=bool)
        first_sorted[:, 1:] = ds[:, 1:] != ds[:, :-1]
        first = np.empty_like(first_sorted)
        np.put_along_axis(first, order, first_sorted, axis=1)
        seen = np.cumsum(first, axis=1)
        keep = first & (seen <= hb[:, None])
        got = keep.sum(axis=1)
        rows = np.nonzero(keep)[0].astype(np.int64)
        words = d[keep].astype(np.int64)
        if np.all(got == hb):
            key = np.sort(rows * v + words)
            col_idx[row_ptr[a]:row_ptr[b]] = (key % v).astype(np.int32)
        else:
            # rare: the block of draws did not contain h_i distinct ids; continue drawing for those rows
            key = rows * v + words
            for r in range(b - a):
                sl = slice(row_ptr[a + r], row_ptr[a + r + 1])
                mine = set((key[rows == r] % v).tolist())
                while len(mine) < hb[r]:
                    w = int(np.searchsorted(cdf, rng.random(), side="right"))
                    mine.add(min(w, v - 1))
                col_idx[sl] = np.array(sorted(mine), dtype=np.int32)

    counts = 1 + rng.poisson(1.0, size=nnz).astype(np.int64)
    tot = np.add.reduceat(counts, row_ptr[:-1]) if nnz else np.zeros(0, np.int64)
    val = (counts.astype(np.float32) / np.repeat(tot, h).astype(np.float32)).astype(np.float32)
    return row_ptr, col_idx, val


def csr_rows(row_ptr, col_idx, val, rows):
    """Sub-matrix made of the given rows (in that order)."""
    rows = np.asarray(rows, dtype=np.int64)
    lens = row_ptr[rows + 1] - row_ptr[rows]
    rp = np.zeros(len(rows) + 1, dtype=np.int64)
    np.cumsum(lens, out=rp[1:])
    idx = np.concatenate([np.arange(row_ptr[r], row_ptr[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
    return rp, col_idx[idx].copy(), val[idx].copy()


def permute_vocabulary(E, sets, seed: int):
    """The same problem under a random renumbering of the vocabulary: word w becomes perm[w] in E's rows and in
    every histogram (rows re-sorted by the new ids).  Distances are unchanged; what changes is that word id no
    longer equals frequency rank, i.e. the frequent words are scattered over E instead of sharing its first rows."""
    v = E.shape[0]
    perm = np.random.Generator(np.random.PCG64(seed)).permutation(v).astype(np.int32)
    E2 = np.empty_like(E)
    E2[perm] = E
    out = []
    for row_ptr, col_idx, val in sets:
        c = perm[col_idx]
        rows = np.repeat(np.arange(len(row_ptr) - 1, dtype=np.int64), np.diff(row_ptr))
        order = np.lexsort((c, rows))
        out.append((row_ptr.copy(), c[order].astype(np.int32), val[order].copy()))
    return E2, out


def make(cfg: Config, *, n: int | None = None, q: int | None = None, v: int | None = None, permute_vocab: bool = False):
    """All inputs of a configuration; n, q, v may be overridden to scale it down."""
    n = cfg.n if n is None else n
    q = cfg.q if q is None else q
    v = cfg.v if v is None else v
    E = embeddings(v, cfg.m, seed_for(cfg.index, 0), bf16_valued=(cfg.precision == "bf16"))
    db = corpus(n, v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, seed_for(cfg.index, 1))
    if cfg.queries_from_db:
        qs = csr_rows(*db, np.arange(min(q, n)))
    else:
        qs = corpus(q, v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, seed_for(cfg.index, 2))
    if permute_vocab:
        E, (db, qs) = permute_vocabulary(E, [db, qs], seed_for(cfg.index, 3))
    return {"cfg": cfg, "E": E, "db": db, "queries": qs, "v": v, "n": n, "q": qs[0].shape[0] - 1}
