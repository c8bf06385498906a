"""The seeded generators: determinism and the structural properties the path relies on."""
import numpy as np

from paper_1711_07227_amd import synth


def test_corpus_structure_and_determinism():
    a = synth.corpus(300, 2000, 5, 40, 1.2, 7)
    b = synth.corpus(300, 2000, 5, 40, 1.2, 7)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    rp, ci, va = a
    assert rp.dtype == np.int64 and ci.dtype == np.int32 and va.dtype == np.float32
    h = np.diff(rp)
    assert h.min() >= 5 and h.max() <= 40 and rp[0] == 0 and rp[-1] == ci.size == va.size
    for i in range(300):
        row = ci[rp[i]:rp[i + 1]]
        assert np.all(np.diff(row) > 0)                      # sorted, distinct
        assert abs(float(va[rp[i]:rp[i + 1]].astype(np.float64).sum()) - 1.0) < 1e-5
    assert ci.min() >= 0 and ci.max() < 2000 and va.min() > 0
    # Zipf: the head of the vocabulary is used far more often than the tail
    assert (ci < 20).sum() > 5 * ((ci >= 1000) & (ci < 1020)).sum()


def test_corpus_fallback_when_block_runs_short():
    # h close to v forces the sequential continuation path
    rp, ci, va = synth.corpus(4, 30, 28, 30, 1.1, 3)
    for i in range(4):
        row = ci[rp[i]:rp[i + 1]]
        assert np.all(np.diff(row) > 0) and 28 <= row.size <= 30


def test_embeddings_unit_norm_and_bf16():
    E = synth.embeddings(100, 300, 11)
    assert E.dtype == np.float32 and np.allclose(np.linalg.norm(E.astype(np.float64), axis=1), 1.0, atol=1e-6)
    assert np.array_equal(E, synth.embeddings(100, 300, 11))
    B = synth.embeddings(100, 300, 11, bf16_valued=True)
    bits = B.view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0)                      # representable in bf16
    assert np.max(np.abs(B - E) / np.abs(E)) <= 2.0 ** -8
    assert np.array_equal(synth.bf16_bits_to_f32(synth.to_bf16_bits(B)), B)


def test_config_table_matches_workloads():
    c = synth.CONFIGS
    assert (c["tiny"].v, c["tiny"].n, c["tiny"].q) == (5000, 1000, 10)
    assert (c["medium"].v, c["medium"].n, c["medium"].q, c["medium"].h_lo, c["medium"].h_hi) == (100000, 100000, 1000, 50, 150)
    assert (c["long"].v, c["long"].n, c["long"].q) == (200000, 50000, 512)
    assert c["short"].queries_from_db and c["short"].precision == "bf16" and c["short"].q == 4096
    assert c["knn"].topk == 16 and c["knn"].v == 1000000
    assert all(x.m == 300 for x in c.values())


def test_permuted_vocabulary_is_the_same_problem():
    cfg = synth.CONFIGS["tiny"]
    a = synth.make(cfg, n=60, q=5)
    b = synth.make(cfg, n=60, q=5, permute_vocab=True)
    assert a["E"].shape == b["E"].shape and not np.array_equal(a["E"], b["E"])
    for key in ("db", "queries"):
        pa, ca, va = a[key]
        pb, cb, vb = b[key]
        assert np.array_equal(pa, pb)
        for r in range(len(pa) - 1):
            sa, sb = slice(pa[r], pa[r + 1]), slice(pb[r], pb[r + 1])
            assert np.all(np.diff(cb[sb]) > 0)                                   # still strictly increasing
            # the same multiset of (embedding row, weight) pairs
            ka = sorted((a["E"][w].tobytes(), float(x)) for w, x in zip(ca[sa], va[sa]))
            kb = sorted((b["E"][w].tobytes(), float(x)) for w, x in zip(cb[sb], vb[sb]))
            assert ka == kb
