"""The other workload families of the benchmark set (long documents, short-text all-pairs batches, large-vocabulary
k-NN), scaled down in the number of documents so that the CPU oracle finishes in seconds; vocabulary size, document
length distribution, Zipf exponent and precision are the configurations' own."""
import numpy as np
import pytest
import torch

import oracle
from paper_1711_07227_amd import binding, synth
from helpers import assert_close, run_rwmd, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def sampled_check(D, p, npairs, seed, rtol, what):
    n, q = D.shape
    rng = np.random.default_rng(seed)
    pi, pj = rng.integers(0, n, npairs), rng.integers(0, q, npairs)
    ref = oracle.rwmd_pairs(p["E"], p["db"], p["queries"], pi, pj)
    assert_close(D[pi, pj], ref, rtol=rtol, what=what)


def test_long_documents_fp32(ctx):
    cfg = synth.CONFIGS["long"]
    print("long: generating", flush=True)
    p = synth.make(cfg, n=2000, q=48)
    assert p["E"].shape == (200000, 300)
    h = np.diff(p["db"][0])
    assert h.min() >= 300 and h.max() <= 700
    D = run_rwmd(ctx, *upload(p))
    print("long: oracle", flush=True)
    sampled_check(D, p, 400, 1, 1e-4, "long sampled pairs")
    cols = np.array([0, 47])
    ref = oracle.rwmd_table(p["E"], p["db"], synth.csr_rows(*p["queries"], cols))
    assert_close(D[:, cols], ref, what="long full columns")


def test_short_text_all_pairs_batches_bf16(ctx):
    """Queries are database rows, processed in batches; bf16 embeddings; D of a batch includes the self pairs."""
    cfg = synth.CONFIGS["short"]
    print("short: generating", flush=True)
    n, qb = 40000, 512
    E = synth.embeddings(cfg.v, cfg.m, synth.seed_for(cfg.index, 0), bf16_valued=True)
    db = synth.corpus(n, cfg.v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, synth.seed_for(cfg.index, 1))
    Ed = torch.from_numpy(E).cuda().to(torch.bfloat16)
    dbd = binding.Csr.from_numpy(db, cfg.v)
    for b0 in (0, n - qb):                                    # first and last batch of the sweep
        rows = np.arange(b0, b0 + qb)
        qs = synth.csr_rows(*db, rows)
        D = run_rwmd(ctx, Ed, dbd, binding.Csr.from_numpy(qs, cfg.v), emb_dtype=binding.BF16)
        assert np.all(D[rows, np.arange(qb)] == 0.0)          # a document against itself
        p = {"E": E, "db": db, "queries": qs}
        sampled_check(D, p, 3000, b0 + 1, 1e-4, f"short batch at {b0}")


def test_large_vocabulary_knn_bf16_topk(ctx):
    cfg = synth.CONFIGS["knn"]
    print("knn: generating", flush=True)
    n, q, k = 30000, 96, 16
    v = 400000
    E = synth.embeddings(v, cfg.m, synth.seed_for(cfg.index, 0), bf16_valued=True)
    db = synth.corpus(n, v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, synth.seed_for(cfg.index, 1))
    qs = synth.corpus(q, v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, synth.seed_for(cfg.index, 2))
    Ed = torch.from_numpy(E).cuda().to(torch.bfloat16)
    dbd, qsd = binding.Csr.from_numpy(db, v), binding.Csr.from_numpy(qs, v)
    R_idx = torch.empty((q, k), dtype=torch.int32, device="cuda")
    R_dist = torch.empty((q, k), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, cfg.m, n, dbd.nnz, q, qsd.nnz, binding.BF16, k))
    ctx.rwmd_topk(qsd, dbd, Ed, k, R_idx, R_dist, ws)
    torch.cuda.synchronize()
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    print("knn: oracle", flush=True)
    cols = np.array([0, 1, 50, 95])
    ref = oracle.rwmd_table(E, db, synth.csr_rows(*qs, cols))
    ridx, rdist = oracle.topk(ref, k + 1)
    assert_close(gd[cols], rdist[:, :k], what="knn top-k distances")
    ambiguous = 0
    for t, j in enumerate(cols):
        gap_ok = np.diff(rdist[t]) > 8e-6 * rdist[t, 1:]
        for r in range(k):
            if (r == 0 or gap_ok[r - 1]) and gap_ok[r]:
                assert gi[j, r] == ridx[t, r], (j, r)
            else:
                ambiguous += 1
        assert set(gi[j]) <= set(np.argsort(ref[:, t])[:k + 4])      # members come from the true head of the list
    assert ambiguous <= 4
    # the distances returned are those of the returned rows
    D = run_rwmd(ctx, Ed, dbd, binding.Csr.from_numpy(synth.csr_rows(*qs, cols), v), emb_dtype=binding.BF16)
    for t, j in enumerate(cols):
        assert np.array_equal(D[gi[j], t], gd[j])
