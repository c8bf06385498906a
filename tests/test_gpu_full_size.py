"""The benchmark set's large workload families at their full sizes (long documents, one batch of the short-text
all-pairs sweep, large-vocabulary k-NN), through lcrwmd_rwmd / lcrwmd_rwmd_topk in the configuration bench.py times.
The oracle cannot produce a whole result at these sizes: each run is checked element-wise on full columns (per-query
table oracle) and on thousands of sampled pairs (per-pair brute force), the k-NN result also for index parity.

Also here: embedding matrices whose rows lie more than 4 GiB apart (the tile kernels address rows with 32-bit offsets
counted in 16-byte pieces)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1711_07227_amd import binding, synth
from helpers import assert_close, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def rwmd_on_device(ctx, E, db, qs, emb_dtype):
    n, q = db.rows, qs.rows
    ws = binding.alloc_workspace(ctx.workspace_bytes(E.shape[0], E.shape[1], n, db.nnz, q, qs.nnz, emb_dtype))
    D = torch.full((n, q), float("nan"), dtype=torch.float32, device="cuda")
    ctx.rwmd(qs, db, E, D, ws)
    torch.cuda.synchronize()
    return D


def check_samples(D, p, npairs, seed, what):
    n, q = D.shape
    rng = np.random.default_rng(seed)
    pi, pj = rng.integers(0, n, npairs), rng.integers(0, q, npairs)
    got = D[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()].cpu().numpy()
    assert_close(got, oracle.rwmd_pairs(p["E"], p["db"], p["queries"], pi, pj), what=what)


def check_columns(D, p, cols, what):
    ref = oracle.rwmd_table(p["E"], p["db"], synth.csr_rows(*p["queries"], cols))
    assert_close(D[:, torch.from_numpy(cols).cuda()].cpu().numpy(), ref, what=what)


def test_long_documents_full_size(ctx):
    cfg = synth.CONFIGS["long"]
    print("long, full size: generating", flush=True)
    p = synth.make(cfg)
    assert p["E"].shape == (200000, 300) and p["n"] == 50000 and p["q"] == 512
    E, db, qs = upload(p)
    for dedup in (0, 1):
        print(f"long, full size: device pass, dedup={dedup}", flush=True)
        ctx.set_options(dedup=dedup)
        try:
            D = rwmd_on_device(ctx, E, db, qs, binding.F32)
        finally:
            ctx.set_options()
        assert bool(torch.isfinite(D).all())
        print("long, full size: oracle", flush=True)
        check_columns(D, p, np.array([0, 511]), f"long, full columns, dedup={dedup}")
        check_samples(D, p, 2000, 31 + dedup, f"long, sampled pairs, dedup={dedup}")
        del D


def test_short_text_batches_full_size(ctx):
    """First and last batch of the all-pairs sweep: 4,096 database rows as queries against all 1,000,000 rows."""
    cfg = synth.CONFIGS["short"]
    print("short, full size: generating", flush=True)
    E = synth.embeddings(cfg.v, cfg.m, synth.seed_for(cfg.index, 0), bf16_valued=True)
    db = synth.corpus(cfg.n, cfg.v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, synth.seed_for(cfg.index, 1))
    Ed = torch.from_numpy(E).cuda().to(torch.bfloat16)
    dbd = binding.Csr.from_numpy(db, cfg.v)
    qb = cfg.q
    for b0 in (0, cfg.n - qb):
        print(f"short, full size: batch at row {b0}", flush=True)
        rows = np.arange(b0, b0 + qb)
        qs = synth.csr_rows(*db, rows)
        D = rwmd_on_device(ctx, Ed, dbd, binding.Csr.from_numpy(qs, cfg.v), binding.BF16)
        assert D.shape == (cfg.n, qb) and bool(torch.isfinite(D).all())
        diag = D[torch.from_numpy(rows).cuda(), torch.arange(qb, device="cuda")]
        assert bool((diag == 0.0).all())                      # a document against itself
        p = {"E": E, "db": db, "queries": qs}
        print("short, full size: oracle", flush=True)
        check_columns(D, p, np.array([0, qb - 1]), f"short batch at {b0}, full columns")
        check_samples(D, p, 3000, b0 + 1, f"short batch at {b0}, sampled pairs")
        del D


def test_short_text_all_pairs_in_one_call_full_size(ctx):
    """The whole all-pairs job, 1,000,000 documents against themselves, through lcrwmd_rwmd_self (245 batches of 4,096,
    every pair evaluated once): lists and sums of documents from the first, a middle and the last batch against the
    oracle's full columns, and the first batch's lists against lcrwmd_rwmd_reduce."""
    cfg = synth.CONFIGS["short"]
    print("short, all pairs in one call: generating", flush=True)
    E = synth.embeddings(cfg.v, cfg.m, synth.seed_for(cfg.index, 0), bf16_valued=True)
    db = synth.corpus(cfg.n, cfg.v, cfg.h_lo, cfg.h_hi, cfg.zipf_s, synth.seed_for(cfg.index, 1))
    Ed = torch.from_numpy(E).cuda().to(torch.bfloat16)
    dbd = binding.Csr.from_numpy(db, cfg.v)
    n, qb, k = cfg.n, cfg.q, 16
    starts = np.arange(0, n, qb)
    most = int(np.max(db[0][np.minimum(starts + qb, n)] - db[0][starts]))
    ws = binding.alloc_workspace(ctx.workspace_bytes(cfg.v, cfg.m, n, dbd.nnz, qb, most, binding.BF16, k))
    R_idx = torch.full((n, k), -3, dtype=torch.int32, device="cuda")
    R_dist = torch.full((n, k), -3.0, dtype=torch.float32, device="cuda")
    S = torch.full((n,), -3.0, dtype=torch.float64, device="cuda")
    print("short, all pairs in one call: device pass", flush=True)
    ctx.rwmd_self(dbd, Ed, qb, k, R_idx, R_dist, S, ws)
    torch.cuda.synchronize()
    assert bool((R_dist[:, 0] == 0.0).all()) and bool((R_idx >= 0).all()) and bool((R_idx < n).all())
    assert bool((R_dist[:, 1:] >= R_dist[:, :-1]).all())
    print("short, all pairs in one call: oracle columns", flush=True)
    pick = np.array([0, qb - 1, qb, n // 2 + 17, n - 1])
    ref = oracle.rwmd_table(E, db, synth.csr_rows(*db, pick))
    ridx, rdist = oracle.topk(ref, k + 1)
    sel = torch.from_numpy(pick).cuda()
    gi, gd = R_idx[sel].cpu().numpy(), R_dist[sel].cpu().numpy()
    assert_close(gd, rdist[:, :k], what="all pairs: list distances")
    assert_close(S[sel].cpu().numpy(), ref.sum(axis=0), rtol=1e-6, what="all pairs: sums")
    for t in range(len(pick)):
        gap_ok = np.diff(rdist[t]) > 8e-6 * np.maximum(rdist[t, 1:], 1e-30)
        sure = [r for r in range(k) if (r == 0 or gap_ok[r - 1]) and gap_ok[r]]
        assert len(sure) >= k - 4
        for r in sure:
            assert gi[t, r] == ridx[t, r], (pick[t], r)
    # the first batch through the batch-by-batch entry point: the same lists
    print("short, all pairs in one call: against lcrwmd_rwmd_reduce", flush=True)
    rows = np.arange(qb)
    qs = binding.Csr.from_numpy(synth.csr_rows(*db, rows), cfg.v)
    Ri = torch.empty((qb, k), dtype=torch.int32, device="cuda")
    Rd = torch.empty((qb, k), dtype=torch.float32, device="cuda")
    Sq = torch.empty((qb,), dtype=torch.float64, device="cuda")
    ctx.rwmd_reduce(qs, dbd, Ed, k, Ri, Rd, Sq, ws)
    torch.cuda.synchronize()
    assert_close(R_dist[:qb].cpu().numpy(), Rd.cpu().numpy(), rtol=2e-6, what="all pairs against reduce: distances")
    assert_close(S[:qb].cpu().numpy(), Sq.cpu().numpy(), rtol=1e-9, what="all pairs against reduce: sums")
    assert float((R_idx[:qb] == Ri).float().mean()) > 0.999


def test_large_vocabulary_knn_full_size(ctx):
    cfg = synth.CONFIGS["knn"]
    print("knn, full size: generating", flush=True)
    p = synth.make(cfg)
    v, n, q, k = cfg.v, cfg.n, cfg.q, cfg.topk
    assert p["E"].shape == (v, 300) and p["n"] == n and p["q"] == q and k == 16
    Ed = torch.from_numpy(p["E"]).cuda().to(torch.bfloat16)
    dbd, qsd = binding.Csr.from_numpy(p["db"], v), binding.Csr.from_numpy(p["queries"], v)
    R_idx = torch.empty((q, k), dtype=torch.int32, device="cuda")
    R_dist = torch.empty((q, k), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, cfg.m, n, dbd.nnz, q, qsd.nnz, binding.BF16, k))
    print("knn, full size: device pass", flush=True)
    ctx.rwmd_topk(qsd, dbd, Ed, k, R_idx, R_dist, ws)
    torch.cuda.synchronize()
    del ws
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    assert np.all((gi >= 0) & (gi < n)) and np.all(np.diff(gd, axis=1) >= 0)

    # full columns: distances, and indices wherever the oracle's neighbouring ranks are further apart than the fp32
    # error bound (8e-6 relative); where they are not, membership must still come from the true head of the list
    print("knn, full size: oracle columns", flush=True)
    cols = np.array([0, 1000, 2047])
    ref = oracle.rwmd_table(p["E"], p["db"], synth.csr_rows(*p["queries"], cols))
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
        assert set(gi[j]) <= set(np.argsort(ref[:, t])[:k + 4])
    assert ambiguous <= 4
    # sampled outputs over all queries: the distance reported for a returned row is that pair's distance
    print("knn, full size: sampled outputs", flush=True)
    rng = np.random.default_rng(5)
    pj, pr = rng.integers(0, q, 2000), rng.integers(0, k, 2000)
    assert_close(gd[pj, pr], oracle.rwmd_pairs(p["E"], p["db"], p["queries"], gi[pj, pr].astype(np.int64), pj),
                 what="knn sampled neighbours")
    # ... and bit for bit the value lcrwmd_rwmd gives for the same pair
    sub = binding.Csr.from_numpy(synth.csr_rows(*p["queries"], cols), v)
    D = rwmd_on_device(ctx, Ed, dbd, sub, binding.BF16)
    for t, j in enumerate(cols):
        assert np.array_equal(D[torch.from_numpy(gi[j].astype(np.int64)).cuda(), t].cpu().numpy(), gd[j])


def test_embedding_rows_more_than_4_gib_apart(ctx):
    """v = 5,000 rows with a pitch of 250,000 floats: the last row starts 5 GB into the buffer."""
    print("wide pitch: 5 GB of rows", flush=True)
    v, m, ld = 5000, 300, 250_000
    p = synth.make(synth.CONFIGS["tiny"], n=300)
    big = torch.zeros((v, ld), dtype=torch.float32, device="cuda")
    big[:, :m] = torch.from_numpy(p["E"]).cuda()
    E = big[:, :m]
    assert E.stride(0) == ld and (v - 1) * ld * 4 > 2 ** 32
    db = binding.Csr.from_numpy(p["db"], v)
    qs = binding.Csr.from_numpy(p["queries"], v)
    ref = oracle.rwmd_table(p["E"], p["db"], p["queries"])
    for compute in (binding.F32, binding.BF16X3):
        for dedup in (0, 1):
            ctx.set_options(compute=compute, dedup=dedup)
            try:
                D = rwmd_on_device(ctx, E, db, qs, binding.F32)
            finally:
                ctx.set_options()
            assert_close(D.cpu().numpy(), ref, what=f"wide pitch, compute {compute}, dedup {dedup}")
    # the first phase alone, every vocabulary row (the frequent words of a Zipf corpus sit in the first rows only)
    Z = torch.empty((v, qs.rows), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, qs.rows, qs.nnz))
    ctx.phase1_mindist(E, qs, Z, ws)
    torch.cuda.synchronize()
    assert_close(Z.cpu().numpy(), oracle.phase1(p["E"], p["queries"]), what="wide pitch, Z")
    del big, E
    torch.cuda.empty_cache()


def test_embedding_rows_beyond_the_offset_range(ctx):
    """130 rows with a pitch of 2^27 floats span 65 GiB, more than the tile kernel's offsets reach: the library must
    take another route (a compact copy) and still be right."""
    print("wide pitch: 65 GiB of rows", flush=True)
    v, m, ld = 130, 300, 1 << 27
    Eh = synth.embeddings(v, m, 41)
    qs = synth.corpus(6, v, 2, 20, 1.0, 42)
    big = torch.empty((v * ld,), dtype=torch.float32, device="cuda")         # not cleared: only the rows are written
    E = torch.as_strided(big, (v, m), (ld, 1))
    E.copy_(torch.from_numpy(Eh).cuda())
    Z = torch.empty((v, 6), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, 6, len(qs[1])))
    ctx.phase1_mindist(E, binding.Csr.from_numpy(qs, v), Z, ws)
    torch.cuda.synchronize()
    assert_close(Z.cpu().numpy(), oracle.phase1(Eh, qs), what="rows beyond the offset range, Z")
    del big, E
    torch.cuda.empty_cache()
