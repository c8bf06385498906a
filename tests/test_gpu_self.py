"""The all-pairs job within one set (lcrwmd_rwmd_self): every histogram's k nearest of the set and the sum of its
distances to the whole set, from half of the tiles (the bound is symmetric).  Checked against the CPU oracle's full
n x n matrix; indices wherever the oracle's neighbouring ranks are further apart than the fp32 error bound."""
import numpy as np
import pytest
import torch

import oracle
from paper_1711_07227_amd import binding, synth
from helpers import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture()
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def run_self(ctx, E, docs, v, batch, k, sums=True, emb_dtype=binding.F32, bf16=False):
    Ed = torch.from_numpy(E).cuda()
    if bf16:
        Ed = Ed.to(torch.bfloat16)
    dd = binding.Csr.from_numpy(docs, v)
    n = dd.rows
    rp = docs[0]
    b = min(batch or 4096, n)
    most = int(max(rp[min(i + b, n)] - rp[i] for i in range(0, n, 1)))          # most entries of `b` consecutive rows
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, E.shape[1], n, dd.nnz, b, most, emb_dtype, k))
    R_idx = torch.full((n, max(k, 1)), -7, dtype=torch.int32, device="cuda")
    R_dist = torch.full((n, max(k, 1)), -7.0, dtype=torch.float32, device="cuda")
    S = torch.full((n,), -7.0, dtype=torch.float64, device="cuda") if sums else None
    ctx.rwmd_self(dd, Ed, batch, k, R_idx if k else None, R_dist if k else None, S, ws)
    torch.cuda.synchronize()
    return R_idx.cpu().numpy(), R_dist.cpu().numpy(), (S.cpu().numpy() if sums else None)


def check(gi, gd, gs, ref, k, what):
    n = ref.shape[0]
    assert np.allclose(ref, ref.T, rtol=1e-12, atol=1e-12)          # the oracle's matrix is symmetric
    if gs is not None:
        assert_close(gs, ref.sum(axis=1), rtol=1e-5, what=f"{what}: sums")
    if not k:
        return
    ridx, rdist = oracle.topk(ref, min(k + 1, n))                    # per column = per histogram
    assert_close(gd, rdist[:, :k], what=f"{what}: distances")
    assert np.all(np.diff(gd, axis=1) >= 0) and np.all((gi >= 0) & (gi < n))
    ambiguous = 0
    for i in range(n):
        assert len(set(gi[i])) == k, (what, i)
        gap_ok = np.diff(rdist[i]) > 8e-6 * np.maximum(rdist[i, 1:], 1e-30)
        for r in range(k):
            left = r == 0 or gap_ok[r - 1]
            right = gap_ok[r] if r < len(gap_ok) else True
            if left and right:
                assert gi[i, r] == ridx[i, r], (what, i, r)
            else:
                ambiguous += 1
    assert ambiguous <= max(4, n * k // 50), (what, ambiguous)          # near-ties: two positions each
    # a histogram is among its own nearest neighbours, at distance exactly 0 (first unless another one has the same words)
    assert np.all(gd[:, 0] == 0.0)
    for i in range(n):
        assert i in gi[i][gd[i] == 0.0], (what, i)


@pytest.mark.parametrize("dedup", [0, 1])
@pytest.mark.parametrize("batch,db_batch", [(64, 100), (200, 0), (0, 150)])
def test_self_against_the_full_matrix(ctx, dedup, batch, db_batch):
    """700 histograms: batches of 64 (ragged last one) with blocks of 100 rows, batches of 200 with one block, one batch."""
    print(f"self: dedup={dedup} batch={batch} db_batch={db_batch}", flush=True)
    v, n = 3000, 700
    E = synth.embeddings(v, 300, 61)
    docs = synth.corpus(n, v, 3, 60, 1.1, 62)
    ctx.set_options(dedup=dedup, max_db_batch=db_batch)
    try:
        gi, gd, gs = run_self(ctx, E, docs, v, batch, 16)
    finally:
        ctx.set_options()
    ref = oracle.rwmd_table(E, docs, docs)
    check(gi, gd, gs, ref, 16, f"dedup={dedup} batch={batch}")


def test_self_sums_only_lists_only_and_k_64(ctx):
    v, n = 2000, 300
    E = synth.embeddings(v, 300, 71)
    docs = synth.corpus(n, v, 2, 40, 1.2, 72)
    ref = oracle.rwmd_table(E, docs, docs)
    _, _, gs = run_self(ctx, E, docs, v, 128, 0)
    check(None, None, gs, ref, 0, "sums only")
    gi, gd, none = run_self(ctx, E, docs, v, 128, 64, sums=False)
    assert none is None
    check(gi, gd, None, ref, 64, "k = 64")
    dd = binding.Csr.from_numpy(docs, v)
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.rwmd_self(dd, torch.from_numpy(E).cuda(), 128, 0, None, None, None, binding.alloc_workspace(1 << 20))
    assert e.value.status == binding.EINVAL


def test_self_bf16_matches_the_batch_by_batch_job(ctx):
    """bf16 embeddings, short documents: against the oracle on the bf16-valued embeddings, and list for list against
    lcrwmd_rwmd_reduce run batch by batch (same distances up to fp32 rounding of the swapped roles)."""
    v, n, k = 20000, 3000, 16
    E = synth.embeddings(v, 300, 81, bf16_valued=True)
    docs = synth.corpus(n, v, 5, 40, 1.2, 82)
    gi, gd, gs = run_self(ctx, E, docs, v, 512, k, emb_dtype=binding.BF16, bf16=True)
    ref = oracle.rwmd_table(E, docs, docs)
    check(gi, gd, gs, ref, k, "bf16")
    Ed = torch.from_numpy(E).cuda().to(torch.bfloat16)
    dd = binding.Csr.from_numpy(docs, v)
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, 300, n, dd.nnz, 512, dd.nnz, binding.BF16, k))
    for b0 in (0, 2560):
        rows = np.arange(b0, min(b0 + 512, n))
        qs = binding.Csr.from_numpy(synth.csr_rows(*docs, rows), v)
        R_idx = torch.empty((len(rows), k), dtype=torch.int32, device="cuda")
        R_dist = torch.empty((len(rows), k), dtype=torch.float32, device="cuda")
        S = torch.empty((len(rows),), dtype=torch.float64, device="cuda")
        ctx.rwmd_reduce(qs, dd, Ed, k, R_idx, R_dist, S, ws)
        torch.cuda.synchronize()
        assert_close(gd[rows], R_dist.cpu().numpy(), rtol=2e-6, what="self against reduce: distances")
        assert_close(gs[rows], S.cpu().numpy(), rtol=1e-6, what="self against reduce: sums")
        assert (gi[rows] == R_idx.cpu().numpy()).mean() > 0.99


@pytest.mark.parametrize("n,batch,k", [(1, 0, 1), (5, 2, 5), (9, 1, 3), (64, 64, 64)])
def test_self_on_very_small_sets(ctx, n, batch, k):
    """One document (its only neighbour is itself), lists as long as the set, batches of one."""
    v = 400
    E = synth.embeddings(v, 300, 91)
    docs = synth.corpus(n, v, 2, 12, 1.0, 92 + n)
    gi, gd, gs = run_self(ctx, E, docs, v, batch, k)
    ref = oracle.rwmd_table(E, docs, docs).reshape(n, n)
    ridx, rdist = oracle.topk(ref, k)
    assert_close(gd, rdist, what=f"n={n}: distances")
    assert_close(gs, ref.sum(axis=1), rtol=1e-6, what=f"n={n}: sums")
    for i in range(n):
        assert sorted(gi[i]) == sorted(ridx[i]) or k < n, (n, i)
        assert i in gi[i][gd[i] == 0.0]
