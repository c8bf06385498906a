"""GPU parity of the exact WMD, the WCD and the pruned top-k against the CPU oracle (LP solver in fp64), through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_1711_07227_amd import binding, synth
from helpers import RTOL_F32, assert_close, upload

pytestmark = pytest.mark.gpu


@pytest.fixture()
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def longest(csr):
    return int(np.max(np.diff(csr[0])))


def run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, in_flight=None, flags=False):
    t = len(pi)
    ws = binding.alloc_workspace(ctx.wmd_pairs_workspace_bytes(hmax[0], hmax[1], in_flight or max(t, 1)))
    out = torch.full((max(t, 1),), float("nan"), dtype=torch.float32, device="cuda")
    fl = torch.full((max(t, 1),), -1, dtype=torch.int32, device="cuda") if flags else None
    ctx.wmd_pairs(qs, db, E, torch.from_numpy(np.asarray(pi, np.int32)).cuda(), torch.from_numpy(np.asarray(pj, np.int32)).cuda(),
                  out, ws, fl)
    torch.cuda.synchronize()
    if flags:
        return out.cpu().numpy()[:t], fl.cpu().numpy()[:t]
    return out.cpu().numpy()[:t]


def problem(v, m, n, q, h_lo, h_hi, seed, s=1.1):
    return {"E": synth.embeddings(v, m, seed), "db": synth.corpus(n, v, h_lo, h_hi, s, seed + 1),
            "queries": synth.corpus(q, v, h_lo, h_hi, s, seed + 2)}


def test_wmd_pairs_small_documents_all_pairs(ctx):
    p = problem(v=200, m=300, n=12, q=9, h_lo=1, h_hi=12, seed=3)
    E, db, qs = upload(p)
    pi, pj = np.divmod(np.arange(12 * 9), 9)
    got, flags = run_wmd_pairs(ctx, E, db, qs, pi, pj, (longest(p["db"]), longest(p["queries"])), flags=True)
    assert np.all(flags == 0)
    assert_close(got, oracle.wmd_pairs(p["E"], p["db"], p["queries"], pi, pj), what="WMD of small documents")


def test_wmd_pairs_tiny_configuration_sampled(ctx, tiny):
    """Documents of 20-80 words over a Zipf vocabulary (shared words give zero-cost edges), several tiles a side."""
    E, db, qs = upload(tiny)
    rng = np.random.default_rng(5)
    pi = np.concatenate([rng.integers(0, 1000, 60), [0, 999]])
    pj = np.concatenate([rng.integers(0, 10, 60), [0, 9]])
    hmax = (longest(tiny["db"]), longest(tiny["queries"]))
    got, flags = run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, flags=True)
    assert np.all(flags == 0)
    ref = oracle.wmd_pairs(tiny["E"], tiny["db"], tiny["queries"], pi, pj)
    assert_close(got, ref, what="WMD, tiny configuration")
    # same pairs a few at a time: results do not depend on how many problems share the workspace
    again = run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, in_flight=7)
    assert np.array_equal(again, got)
    # bounds of Sec. III on the device results: RWMD <= WMD
    rw = oracle.rwmd_pairs(tiny["E"], tiny["db"], tiny["queries"], pi, pj)
    assert np.all(rw <= got * (1 + 1e-5))


def test_wmd_identical_and_single_word_documents(ctx):
    E = synth.embeddings(60, 300, 1)
    docs = synth.corpus(20, 60, 1, 9, 1.0, 2)
    Eg, db, qs = upload({"E": E, "db": docs, "queries": docs})
    pi = np.arange(20)
    got = run_wmd_pairs(ctx, Eg, db, qs, pi, pi, (longest(docs), longest(docs)))
    assert np.all(got == 0.0)                                              # a histogram against itself
    one = (np.array([0, 1], np.int64), np.array([7], np.int32), np.array([1.0], np.float32))
    Eg, db, qs = upload({"E": E, "db": docs, "queries": one})
    got = run_wmd_pairs(ctx, Eg, db, qs, pi, np.zeros(20, np.int64), (longest(docs), 1))
    ptr, col, val = docs
    ref = np.array([np.sum(val[ptr[i]:ptr[i + 1]].astype(np.float64) / val[ptr[i]:ptr[i + 1]].astype(np.float64).sum()
                           * np.linalg.norm(E[col[ptr[i]:ptr[i + 1]]].astype(np.float64) - E[7].astype(np.float64), axis=1))
                    for i in range(20)])
    assert_close(got, ref, what="one-word query: every flow is forced")


def test_wmd_on_a_line_and_other_embedding_widths(ctx):
    """m = 1: the closed form is the area between the cumulative distributions; m = 50 and bf16 storage against the LP."""
    rng = np.random.default_rng(4)
    v = 40
    E1 = rng.uniform(-3, 3, (v, 1)).astype(np.float32)
    docs = synth.corpus(8, v, 2, 9, 1.0, 6)
    Eg, db, qs = upload({"E": E1, "db": docs, "queries": docs})
    pi, pj = np.divmod(np.arange(64), 8)
    got = run_wmd_pairs(ctx, Eg, db, qs, pi, pj, (longest(docs), longest(docs)))
    ptr, col, val = docs
    ref = []
    for i, j in zip(pi, pj):
        xa, fa = E1[col[ptr[i]:ptr[i + 1]], 0].astype(np.float64), val[ptr[i]:ptr[i + 1]].astype(np.float64)
        xb, fb = E1[col[ptr[j]:ptr[j + 1]], 0].astype(np.float64), val[ptr[j]:ptr[j + 1]].astype(np.float64)
        pts = np.unique(np.concatenate([xa, xb]))
        Fa = np.array([fa[xa <= t].sum() / fa.sum() for t in pts])
        Fb = np.array([fb[xb <= t].sum() / fb.sum() for t in pts])
        ref.append(np.sum(np.abs(Fa - Fb)[:-1] * np.diff(pts)))
    assert_close(got, np.array(ref), what="WMD on a line")
    p = problem(v=300, m=50, n=6, q=5, h_lo=3, h_hi=40, seed=9)
    E, db, qs = upload(p)
    pi, pj = np.divmod(np.arange(30), 5)
    hmax = (longest(p["db"]), longest(p["queries"]))
    assert_close(run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax), oracle.wmd_pairs(p["E"], p["db"], p["queries"], pi, pj), what="m = 50")
    Er = synth.bf16_bits_to_f32(synth.to_bf16_bits(p["E"]))
    E, db, qs = upload({"E": Er, "db": p["db"], "queries": p["queries"]}, dtype=torch.bfloat16)
    assert_close(run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax), oracle.wmd_pairs(Er, p["db"], p["queries"], pi, pj), what="bf16 storage")


@pytest.mark.parametrize("m,pitch,offset,dtype", [(300, 300, 0, "bf16"), (298, 300, 0, "f32"), (298, 304, 0, "bf16"),
                                                  (300, 300, 1, "f32"), (300, 301, 0, "bf16"), (70, 72, 0, "f32")])
def test_wmd_pairs_embedding_layouts(ctx, m, pitch, offset, dtype):
    """Rows that start on 16-byte (bf16: 8-byte) boundaries are gathered four values per load, others one value per
    load; m need not be a multiple of four or of the slice, and the columns between m and the pitch hold other data."""
    rng = np.random.default_rng(21)
    v = 500
    E = synth.embeddings(v, m, 3)
    if dtype == "bf16":
        E = synth.bf16_bits_to_f32(synth.to_bf16_bits(E))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    flat = torch.full((v * pitch + 8,), 7.0, dtype=tdt, device="cuda")           # 7s wherever no embedding value sits
    Eg = flat[offset:offset + v * pitch].view(v, pitch)[:, :m]
    Eg.copy_(torch.from_numpy(E).cuda().to(tdt))
    p = {"E": E, "db": synth.corpus(9, v, 10, 60, 1.0, 22), "queries": synth.corpus(4, v, 10, 60, 1.0, 23)}
    db = binding.Csr.from_numpy(p["db"], v)
    qs = binding.Csr.from_numpy(p["queries"], v)
    pi, pj = np.divmod(np.arange(36), 4)
    got = run_wmd_pairs(ctx, Eg, db, qs, pi, pj, (longest(p["db"]), longest(p["queries"])))
    assert_close(got, oracle.wmd_pairs(E, p["db"], p["queries"], pi, pj), what=f"m = {m}, pitch {pitch}, offset {offset}, {dtype}")


def test_wmd_pairs_medium_sized_documents(ctx):
    """Documents of the Medium configuration's lengths (50-150 words): the sizes the benchmark solves."""
    p = synth.make(synth.CONFIGS["medium"], n=40, q=4, v=20000)
    E, db, qs = upload(p)
    pi, pj = np.divmod(np.arange(24), 4)
    got, flags = run_wmd_pairs(ctx, E, db, qs, pi, pj, (longest(p["db"]), longest(p["queries"])), flags=True)
    assert np.all(flags == 0)
    assert_close(got, oracle.wmd_pairs(p["E"], p["db"], p["queries"], pi, pj), what="WMD of 50-150 word documents")


@pytest.mark.parametrize("spread", [1e-3, 0.05, 0.6])
def test_wmd_pairs_with_words_that_lie_close_together(ctx, spread):
    """Clusters of near-identical embeddings: the distance between two words of a cluster is a small difference of
    large numbers in the norm expansion the matrix cores evaluate, so those tiles must come from coordinate
    differences.  spread = 0.6 puts part of the pairs on either side of the switch."""
    rng = np.random.default_rng(9)
    v, m = 600, 300
    centres = rng.standard_normal((12, m))
    E = (centres[np.arange(v) // 50] * 3.0 + spread * rng.standard_normal((v, m))).astype(np.float32)   # word w: cluster w // 50
    for vocab, what in ((v, "documents over all clusters"), (50, "documents inside one cluster")):
        p = {"E": E, "db": synth.corpus(14, vocab, 20, 45, 1.0, 10), "queries": synth.corpus(3, vocab, 20, 45, 1.0, 11)}
        Eg, db, qs = upload(p)
        pi, pj = np.divmod(np.arange(14 * 3), 3)
        got, flags = run_wmd_pairs(ctx, Eg, db, qs, pi, pj, (longest(p["db"]), longest(p["queries"])), flags=True)
        assert np.all(flags == 0)
        ref = oracle.wmd_pairs(p["E"], p["db"], p["queries"], pi, pj)
        assert_close(got, ref, what=f"WMD with clustered embeddings, spread {spread}, {what}")
        if vocab == 50:
            assert ref.max() < 2.0 * spread * np.sqrt(2 * m)      # these distances are differences inside a cluster


def test_wmd_pairs_long_documents(ctx):
    """About 400 words a side: beyond the size up to which the solver keeps its map of positive flows in LDS."""
    p = {"E": synth.embeddings(3000, 300, 1), "db": synth.corpus(2, 3000, 380, 420, 1.0, 2),
         "queries": synth.corpus(1, 3000, 380, 420, 1.0, 3)}
    E, db, qs = upload(p)
    got, flags = run_wmd_pairs(ctx, E, db, qs, [0, 1], [0, 0], (longest(p["db"]), longest(p["queries"])), flags=True)
    assert np.all(flags == 0)
    assert_close(got, oracle.wmd_pairs(p["E"], p["db"], p["queries"], [0, 1], [0, 0]), what="WMD of 400-word documents")


def test_wmd_largest_supported_documents(ctx):
    """2,048 words a side is the limit: closed forms at the limit, LCRWMD_EUNSUPPORTED one word beyond it."""
    v = 6000
    E = synth.embeddings(v, 300, 4)
    big = synth.corpus(1, v, 2048, 2048, 0.6, 5)
    one = (np.array([0, 1], np.int64), np.array([11], np.int32), np.array([1.0], np.float32))
    Eg, db, qs = upload({"E": E, "db": big, "queries": one})
    got = run_wmd_pairs(ctx, Eg, db, qs, [0], [0], (2048, 1))
    ptr, col, val = big
    w = val.astype(np.float64) / val.astype(np.float64).sum()
    ref = np.sum(w * np.linalg.norm(E[col].astype(np.float64) - E[11].astype(np.float64), axis=1))
    assert_close(got, np.array([ref]), what="2,048 words against one word")
    Eg, db, qs = upload({"E": E, "db": big, "queries": big})
    got, flags = run_wmd_pairs(ctx, Eg, db, qs, [0], [0], (2048, 2048), in_flight=1, flags=True)
    assert got[0] == 0.0 and flags[0] == 0                                   # against itself
    too_big = synth.corpus(1, v, 2049, 2049, 0.6, 6)
    Eg, db, qs = upload({"E": E, "db": too_big, "queries": one})
    with pytest.raises(binding.LcrwmdError) as e:
        run_wmd_pairs(ctx, Eg, db, qs, [0], [0], (2049, 1))
    assert e.value.status == binding.EUNSUPPORTED


def test_wmd_argument_checks(ctx, tiny):
    E, db, qs = upload(tiny)
    out = torch.zeros(4, dtype=torch.float32, device="cuda")
    pi = torch.tensor([0, 1, 2, 1000], dtype=torch.int32, device="cuda")       # 1000 is one past the last row
    pj = torch.tensor([0, 1, 2, 3], dtype=torch.int32, device="cuda")
    ws = binding.alloc_workspace(ctx.wmd_pairs_workspace_bytes(70, 70, 4))
    ctx.set_options(validate=1)
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_pairs(qs, db, E, pi, pj, out, ws)
    assert e.value.status == binding.EINVAL
    ctx.set_options(validate=0)
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_pairs(qs, db, E, pi[:3], pj[:3], out, binding.alloc_workspace(4096))
    assert e.value.status == binding.EWORKSPACE
    ctx.set_options(compute=binding.BF16)
    R_idx = torch.zeros((10, 4), dtype=torch.int32, device="cuda")
    R_dist = torch.zeros((10, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_topk(qs, db, E, 4, R_idx, R_dist, binding.alloc_workspace(1 << 20))
    assert e.value.status == binding.EUNSUPPORTED


def test_wcd_and_wmd_error_codes(ctx, tiny):
    E, db, qs = upload(tiny)
    n, q = db.rows, qs.rows
    D = torch.empty((n, q), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(1 << 24)
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wcd(qs, db, E, D, None)
    assert e.value.status == binding.EWORKSPACE
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wcd(qs, db, E, D, ws[:1024])                        # no room for the centroids
    assert e.value.status == binding.EWORKSPACE
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wcd(qs, db, E, torch.empty((n, 4), dtype=torch.float32, device="cuda"), ws)      # ldd < q
    assert e.value.status == binding.EINVAL
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wcd(qs, db, E[:50], D, ws)                          # histogram columns != v
    assert e.value.status == binding.EINVAL
    R_idx = torch.zeros((q, 3), dtype=torch.int32, device="cuda")
    R_dist = torch.zeros((q, 3), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_topk(qs, db, E, 0, R_idx, R_dist, ws)
    assert e.value.status == binding.EINVAL
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_topk(qs, db, E, 65, torch.zeros((q, 65), dtype=torch.int32, device="cuda"),
                     torch.zeros((q, 65), dtype=torch.float32, device="cuda"), ws)
    assert e.value.status == binding.EUNSUPPORTED
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_topk(qs, db, E, 3, R_idx, R_dist, ws[:65536])
    assert e.value.status == binding.EWORKSPACE
    with pytest.raises(binding.LcrwmdError):
        ctx.wmd_pairs_workspace_bytes(0, 5, 1)
    # a context that has seen errors keeps working
    ctx.wcd(qs, db, E, D, binding.alloc_workspace((n + q) * 300 * 4 + 1024))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(D).all())


def test_wcd_against_oracle(ctx, tiny):
    E, db, qs = upload(tiny)
    ws = binding.alloc_workspace((db.rows + qs.rows) * 300 * 4 + 1024)
    D = torch.full((db.rows, qs.rows), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wcd(qs, db, E, D, ws)
    torch.cuda.synchronize()
    assert_close(D.cpu().numpy(), oracle.wcd(tiny["E"], tiny["db"], tiny["queries"]), what="WCD, tiny configuration")
    # ragged sizes that are not multiples of the 64 x 64 tile, another width, a set against itself
    p = problem(v=500, m=37, n=131, q=67, h_lo=1, h_hi=20, seed=12)
    E, db, qs = upload(p)
    D = torch.full((131, 67), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wcd(qs, db, E, D, binding.alloc_workspace((131 + 67) * 40 * 4 + 1024))
    torch.cuda.synchronize()
    assert_close(D.cpu().numpy(), oracle.wcd(p["E"], p["db"], p["queries"]), what="WCD, m = 37")
    S = torch.full((131, 131), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wcd(db, db, E, S, binding.alloc_workspace(2 * 131 * 40 * 4 + 1024))
    torch.cuda.synchronize()
    assert np.all(np.diag(S.cpu().numpy()) == 0.0)


def check_topk(gi, gd, W):
    """gi/gd: device result (q x k); W: n x q exact WMD from the oracle."""
    n, q = W.shape
    k = gi.shape[1]
    for j in range(q):
        order = np.lexsort((np.arange(n), W[:, j]))
        assert_close(gd[j], W[order[:k], j], what=f"top-k WMD distances of query {j}")
        assert_close(W[gi[j], j], gd[j], what="reported rows carry the reported distances")
        assert len(set(gi[j].tolist())) == k
        gaps = np.diff(W[order[:k + 1], j])
        if np.min(gaps) > 1e-4 * W[order[k - 1], j]:
            assert np.array_equal(gi[j], order[:k])


def test_wmd_topk_pruned_equals_exhaustive(ctx):
    """Small enough for the oracle to evaluate every pair: the pruned search must return the true k nearest."""
    p = problem(v=400, m=300, n=150, q=6, h_lo=2, h_hi=14, seed=17, s=1.0)
    E, db, qs = upload(p)
    n, q, k = 150, 6, 5
    pi, pj = np.divmod(np.arange(n * q), q)
    W = oracle.wmd_pairs(p["E"], p["db"], p["queries"], pi, pj).reshape(n, q)
    hmax = (longest(p["db"]), longest(p["queries"]))
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(400, 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
    R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ev = torch.zeros(q, dtype=torch.int64)
    ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws, ev)
    torch.cuda.synchronize()
    check_topk(R_idx.cpu().numpy(), R_dist.cpu().numpy(), W)
    # evaluations: the first round may be wider than k (it fills the device), which lowers the cut-off; the survivors
    # are then at most those of the cut-off rule of Sec. III with its slack of 1e-5
    R = oracle.rwmd_bruteforce(p["E"], p["db"], p["queries"])
    ev = ev.numpy()
    for j in range(q):
        first = np.lexsort((np.arange(n), R[:, j]))[:k]
        L = W[first, j].max()
        most = len(set(np.nonzero(R[:, j] < L * (1 + 3e-5))[0]) | set(first))
        assert k <= ev[j] <= most + 64, (j, ev[j], most)
    assert ev.sum() < n * q
    # every query in a batch of its own, and a small workspace: same result
    ctx.set_options(max_query_batch=1)
    R2 = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    D2 = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wmd_topk(qs, db, E, k, R2, D2, ws)
    torch.cuda.synchronize()
    assert torch.equal(R2, R_idx) and torch.equal(D2, R_dist)


def test_wmd_topk_abandons_survivors_without_losing_a_neighbour(ctx):
    """Survivors are dropped as soon as the solver's lower bound on their distance passes the cut-off.  On a problem
    where that happens hundreds of times, the k nearest must still be those of the exhaustive matrix (every pair
    solved to the end by lcrwmd_wmd_pairs, itself checked against the oracle on the rows returned)."""
    p = problem(v=3000, m=300, n=2500, q=12, h_lo=8, h_hi=40, seed=41)
    E, db, qs = upload(p)
    n, q, k = 2500, 12, 7
    hmax = (longest(p["db"]), longest(p["queries"]))
    pi, pj = np.divmod(np.arange(n * q), q)
    W = run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, in_flight=4096).reshape(n, q).astype(np.float64)
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(3000, 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
    R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ev = torch.zeros(q, dtype=torch.int64)
    ctx.profile_begin()
    ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws, ev)
    pr = ctx.profile_end()
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    assert pr["emd_pairs"] == int(ev.sum())                                        # every pair counted was handed to the solver
    assert 100 < pr["emd_abandoned"] < int(ev.sum()) - q * k                       # abandoned: some, never a kept one
    for j in range(q):
        order = np.lexsort((np.arange(n), W[:, j]))[:k]
        assert np.array_equal(gd[j], W[order, j].astype(np.float32))               # same solver, same pairs: bit-equal
        assert np.array_equal(gi[j], order)
        assert_close(gd[j], oracle.wmd_pairs(p["E"], p["db"], p["queries"], gi[j], np.full(k, j)), what="top-k WMD values")


def test_wmd_topk_with_more_queries_than_the_first_round_can_widen_for(ctx):
    """With hundreds of queries in a batch the first round is k per query (the device is full), the second round
    takes the next nearest up to 64 against the first cut-off.  Same result as the exhaustive matrix."""
    p = problem(v=2000, m=300, n=900, q=500, h_lo=3, h_hi=16, seed=51)
    E, db, qs = upload(p)
    n, q, k = 900, 500, 16
    hmax = (longest(p["db"]), longest(p["queries"]))
    pi, pj = np.divmod(np.arange(n * q), q)
    W = run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, in_flight=8192).reshape(n, q).astype(np.float64)
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(2000, 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
    R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ev = torch.zeros(q, dtype=torch.int64)
    ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws, ev)
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    assert int(ev.min()) >= 64 and int(ev.sum()) < n * q
    for j in range(q):
        order = np.lexsort((np.arange(n), W[:, j]))[:k]
        assert np.array_equal(gd[j], W[order, j].astype(np.float32)), j
        assert np.array_equal(gi[j], order), j
    for j in (0, 499):
        assert_close(gd[j], oracle.wmd_pairs(p["E"], p["db"], p["queries"], gi[j], np.full(k, j)), what="top-k WMD values")
    # the same queries in batches of 190 (one first round each, wider): same result
    try:
        ctx.set_options(max_query_batch=190)
        R2 = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
        D2 = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
        ctx.wmd_topk(qs, db, E, k, R2, D2, ws)
        assert torch.equal(R2, R_idx) and torch.equal(D2, R_dist)
    finally:
        ctx.set_options()


@pytest.mark.parametrize("options", [{"dedup": 1}, {"compute": binding.BF16X3}, {"dedup": 1, "compute": binding.BF16X3}])
def test_wmd_topk_does_not_depend_on_the_form_of_the_bounds(ctx, options):
    """The de-duplicated form and the split-bf16 arithmetic give the same bounds up to fp32 rounding; the k nearest by
    WMD and their distances must come out bit-identical to the default form's."""
    p = problem(v=3000, m=300, n=1500, q=12, h_lo=8, h_hi=40, seed=71)
    E, db, qs = upload(p)
    n, q, k = 1500, 12, 7
    hmax = (longest(p["db"]), longest(p["queries"]))

    def run():
        ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(3000, 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
        R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
        R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
        ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws)
        return R_idx.cpu(), R_dist.cpu()

    ref = run()
    try:
        ctx.set_options(**options)
        got = run()
    finally:
        ctx.set_options()
    assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
    assert_close(ref[1][0].numpy(), oracle.wmd_pairs(p["E"], p["db"], p["queries"], ref[0][0].numpy(), np.zeros(k, np.int64)),
                 what="top-k WMD values")


def test_wmd_topk_with_bf16_embeddings(ctx):
    """Embeddings stored as bf16: bounds and transport costs are both taken from the stored values, so the bound stays
    a bound and the search returns the k nearest of the exhaustive matrix; values against the oracle on those values."""
    p = problem(v=1500, m=300, n=700, q=9, h_lo=5, h_hi=30, seed=61)
    Er = synth.bf16_bits_to_f32(synth.to_bf16_bits(p["E"]))
    E, db, qs = upload({"E": Er, "db": p["db"], "queries": p["queries"]}, dtype=torch.bfloat16)
    n, q, k = 700, 9, 6
    hmax = (longest(p["db"]), longest(p["queries"]))
    pi, pj = np.divmod(np.arange(n * q), q)
    W = run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, in_flight=4096).reshape(n, q).astype(np.float64)
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(1500, 300, n, db.nnz, q, qs.nnz, binding.BF16, k, *hmax))
    R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws)
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    for j in range(q):
        order = np.lexsort((np.arange(n), W[:, j]))[:k]
        assert np.array_equal(gi[j], order) and np.array_equal(gd[j], W[order, j].astype(np.float32))
    for j in (0, 8):
        assert_close(gd[j], oracle.wmd_pairs(Er, p["db"], p["queries"], gi[j], np.full(k, j)), what="top-k WMD values, bf16 storage")


def test_wmd_topk_with_queries_longer_than_the_register_variants_hold(ctx):
    """Queries of 260-300 words take the solver variant that keeps the sinks' state in LDS; survivors are abandoned
    there by the same rule.  Reference: every pair solved to the end on the device, the rows returned re-solved by
    the oracle."""
    p = {"E": synth.embeddings(3000, 300, 1), "db": synth.corpus(400, 3000, 200, 300, 1.0, 2),
         "queries": synth.corpus(2, 3000, 260, 300, 1.0, 3)}
    E, db, qs = upload(p)
    n, q, k = 400, 2, 3
    hmax = (longest(p["db"]), longest(p["queries"]))
    assert hmax[1] > 256
    pi, pj = np.divmod(np.arange(n * q), q)
    W = run_wmd_pairs(ctx, E, db, qs, pi, pj, hmax, in_flight=512).reshape(n, q).astype(np.float64)
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(3000, 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
    R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ctx.profile_begin()
    ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws)
    pr = ctx.profile_end()
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    assert pr["emd_abandoned"] > 0
    for j in range(q):
        order = np.lexsort((np.arange(n), W[:, j]))[:k]
        assert np.array_equal(gi[j], order) and np.array_equal(gd[j], W[order, j].astype(np.float32))
    assert_close(gd[0], oracle.wmd_pairs(p["E"], p["db"], p["queries"], gi[0], np.zeros(k, np.int64)), what="top-k WMD values")


def test_wmd_topk_with_the_smallest_workspace_that_works(ctx):
    """Shrinking the workspace makes the library walk the queries in smaller batches and the survivor lists in ranges;
    the result and (with the first round at its full width of 64) the evaluation counts must not change.  Below some size the call must refuse, not misbehave."""
    p = problem(v=600, m=300, n=8000, q=40, h_lo=20, h_hi=40, seed=23, s=1.0)
    E, db, qs = upload(p)
    n, q, k = 8000, 40, 64            # k at its maximum: the first round cannot be widened, many survivors
    hmax = (longest(p["db"]), longest(p["queries"]))
    full = ctx.wmd_topk_workspace_bytes(600, 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax)

    def run(nbytes):
        ws = binding.alloc_workspace(nbytes)
        R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
        R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
        ev = torch.zeros(q, dtype=torch.int64)
        ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws, ev)
        torch.cuda.synchronize()
        return R_idx.cpu(), R_dist.cpu(), ev.clone()

    ref = run(full)
    ok_sizes, nbytes = [], full
    while nbytes > 1024:
        nbytes = nbytes * 3 // 4
        try:
            got = run(nbytes)
        except binding.LcrwmdError as e:
            assert e.status == binding.EWORKSPACE
            break
        ok_sizes.append(nbytes)
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1]) and torch.equal(got[2], ref[2]), nbytes
        last = got
    assert len(ok_sizes) >= 3
    # the lists (12 bytes per survivor) get at most half of the workspace: at the smallest size they cannot have fitted at once
    assert (int(last[2].sum()) - q * k) * 12 > ok_sizes[-1] // 2, (int(last[2].sum()), ok_sizes)
    # spot check of the reference itself against the oracle
    gi, gd = ref[0].numpy(), ref[1].numpy()
    for j in range(2):
        assert_close(gd[j], oracle.wmd_pairs(p["E"], p["db"], p["queries"], gi[j], np.full(k, j)), what="top-k WMD values")


def test_wmd_topk_degenerate_shapes(ctx):
    """k = n (nothing left to prune), one document against one query, no queries, no pairs."""
    p = problem(v=100, m=300, n=5, q=3, h_lo=1, h_hi=9, seed=31)
    E, db, qs = upload(p)
    hmax = (longest(p["db"]), longest(p["queries"]))
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(100, 300, 5, db.nnz, 3, qs.nnz, binding.F32, 5, *hmax))
    R_idx = torch.full((3, 5), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((3, 5), float("nan"), dtype=torch.float32, device="cuda")
    ev = torch.zeros(3, dtype=torch.int64)
    ctx.wmd_topk(qs, db, E, 5, R_idx, R_dist, ws, ev)
    torch.cuda.synchronize()
    assert ev.tolist() == [5, 5, 5]
    pi, pj = np.divmod(np.arange(15), 3)
    W = oracle.wmd_pairs(p["E"], p["db"], p["queries"], pi, pj).reshape(5, 3)
    check_topk(R_idx.cpu().numpy(), R_dist.cpu().numpy(), W)
    one_db = binding.Csr.from_numpy(synth.csr_rows(*p["db"], np.arange(1)), 100)
    one_q = binding.Csr.from_numpy(synth.csr_rows(*p["queries"], np.arange(1)), 100)
    R_idx = torch.full((1, 1), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((1, 1), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wmd_topk(one_q, one_db, E, 1, R_idx, R_dist, ws)
    torch.cuda.synchronize()
    assert int(R_idx[0, 0]) == 0
    assert_close(R_dist.cpu().numpy()[0], W[:1, 0], what="one document, one query")
    # no queries / no pairs: nothing is launched, nothing is written
    none = binding.Csr(torch.zeros(1, dtype=torch.int64, device="cuda"), torch.zeros(0, dtype=torch.int32, device="cuda"),
                       torch.zeros(0, dtype=torch.float32, device="cuda"), 100, torch.zeros(1, dtype=torch.int64))
    ctx.wmd_topk(none, db, E, 1, R_idx, R_dist, ws)
    out = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    empty = torch.zeros(0, dtype=torch.int32, device="cuda")
    ctx.wmd_pairs(qs, db, E, empty, empty, out, ws)
    torch.cuda.synchronize()
    assert float(out[0]) == 7.0
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.wmd_topk(qs, db, E, 6, torch.zeros((3, 6), dtype=torch.int32, device="cuda"),
                     torch.zeros((3, 6), dtype=torch.float32, device="cuda"), ws)
    assert e.value.status == binding.EINVAL                      # k > n


def test_wmd_topk_tiny_configuration(ctx, tiny):
    """Tiny configuration (300 of its 1,000 documents x 10 queries, 20-80 words): the oracle follows the same pruning procedure."""
    sub = synth.csr_rows(*tiny["db"], np.arange(300))
    prob = {"E": tiny["E"], "db": sub, "queries": tiny["queries"]}
    E, db, qs = upload(prob)
    n, q, k = 300, 10, 4
    hmax = (longest(sub), longest(tiny["queries"]))
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(E.shape[0], 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
    R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ev = torch.zeros(q, dtype=torch.int64)
    print("wmd_topk on the device", flush=True)
    ctx.wmd_topk(qs, db, E, k, R_idx, R_dist, ws, ev)
    torch.cuda.synchronize()
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    print("evaluations per query:", ev.numpy().tolist(), flush=True)
    # the oracle evaluates the first three queries with the same procedure (its LP solves take ~30 ms each)
    R = oracle.rwmd_table(prob["E"], sub, tiny["queries"])
    three = synth.csr_rows(*tiny["queries"], np.arange(3))
    oi, od, need = oracle.wmd_topk_pruned(prob["E"], sub, three, k, R[:, :3])
    for j in range(3):
        assert_close(gd[j], od[j], what=f"pruned top-k distances of query {j}")
        if np.min(np.diff(od[j])) > 1e-4 * od[j][-1]:
            assert np.array_equal(gi[j], oi[j])
        assert k <= ev[j] <= need[j] + 64
    # for the other queries: the reported rows carry the reported distances
    for j in range(3, q):
        ref = oracle.wmd_pairs(prob["E"], sub, tiny["queries"], gi[j], np.full(k, j))
        assert_close(gd[j], ref, what="reported distances are WMDs of the reported rows")
        assert np.all(np.diff(gd[j]) >= 0)
