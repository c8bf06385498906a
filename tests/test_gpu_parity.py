"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_1711_07227_amd import binding, synth
from helpers import ATOL_ZERO, RTOL_F32, assert_close, run_rwmd, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    c.close()


def problem(v, m, n, q, h_lo, h_hi, seed, s=1.1):
    E = synth.embeddings(v, m, seed)
    db = synth.corpus(n, v, h_lo, h_hi, s, seed + 1)
    qs = synth.corpus(q, v, h_lo, h_hi, s, seed + 2)
    return {"E": E, "db": db, "queries": qs}


# ------------------------------------------------------------------------------------------- phase 1
@pytest.mark.parametrize("v,m,q,h_lo,h_hi", [
    (700, 300, 9, 1, 40),       # several vocabulary tiles with a ragged last one, histograms of 1..40 words
    (130, 300, 70, 3, 9),       # more histograms than tokens per tile
    (257, 7, 5, 2, 12),         # m not a multiple of 4: scalar load path, single K piece
    (300, 64, 3, 100, 200),     # histograms longer than one token tile
])
def test_phase1_matches_oracle(ctx, v, m, q, h_lo, h_hi):
    print(f"phase1 v={v} m={m} q={q} h={h_lo}..{h_hi}", flush=True)
    E = synth.embeddings(v, m, 5)
    qs = synth.corpus(q, v, h_lo, h_hi, 1.1, 6)
    ref = oracle.phase1(E, qs)
    Ed = torch.from_numpy(E).cuda()
    Q = binding.Csr.from_numpy(qs, v)
    ldz = q + 3
    Z = torch.full((v, ldz), -7.0, dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, q, Q.nnz))
    ctx.phase1_mindist(Ed, Q, Z, ws)
    torch.cuda.synchronize()
    Zh = Z.cpu().numpy()
    assert np.all(Zh[:, q:] == -7.0)                         # padding columns untouched
    assert_close(Zh[:, :q], ref, what="Z")
    ptr, col, _ = qs
    for j in range(q):
        assert np.all(Zh[col[ptr[j]:ptr[j + 1]], j] == 0.0)  # exact zeros for the histogram's own words


def test_phase1_with_row_pitch_and_unnormalised_embeddings(ctx):
    rng = np.random.default_rng(3)
    v, m, q = 200, 300, 6
    E = (rng.standard_normal((v, m)) * rng.uniform(0.2, 3.0, size=(v, 1))).astype(np.float32)
    qs = synth.corpus(q, v, 2, 30, 1.1, 8)
    ref = oracle.phase1(E, qs)
    big = torch.zeros((v, 304), dtype=torch.float32, device="cuda")
    big[:, :m] = torch.from_numpy(E).cuda()
    Ed = big[:, :m]                                          # ld = 304 > m
    Z = torch.empty((v, q), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, q, len(qs[1])))
    ctx.phase1_mindist(Ed, binding.Csr.from_numpy(qs, v), Z, ws)
    torch.cuda.synchronize()
    assert_close(Z.cpu().numpy(), ref, what="Z unnormalised")


# ------------------------------------------------------------------------------------------- phase 2
@pytest.mark.parametrize("rows,v,ncols,ld_extra", [(3000, 5000, 1500, 0), (2100, 150, 2050, 2), (5000, 40000, 1024, 4)])
def test_phase2_large_products(ctx, rows, v, ncols, ld_extra):
    """Millions of outputs: many strips and row tiles, a Z with few rows, a ragged last strip with padding columns that
    hold NaN, all three write-backs."""
    print(f"phase2 large rows={rows} v={v} ncols={ncols}", flush=True)
    rng = np.random.default_rng(rows)
    X = synth.corpus(rows, v, 1, min(70, v), 1.1, 3)
    Zh = rng.random((v, ncols)).astype(np.float32)
    ref = oracle.phase2(X, Zh.astype(np.float64))
    Xd = binding.Csr.from_numpy(X, v)
    Z = torch.full((v, ncols + ld_extra), float("nan"), dtype=torch.float32, device="cuda")
    Z[:, :ncols] = torch.from_numpy(Zh).cuda()
    Zv = Z[:, :ncols]
    D = torch.full((rows, ncols), -1.0, dtype=torch.float32, device="cuda")
    ctx.phase2_spmm(Xd, Zv, ncols, D, combine=0)
    torch.cuda.synchronize()
    assert_close(D.cpu().numpy(), ref, rtol=1e-5, what="large X*Z")
    prev = rng.random((rows, ncols)).astype(np.float32) * 0.3
    D1 = torch.from_numpy(prev).cuda()
    ctx.phase2_spmm(Xd, Zv, ncols, D1, combine=1)
    torch.cuda.synchronize()
    assert_close(D1.cpu().numpy(), np.maximum(prev.astype(np.float64), ref), rtol=1e-5, what="large max")
    prevT = rng.random((ncols, rows)).astype(np.float32) * 0.3
    D2 = torch.from_numpy(prevT).cuda()
    ctx.phase2_spmm(Xd, Zv, ncols, D2, combine=2)
    torch.cuda.synchronize()
    assert_close(D2.cpu().numpy(), np.maximum(prevT.astype(np.float64), ref.T), rtol=1e-5, what="large transposed max")



@pytest.mark.parametrize("rows,v,ncols", [(90, 400, 10), (333, 1000, 64), (200, 500, 517), (5, 50, 1)])
def test_phase2_store_and_max(ctx, rows, v, ncols):
    print(f"phase2 rows={rows} v={v} ncols={ncols}", flush=True)
    rng = np.random.default_rng(rows)
    X = synth.corpus(rows, v, 1, min(60, v), 1.1, 2)
    Zh = rng.random((v, ncols)).astype(np.float32)
    ref = oracle.phase2(X, Zh.astype(np.float64))
    Xd = binding.Csr.from_numpy(X, v)
    ldz = (ncols + 3) // 4 * 4
    Z = torch.zeros((v, ldz), dtype=torch.float32, device="cuda")
    Z[:, :ncols] = torch.from_numpy(Zh).cuda()
    D = torch.full((rows, ncols + 2), -1.0, dtype=torch.float32, device="cuda")
    ctx.phase2_spmm(Xd, Z, ncols, D, combine=0)
    torch.cuda.synchronize()
    Dh = D.cpu().numpy()
    assert np.all(Dh[:, ncols:] == -1.0)
    assert_close(Dh[:, :ncols], ref, rtol=1e-5, what="X*Z")
    # maximum with existing content
    prev = rng.random((rows, ncols)).astype(np.float32)
    D2 = torch.from_numpy(prev).cuda()
    ctx.phase2_spmm(Xd, Z, ncols, D2, combine=1)
    torch.cuda.synchronize()
    assert np.array_equal(D2.cpu().numpy(), np.maximum(prev, Dh[:, :ncols]))
    # transposed maximum
    prevT = rng.random((ncols, rows)).astype(np.float32)
    D3 = torch.from_numpy(prevT).cuda()
    ctx.phase2_spmm(Xd, Z, ncols, D3, combine=2)
    torch.cuda.synchronize()
    assert_close(D3.cpu().numpy(), np.maximum(prevT.astype(np.float64), ref.T), rtol=1e-5, what="transposed max")


# ------------------------------------------------------------------------------------------- full bound
def test_rwmd_tiny_config_full_matrix(ctx, tiny):
    ref = oracle.rwmd_table(tiny["E"], tiny["db"], tiny["queries"])
    E, db, qs = upload(tiny)
    got = run_rwmd(ctx, E, db, qs)
    assert_close(got, ref, what="tiny D")


def test_rwmd_without_host_row_pointers(ctx, tiny):
    ref = oracle.rwmd_table(tiny["E"], tiny["db"], tiny["queries"])
    E, db, qs = upload(tiny, host_rows=False)
    assert_close(run_rwmd(ctx, E, db, qs), ref, what="tiny D (row_ptr fetched by the library)")


def test_rwmd_ragged_mid_size_and_batch_independence(ctx):
    p = problem(v=3000, m=300, n=700, q=37, h_lo=1, h_hi=90, seed=21)
    ref = oracle.rwmd_table(p["E"], p["db"], p["queries"])
    E, db, qs = upload(p)
    whole = run_rwmd(ctx, E, db, qs)
    assert_close(whole, ref, what="mid D")
    ctx.set_options(max_query_batch=5, max_db_batch=64)
    try:
        batched = run_rwmd(ctx, E, db, qs)
    finally:
        ctx.set_options()
    assert_close(batched, ref, what="mid D in small batches")
    assert np.max(np.abs(batched - whole)) <= 2e-6           # same sums, same order: batches change nothing


def test_rwmd_self_distance_zero_and_symmetry(ctx, tiny):
    sub = synth.csr_rows(*tiny["db"], np.arange(150))
    p = {"E": tiny["E"], "db": sub, "queries": sub}
    E, db, qs = upload(p)
    got = run_rwmd(ctx, E, db, qs)
    assert np.all(np.diag(got) == 0.0)
    assert np.max(np.abs(got - got.T)) <= 1e-5
    assert_close(got, oracle.rwmd_table(tiny["E"], sub, sub), what="self D")


def test_rwmd_is_invariant_under_vocabulary_renumbering(ctx, tiny):
    """A consistent permutation of the word ids (rows of E and every histogram) changes no distance; it does change
    which words share a vocabulary tile and the order of the sums, hence a tolerance of a few ulps."""
    E2, (db2, qs2) = synth.permute_vocabulary(tiny["E"], [tiny["db"], tiny["queries"]], 99)
    a = run_rwmd(ctx, *upload(tiny))
    b = run_rwmd(ctx, *upload({"E": E2, "db": db2, "queries": qs2}))
    assert np.max(np.abs(a - b)) <= 2e-6
    assert_close(b, oracle.rwmd_table(E2, db2, qs2), what="tiny D, renumbered vocabulary")


def test_rwmd_degenerate_shapes(ctx):
    # one database doc, one query, single-word documents
    E = synth.embeddings(50, 300, 1)
    one = (np.array([0, 1], np.int64), np.array([7], np.int32), np.array([1.0], np.float32))
    other = (np.array([0, 1], np.int64), np.array([9], np.int32), np.array([1.0], np.float32))
    p = {"E": E, "db": one, "queries": other}
    got = run_rwmd(ctx, *upload(p))
    ref = np.linalg.norm(E[7].astype(np.float64) - E[9].astype(np.float64))
    assert got.shape == (1, 1) and abs(got[0, 0] - ref) <= RTOL_F32 * ref
    p = {"E": E, "db": one, "queries": one}
    assert run_rwmd(ctx, *upload(p))[0, 0] == 0.0
    # orthonormal embeddings: closed form sqrt(2) * weight outside the other document
    v = 64
    p = {"E": np.eye(v, dtype=np.float32), "db": synth.corpus(40, v, 2, 20, 1.0, 4),
         "queries": synth.corpus(9, v, 2, 20, 1.0, 5)}
    assert_close(run_rwmd(ctx, *upload(p)), oracle.rwmd_bruteforce(p["E"], p["db"], p["queries"]), what="eye D")


def test_empty_inputs_are_noops(ctx):
    E = torch.from_numpy(synth.embeddings(20, 300, 1)).cuda()
    empty = binding.Csr(torch.zeros(1, dtype=torch.int64, device="cuda"), torch.zeros(0, dtype=torch.int32, device="cuda"),
                        torch.zeros(0, dtype=torch.float32, device="cuda"), 20, torch.zeros(1, dtype=torch.int64))
    db = binding.Csr.from_numpy(synth.corpus(5, 20, 1, 5, 1.0, 1), 20)
    D = torch.zeros((5, 1), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(1 << 20)
    ctx.rwmd(empty, db, E, D, ws)
    ctx.phase1_mindist(E, empty, D, ws)
    ctx.phase2_spmm(empty, D, 1, D)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------- top-k
@pytest.mark.parametrize("n,q,k", [(1000, 10, 16), (5000, 70, 5), (300, 33, 64), (40, 3, 40)])
def test_topk_of_a_matrix_is_exact(ctx, n, q, k):
    rng = np.random.default_rng(n + k)
    Dh = rng.random((n, q)).astype(np.float32)
    Dh[rng.integers(0, n, 50), rng.integers(0, q, 50)] = 0.25      # ties across rows
    D = torch.from_numpy(Dh).cuda()
    ridx, rdist = oracle.topk(Dh.astype(np.float64), k)
    for ws in (None, binding.alloc_workspace(1 << 24)):
        R_idx = torch.empty((q, k), dtype=torch.int32, device="cuda")
        R_dist = torch.empty((q, k), dtype=torch.float32, device="cuda")
        ctx.topk(D, k, R_idx, R_dist, ws)
        torch.cuda.synchronize()
        assert np.array_equal(R_idx.cpu().numpy().astype(np.int64), ridx)
        assert np.array_equal(R_dist.cpu().numpy().astype(np.float64), rdist)


def test_rwmd_topk_matches_oracle_on_tiny(ctx, tiny):
    k = 16
    E, db, qs = upload(tiny)
    n, q = db.rows, qs.rows
    R_idx = torch.empty((q, k), dtype=torch.int32, device="cuda")
    R_dist = torch.empty((q, k), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(E.shape[0], E.shape[1], n, db.nnz, q, qs.nnz, k=k))
    ctx.rwmd_topk(qs, db, E, k, R_idx, R_dist, ws)
    torch.cuda.synchronize()
    ref = oracle.rwmd_table(tiny["E"], tiny["db"], tiny["queries"])
    ridx, rdist = oracle.topk(ref, k + 1)
    gi, gd = R_idx.cpu().numpy(), R_dist.cpu().numpy()
    assert_close(gd, rdist[:, :k], what="top-k distances")
    # indices must agree wherever the oracle's neighbouring gaps exceed the fp32 error bound
    gap_ok = np.diff(rdist, axis=1) > 8e-6 * rdist[:, 1:]
    for j in range(q):
        for r in range(k):
            left_ok = r == 0 or gap_ok[j, r - 1]
            if left_ok and gap_ok[j, r]:
                assert gi[j, r] == ridx[j, r], (j, r)
    assert (~gap_ok).sum() <= 2, "tiny config should be nearly ties-free at fp32 resolution"
    # batches of queries give the same answer
    ctx.set_options(max_query_batch=4)
    try:
        R2 = torch.empty_like(R_idx)
        ctx.rwmd_topk(qs, db, E, k, R2, R_dist, ws)
        torch.cuda.synchronize()
    finally:
        ctx.set_options()
    assert np.array_equal(R2.cpu().numpy(), gi)


# ------------------------------------------------------------------------------------------- error paths
def test_error_codes_never_crash(ctx, tiny):
    E, db, qs = upload(tiny)
    D = torch.empty((db.rows, qs.rows), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(1 << 26)
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.rwmd(qs, db, E, D, None)
    assert e.value.status == binding.EWORKSPACE
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.rwmd(qs, db, E, D, ws[:4096])
    assert e.value.status == binding.EWORKSPACE and "workspace" in str(e.value)
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.rwmd(qs, db, E, torch.empty((db.rows, 5), dtype=torch.float32, device="cuda"), ws)   # ldd < q
    assert e.value.status == binding.EINVAL
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.rwmd(qs, db, E[:100], D, ws)                      # columns != v
    assert e.value.status == binding.EINVAL
    with pytest.raises(binding.LcrwmdError) as e:
        ctx.topk(D, 65, torch.empty((qs.rows, 65), dtype=torch.int32, device="cuda"),
                 torch.empty((qs.rows, 65), dtype=torch.float32, device="cuda"))
    assert e.value.status == binding.EUNSUPPORTED
    # device-side validation of malformed histograms
    ctx.set_options(validate=1)
    try:
        v = E.shape[0]
        ptr, col, val = [a.copy() for a in tiny["queries"]]
        col[3] = col[2]                                        # duplicate word inside a row
        with pytest.raises(binding.LcrwmdError) as e:
            ctx.rwmd(binding.Csr.from_numpy((ptr, col, val), v), db, E, D, ws)
        assert e.value.status == binding.EBADCSR
        ptr2 = tiny["queries"][0].copy()
        ptr2[4] = ptr2[3]                                      # an empty histogram
        with pytest.raises(binding.LcrwmdError) as e:
            ctx.rwmd(binding.Csr.from_numpy((ptr2, tiny["queries"][1], tiny["queries"][2]), v), db, E, D, ws)
        assert e.value.status == binding.EEMPTYDOC
        col3 = tiny["queries"][1].copy()
        col3[-1] = v + 5                                       # word id outside the vocabulary
        with pytest.raises(binding.LcrwmdError) as e:
            ctx.rwmd(binding.Csr.from_numpy((tiny["queries"][0], col3, tiny["queries"][2]), v), db, E, D, ws)
        assert e.value.status == binding.EBADCSR
        ctx.rwmd(qs, db, E, D, binding.alloc_workspace(ctx.workspace_bytes(v, 300, db.rows, db.nnz, qs.rows, qs.nnz)))
        torch.cuda.synchronize()
    finally:
        ctx.set_options()


def test_results_are_deterministic(ctx, tiny):
    E, db, qs = upload(tiny)
    a = run_rwmd(ctx, E, db, qs)
    b = run_rwmd(ctx, E, db, qs)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------------------------------- bf16 path
def bf16_round(E):
    return synth.bf16_bits_to_f32(synth.to_bf16_bits(E))


@pytest.mark.parametrize("v,m,q,h_lo,h_hi", [(700, 300, 9, 1, 40), (300, 64, 3, 100, 200), (515, 290, 20, 2, 30),
                                             (200, 13, 4, 1, 9)])
def test_phase1_bf16_matches_oracle_on_rounded_embeddings(ctx, v, m, q, h_lo, h_hi):
    print(f"phase1 bf16 v={v} m={m} q={q}", flush=True)
    E = synth.embeddings(v, m, 15)
    Er = bf16_round(E)
    qs = synth.corpus(q, v, h_lo, h_hi, 1.1, 16)
    ref_rounded = oracle.phase1(Er, qs)
    ref_exact = oracle.phase1(E, qs)
    Q = binding.Csr.from_numpy(qs, v)
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, q, Q.nnz, binding.BF16))
    # (a) fp32 E, bf16 compute requested through the options: the library rounds to nearest even itself
    ctx.set_options(compute=binding.BF16)
    try:
        Z = torch.full((v, q), -3.0, dtype=torch.float32, device="cuda")
        ctx.phase1_mindist(torch.from_numpy(E).cuda(), Q, Z, ws)
        torch.cuda.synchronize()
    finally:
        ctx.set_options()
    Za = Z.cpu().numpy()
    assert_close(Za, ref_rounded, rtol=1e-4, what="bf16 Z vs oracle on bf16-rounded E")
    assert_close(Za, ref_exact, rtol=2e-2, atol=1e-5, what="bf16 Z vs oracle on fp32 E")
    # (b) E handed over as bf16
    Z2 = torch.full((v, q), -3.0, dtype=torch.float32, device="cuda")
    ctx.phase1_mindist(torch.from_numpy(Er).cuda().to(torch.bfloat16), Q, Z2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(Z2.cpu().numpy(), Za)
    ptr, col, _ = qs
    for j in range(q):
        assert np.all(Za[col[ptr[j]:ptr[j + 1]], j] == 0.0)


@pytest.mark.parametrize("compute", ["f32", "bf16", "bf16x3"])
def test_phase1_tile_and_pipeline_boundaries(ctx, compute):
    """Token counts around the tile sizes (32 / 64 rows), the depth of the copy pipeline (1..5 tiles per chunk) and the
    chunk length; vocabulary sizes around the workgroup widths (256 / 512 words)."""
    bf16 = compute == "bf16"
    rng = np.random.default_rng(11)
    ctx.set_options(compute={"f32": binding.F32, "bf16": binding.BF16, "bf16x3": binding.BF16X3}[compute])
    try:
        for v, lens in [(1, [1]), (255, [8]), (256, [7, 1]), (257, [64]), (511, [63, 9]), (512, [128]), (513, [65, 64, 63]),
                        (1025, [200, 56]), (300, [320]), (600, [31] * 17), (700, [8] * 70), (530, [1] * 300),
                        (520, [100] * 6), (1100, [3, 250, 2, 260, 1])]:
            print(f"boundaries {compute} v={v} lens={lens[:6]}", flush=True)
            E = synth.embeddings(v, 300, 100 + v)
            Er = bf16_round(E) if bf16 else E
            lens = [min(l, v) for l in lens]
            ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
            col = np.concatenate([np.sort(rng.choice(v, size=l, replace=False)) for l in lens]).astype(np.int32)
            val = np.concatenate([np.full(l, 1.0 / l) for l in lens]).astype(np.float32)
            qs = (ptr, col, val)
            q = len(lens)
            ref = oracle.phase1(Er, qs)
            Z = torch.full((v, q), -5.0, dtype=torch.float32, device="cuda")
            dt = binding.BF16 if bf16 else binding.F32
            ws = binding.alloc_workspace(ctx.workspace_bytes(v, 300, 0, 0, q, len(col), dt))
            ctx.phase1_mindist(torch.from_numpy(E).cuda(), binding.Csr.from_numpy(qs, v), Z, ws)
            torch.cuda.synchronize()
            assert_close(Z.cpu().numpy(), ref, what=f"Z {compute} v={v} q={q}")
    finally:
        ctx.set_options()


def test_split_bf16_compute_keeps_fp32_tolerance(ctx, tiny):
    """compute = BF16X3 (hi*hi + hi*lo + lo*hi on the bf16 units): same tolerance as fp32 against the oracle on the
    unrounded embeddings, for one phase and for the whole bound, also with m < 300 and unnormalised rows."""
    ctx.set_options(compute=binding.BF16X3)
    try:
        for v, m, q, h_lo, h_hi in [(700, 300, 9, 1, 40), (515, 290, 20, 2, 30), (300, 64, 3, 100, 200)]:
            E = synth.embeddings(v, m, 25)
            qs = synth.corpus(q, v, h_lo, h_hi, 1.1, 26)
            Q = binding.Csr.from_numpy(qs, v)
            Z = torch.full((v, q), -3.0, dtype=torch.float32, device="cuda")
            ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, q, Q.nnz))
            ctx.phase1_mindist(torch.from_numpy(E).cuda(), Q, Z, ws)
            torch.cuda.synchronize()
            assert_close(Z.cpu().numpy(), oracle.phase1(E, qs), what=f"split-bf16 Z v={v} m={m}")
        rng = np.random.default_rng(4)
        E = (rng.standard_normal((400, 300)) * rng.uniform(0.2, 3.0, size=(400, 1))).astype(np.float32)
        qs = synth.corpus(8, 400, 2, 30, 1.1, 27)
        Z = torch.empty((400, 8), dtype=torch.float32, device="cuda")
        ws = binding.alloc_workspace(ctx.workspace_bytes(400, 300, 0, 0, 8, len(qs[1])))
        ctx.phase1_mindist(torch.from_numpy(E).cuda(), binding.Csr.from_numpy(qs, 400), Z, ws)
        torch.cuda.synchronize()
        assert_close(Z.cpu().numpy(), oracle.phase1(E, qs), what="split-bf16 Z unnormalised")
        for p in (tiny, problem(v=3000, m=300, n=700, q=37, h_lo=1, h_hi=90, seed=21)):
            got = run_rwmd(ctx, *upload(p))
            assert_close(got, oracle.rwmd_table(p["E"], p["db"], p["queries"]), what="split-bf16 D")
        sub = synth.csr_rows(*tiny["db"], np.arange(100))
        assert np.all(np.diag(run_rwmd(ctx, *upload({"E": tiny["E"], "db": sub, "queries": sub}))) == 0.0)
    finally:
        ctx.set_options()


@pytest.mark.parametrize("offset,pad", [(0, 3), (1, 2), (2, 1), (3, 0), (0, 0), (2, 2)])      # pitch 304 four times, then 301 and 305
def test_phase1_bf16_with_z_at_any_alignment(ctx, offset, pad):
    """The bf16 kernel stores four histograms' results at a time where the rows of Z allow aligned 16-byte stores (row
    pitch a multiple of 4, quads counted from a 16-byte boundary wherever the first column lies) and value by value
    otherwise: Z as a view that starts `offset` floats into a row of pitch q + offset + pad, hundreds of short
    histograms, several vocabulary tiles."""
    print(f"phase1 bf16 offset={offset} pad={pad}", flush=True)
    v, m, q = 1100, 300, 301
    Er = bf16_round(synth.embeddings(v, m, 61))
    qs = synth.corpus(q, v, 1, 12, 1.1, 62)
    ref = oracle.phase1(Er, qs)
    Q = binding.Csr.from_numpy(qs, v)
    big = torch.full((v, q + offset + pad), -9.0, dtype=torch.float32, device="cuda")
    Z = big[:, offset:offset + q]
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, 0, 0, q, Q.nnz, binding.BF16))
    ctx.phase1_mindist(torch.from_numpy(Er).cuda().to(torch.bfloat16), Q, Z, ws)
    torch.cuda.synchronize()
    bigh = big.cpu().numpy()
    assert_close(bigh[:, offset:offset + q], ref, what="bf16 Z in an offset view")
    assert np.all(bigh[:, :offset] == -9.0) and np.all(bigh[:, offset + q:] == -9.0)      # nothing outside the view is touched


def test_rwmd_bf16_forward_batches_at_odd_columns(ctx):
    """Forward batches of 7 queries write column ranges of Z that start at every alignment; blocks of 50 database rows."""
    p = problem(v=3000, m=300, n=330, q=45, h_lo=1, h_hi=60, seed=71)
    Er = bf16_round(p["E"])
    ref = oracle.rwmd_table(Er, p["db"], p["queries"])
    E, db, qs = upload({"E": Er, "db": p["db"], "queries": p["queries"]}, dtype=torch.bfloat16)
    ctx.set_options(max_query_batch=7, max_db_batch=50)
    try:
        got = run_rwmd(ctx, E, db, qs, emb_dtype=binding.BF16)
    finally:
        ctx.set_options()
    assert_close(got, ref, what="bf16 D, forward batches of 7")


def test_rwmd_bf16_tiny_and_ragged(ctx, tiny):
    for p in (tiny, problem(v=3000, m=300, n=700, q=37, h_lo=1, h_hi=90, seed=21)):
        Er = bf16_round(p["E"])
        ref_rounded = oracle.rwmd_table(Er, p["db"], p["queries"])
        ref_exact = oracle.rwmd_table(p["E"], p["db"], p["queries"])
        E, db, qs = upload({"E": Er, "db": p["db"], "queries": p["queries"]}, dtype=torch.bfloat16)
        got = run_rwmd(ctx, E, db, qs, emb_dtype=binding.BF16)
        assert_close(got, ref_rounded, rtol=1e-4, what="bf16 D vs oracle on bf16-valued E")
        assert_close(got, ref_exact, rtol=2e-2, what="bf16 D vs oracle on fp32 E")


def test_bf16_wide_embeddings_run_in_fp32_on_the_rounded_values(ctx):
    """The bf16 kernels take m <= 300; wider embeddings in bf16 (storage or compute option) go through an fp32 copy of
    the bf16 values: same definition of the result."""
    v, m = 600, 400
    p = problem(v, m, 120, 7, 1, 30, seed=41)
    Er = synth.bf16_bits_to_f32(synth.to_bf16_bits(p["E"]))
    ref = oracle.rwmd_table(Er, p["db"], p["queries"])
    db = binding.Csr.from_numpy(p["db"], v)
    qs = binding.Csr.from_numpy(p["queries"], v)
    Eb = torch.from_numpy(Er).cuda().to(torch.bfloat16)
    got = run_rwmd(ctx, Eb, db, qs, emb_dtype=binding.BF16)
    assert_close(got, ref, what="bf16 storage, m = 400")
    ctx.set_options(compute=binding.BF16)
    try:
        got = run_rwmd(ctx, torch.from_numpy(p["E"]).cuda(), db, qs)
    finally:
        ctx.set_options()
    assert_close(got, ref, what="fp32 storage with the bf16 compute option, m = 400")


# ------------------------------------------------------------------------------------------- full-size workload
def test_medium_workload_at_full_size_sampled_pairs(ctx):
    """The benchmark's workload and launch configuration; the oracle evaluates sampled pairs one by one."""
    cfg = synth.CONFIGS["medium"]
    print("generating medium", flush=True)
    p = synth.make(cfg)
    E, db, qs = upload(p)
    n, q = db.rows, qs.rows
    assert (n, q, E.shape[0]) == (100000, 1000, 100000)
    ws = binding.alloc_workspace(ctx.workspace_bytes(E.shape[0], 300, n, db.nnz, q, qs.nnz))
    D = torch.full((n, q), float("nan"), dtype=torch.float32, device="cuda")
    print("running lcrwmd_rwmd", flush=True)
    ctx.rwmd(qs, db, E, D, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(D).all())
    assert float(D.min()) >= 0.0 and float(D.max()) <= 2.0 + 1e-4           # unit vectors
    rng = np.random.default_rng(7)
    pi = np.concatenate([rng.integers(0, n, 3000), [0, n - 1, 0, n - 1]])
    pj = np.concatenate([rng.integers(0, q, 3000), [0, q - 1, q - 1, 0]])
    print("oracle on sampled pairs", flush=True)
    ref = oracle.rwmd_pairs(p["E"], p["db"], p["queries"], pi, pj)
    got = D[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()].cpu().numpy()
    assert_close(got, ref, what="medium sampled pairs")
    # two full columns through the per-query table oracle
    cols = np.array([3, q - 1])
    ref_cols = oracle.rwmd_table(p["E"], p["db"], synth.csr_rows(*p["queries"], cols))
    assert_close(D[:, torch.from_numpy(cols).cuda()].cpu().numpy(), ref_cols, what="medium full columns")


def test_calls_on_a_side_stream_give_the_same_results(ctx, tiny):
    """Everything is enqueued on the caller's stream: a side stream (default priority) must give identical results,
    with its inputs produced on that stream right before the call."""
    E, db, qs = upload(tiny)
    base = run_rwmd(ctx, E, db, qs)
    side = torch.cuda.Stream()
    n, q, k = db.rows, qs.rows, 4
    with torch.cuda.stream(side):
        E2 = E * 1.0                                   # produced on the side stream, consumed by the library there
        ws = binding.alloc_workspace(ctx.workspace_bytes(E.shape[0], 300, n, db.nnz, q, qs.nnz))
        D = torch.full((n, q), float("nan"), dtype=torch.float32, device="cuda")
        ctx.rwmd(qs, db, E2, D, ws)
        R_idx = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
        R_dist = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
        hmax = (int(np.max(np.diff(tiny["db"][0]))), int(np.max(np.diff(tiny["queries"][0]))))
        ws2 = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(E.shape[0], 300, n, db.nnz, q, qs.nnz, binding.F32, k, *hmax))
        ctx.wmd_topk(qs, db, E2, k, R_idx, R_dist, ws2)
    side.synchronize()
    assert np.array_equal(D.cpu().numpy(), base)
    ws3 = binding.alloc_workspace(ws2.numel())
    R_idx0 = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    R_dist0 = torch.full((q, k), float("nan"), dtype=torch.float32, device="cuda")
    ctx.wmd_topk(qs, db, E, k, R_idx0, R_dist0, ws3)
    torch.cuda.synchronize()
    assert torch.equal(R_idx0, R_idx) and torch.equal(R_dist0, R_dist)


@pytest.mark.parametrize("compute", [binding.F32, binding.BF16X3])
def test_histograms_longer_than_a_chunk(ctx, compute):
    """Documents of 1,500-3,000 words are longer than the 1,024-token chunks the first phase balances its load with:
    a chunk then holds one whole histogram, and some chunks are empty."""
    v = 6000
    p = {"E": synth.embeddings(v, 300, 3), "db": synth.corpus(24, v, 1500, 3000, 0.8, 4),
         "queries": synth.corpus(3, v, 1100, 2100, 0.8, 5)}
    ref = oracle.rwmd_table(p["E"], p["db"], p["queries"])
    ctx.set_options(compute=compute)
    try:
        got = run_rwmd(ctx, *upload(p))
    finally:
        ctx.set_options()                                    # the context is shared by the tests of this module
    assert_close(got, ref, what="very long documents")


@pytest.mark.parametrize("m,pitch,offset", [(300, 301, 0), (300, 304, 1), (256, 256, 0), (208, 211, 0), (299, 300, 0)])
def test_fp32_shapes_served_by_the_padded_copy(ctx, m, pitch, offset):
    """fp32 E that the tile kernel cannot read in place (odd pitch, unaligned base, 208 <= m < 300) goes through a
    zero-padded copy; a workspace without room for the copy falls back to the general kernels.  Same results."""
    ctx.set_options()
    v = 1500
    p = {"E": synth.embeddings(v, m, 11), "db": synth.corpus(400, v, 1, 60, 1.1, 12),
         "queries": synth.corpus(9, v, 1, 60, 1.1, 13)}
    ref = oracle.rwmd_table(p["E"], p["db"], p["queries"])
    flat = torch.zeros(v * pitch + 8, dtype=torch.float32, device="cuda")
    view = flat[offset:offset + v * pitch].view(v, pitch)[:, :m]
    view.copy_(torch.from_numpy(p["E"]).cuda())
    db = binding.Csr.from_numpy(p["db"], v)
    qs = binding.Csr.from_numpy(p["queries"], v)
    full = ctx.workspace_bytes(v, m, db.rows, db.nnz, qs.rows, qs.nnz)
    assert_close(run_rwmd(ctx, view, db, qs, ws_bytes=full), ref, what=f"m={m} pitch={pitch} offset={offset}")
    # without the copy's share of the workspace the call still succeeds (general kernels) with the same result
    assert_close(run_rwmd(ctx, view, db, qs, ws_bytes=full - v * 304 * 4), ref, what="no room for the copy")
    # the stand-alone first phase takes the same route
    Z = torch.full((v, 12), -1.0, dtype=torch.float32, device="cuda")
    ctx.phase1_mindist(view, qs, Z, binding.alloc_workspace(full))
    torch.cuda.synchronize()
    assert_close(Z.cpu().numpy()[:, :9], oracle.phase1(p["E"], p["queries"]), what="Z through the padded copy")
