"""lcrwmd_topk_noalloc (partial lists in a file-scope device array, no workspace, no allocation) against lcrwmd_topk,
through the C ABI: bit-identical indices and distances, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_1711_07227_amd import binding

pytestmark = pytest.mark.gpu


def both(ctx, n, q, k, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    D = torch.rand((n, q + 3), generator=g, device="cuda", dtype=torch.float32)[:, :q]     # ldd > q
    dup = D[3::7].clone()
    D[0:7 * dup.shape[0]:7] = dup                                                          # ties between rows
    ref_i = torch.empty((q, k), dtype=torch.int32, device="cuda")
    ref_d = torch.empty((q, k), dtype=torch.float32, device="cuda")
    ws = binding.alloc_workspace(ctx.workspace_bytes(10, 10, n, n, q, q, binding.F32, k))
    ctx.topk(D, k, ref_i, ref_d, ws)
    got_i = torch.full((q, k), -1, dtype=torch.int32, device="cuda")
    got_d = torch.full((q, k), -1.0, dtype=torch.float32, device="cuda")
    ctx.topk_noalloc(D, k, got_i, got_d)
    torch.cuda.synchronize()
    return (got_i.cpu().numpy(), got_d.cpu().numpy()), (ref_i.cpu().numpy(), ref_d.cpu().numpy()), D


def test_topk_noalloc_matches_topk_on_two_calls_in_a_row():
    ctx = binding.Context(0)
    try:
        for n, q, k, seed in ((20000, 50, 16, 1), (5000, 7, 5, 2)):       # row splits: 9, then 2 - the scratch is used
            print(f"no-alloc top-k: n={n} q={q} k={k}", flush=True)
            (gi, gd), (ri, rd), D = both(ctx, n, q, k, seed)
            assert np.array_equal(gi, ri) and np.array_equal(gd, rd)
            # and the result is the top-k: against a sort on the device
            order = torch.sort(D.t().contiguous(), dim=1, stable=True)
            assert np.array_equal(gd, order.values[:, :k].cpu().numpy())
            assert np.array_equal(gi, order.indices[:, :k].cpu().numpy().astype(np.int32))
    finally:
        ctx.close()


def test_topk_noalloc_rejects_what_does_not_fit():
    ctx = binding.Context(0)
    try:
        n, q, k = 300000, 4096, 64                       # 16 row splits x 4096 x 64 x 8 bytes = 32 MiB of partial lists
        D = torch.zeros((8, 8), dtype=torch.float32, device="cuda")     # never read: the call must refuse before any launch
        R_i = torch.empty((q, k), dtype=torch.int32, device="cuda")
        R_d = torch.empty((q, k), dtype=torch.float32, device="cuda")
        st = ctx._lib.lcrwmd_topk_noalloc(ctx._h, D.data_ptr(), n, q, q, k, R_i.data_ptr(), R_d.data_ptr(), None)
        assert st == binding.EWORKSPACE and "scratch" in ctx.last_error()
    finally:
        ctx.close()
