"""Shared by the GPU parity tests: upload helpers and the comparison rule."""
import numpy as np
import torch

from paper_1711_07227_amd import binding

# Relative tolerance of the fp32 path against the fp64 oracle (element-wise), with an absolute floor for
# entries whose true value is 0 (same support in both directions).
RTOL_F32 = 1e-4
ATOL_ZERO = 1e-6
RTOL_BF16 = 2e-2


def upload(problem, host_rows=True, dtype=torch.float32):
    E = torch.from_numpy(problem["E"]).cuda().to(dtype)
    v = problem["E"].shape[0]
    db = binding.Csr.from_numpy(problem["db"], v, host_rows=host_rows)
    qs = binding.Csr.from_numpy(problem["queries"], v, host_rows=host_rows)
    return E, db, qs


def run_rwmd(ctx, E, db, qs, ws_bytes=None, emb_dtype=binding.F32):
    n, q = db.rows, qs.rows
    if ws_bytes is None:
        ws_bytes = ctx.workspace_bytes(E.shape[0], E.shape[1], n, db.nnz, q, qs.nnz, emb_dtype)
    ws = binding.alloc_workspace(ws_bytes)
    D = torch.full((n, q), float("nan"), dtype=torch.float32, device="cuda")
    ctx.rwmd(qs, db, E, D, ws)
    torch.cuda.synchronize()
    return D.cpu().numpy()


def assert_close(got, ref, rtol=RTOL_F32, atol=ATOL_ZERO, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values in the device result"
    err = np.abs(got - ref)
    bad = err > (atol + rtol * np.abs(ref))
    if bad.any():
        k = np.unravel_index(np.argmax(err / (atol + rtol * np.abs(ref))), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} entries off; worst at {k}: got {got[k]!r} "
                             f"ref {ref[k]!r} rel {err[k] / max(abs(ref[k]), 1e-30):.3e}")
