"""ctypes binding of liblcrwmd.so: the same entry points as include/lcrwmd.h, argument marshalling only.

Every function takes torch CUDA tensors (PyTorch-ROCm is used for device memory and streams only),
passes their raw device pointers and the current HIP stream to the C ABI and raises LcrwmdError on a
non-OK status.  There is no fallback: if the shared library is missing the import of the symbols fails.
"""
from __future__ import annotations

import ctypes
import pathlib

import torch

import os

_HERE = pathlib.Path(__file__).resolve().parent
# LCRWMD_LIB lets a developer point the binding at another build of the same library
LIB_PATH = pathlib.Path(os.environ.get("LCRWMD_LIB", _HERE / "liblcrwmd.so"))

OK, EINVAL, EBADCSR, EEMPTYDOC, EWORKSPACE, EUNSUPPORTED, EHIP, ENOCONVERGE = range(8)
F32, BF16, BF16X3 = 0, 1, 2     # BF16X3: only as the compute option
STATUS_NAMES = {0: "OK", 1: "EINVAL", 2: "EBADCSR", 3: "EEMPTYDOC", 4: "EWORKSPACE", 5: "EUNSUPPORTED", 6: "EHIP",
                7: "ENOCONVERGE"}

EXPORTS = (
    "lcrwmd_create", "lcrwmd_destroy", "lcrwmd_last_error", "lcrwmd_set_options", "lcrwmd_get_options",
    "lcrwmd_workspace_bytes", "lcrwmd_phase1_mindist", "lcrwmd_phase2_spmm", "lcrwmd_rwmd",
    "lcrwmd_rwmd_topk", "lcrwmd_topk", "lcrwmd_profile_begin", "lcrwmd_profile_end",
    "lcrwmd_wcd", "lcrwmd_wmd_pairs_workspace_bytes", "lcrwmd_wmd_pairs", "lcrwmd_wmd_topk_workspace_bytes",
    "lcrwmd_wmd_topk", "lcrwmd_topk_noalloc", "lcrwmd_rwmd_reduce", "lcrwmd_forms_ran",
    "lcrwmd_rwmd_quadratic", "lcrwmd_rwmd_quadratic_workspace_bytes", "lcrwmd_probe_mfma", "lcrwmd_rwmd_self",
    "lcrwmd_probe_gather",
)


class CsrStruct(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("val", ctypes.c_void_p),
                ("row_ptr_host", ctypes.c_void_p)]


class EmbStruct(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("v", ctypes.c_int64), ("m", ctypes.c_int64), ("ld", ctypes.c_int64),
                ("dtype", ctypes.c_int)]


class OptionsStruct(ctypes.Structure):
    _fields_ = [("validate", ctypes.c_int), ("compute", ctypes.c_int),
                ("max_query_batch", ctypes.c_int64), ("max_db_batch", ctypes.c_int64), ("dedup", ctypes.c_int)]


class ProfileStruct(ctypes.Structure):
    _fields_ = [("phase1_ms", ctypes.c_double), ("phase1_launches", ctypes.c_int64), ("phase1_flops", ctypes.c_double),
                ("phase2_ms", ctypes.c_double), ("phase2_launches", ctypes.c_int64), ("phase2_bytes", ctypes.c_double),
                ("phase2_gather_bytes", ctypes.c_double),
                ("table_fwd_ms", ctypes.c_double), ("table_fwd_launches", ctypes.c_int64), ("table_fwd_bytes", ctypes.c_double),
                ("table_rev_ms", ctypes.c_double), ("table_rev_launches", ctypes.c_int64), ("table_rev_bytes", ctypes.c_double),
                ("emd_ms", ctypes.c_double), ("emd_launches", ctypes.c_int64), ("emd_pairs", ctypes.c_double),
                ("emd_abandoned", ctypes.c_double),
                ("phase1_swapped_ms", ctypes.c_double), ("phase1_swapped_flops", ctypes.c_double)]


class LcrwmdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lcrwmd status {STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load liblcrwmd.so (built by paper_1711_07227_amd.build).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_1711_07227_amd.build` "
                                    "(or __graft_entry__.build()) first; there is no fallback path")
        lib = ctypes.CDLL(str(LIB_PATH))
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        P = ctypes.POINTER
        lib.lcrwmd_create.argtypes = [P(vp), i32]
        lib.lcrwmd_destroy.argtypes = [vp]
        lib.lcrwmd_destroy.restype = None
        lib.lcrwmd_last_error.argtypes = [vp]
        lib.lcrwmd_last_error.restype = ctypes.c_char_p
        lib.lcrwmd_set_options.argtypes = [vp, P(OptionsStruct)]
        lib.lcrwmd_get_options.argtypes = [vp, P(OptionsStruct)]
        lib.lcrwmd_workspace_bytes.argtypes = [vp, i64, i64, i64, i64, i64, i64, i32, i32, P(sz)]
        lib.lcrwmd_phase1_mindist.argtypes = [vp, P(EmbStruct), P(CsrStruct), vp, i64, vp, sz, vp]
        lib.lcrwmd_phase2_spmm.argtypes = [vp, P(CsrStruct), vp, i64, i64, vp, i64, i32, vp]
        lib.lcrwmd_rwmd.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), vp, i64, vp, sz, vp]
        lib.lcrwmd_rwmd_topk.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), i32, vp, vp, vp, sz, vp]
        lib.lcrwmd_rwmd_reduce.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), i32, vp, vp, vp, vp, sz, vp]
        lib.lcrwmd_rwmd_self.argtypes = [vp, P(CsrStruct), P(EmbStruct), i64, i32, vp, vp, vp, vp, sz, vp]
        lib.lcrwmd_probe_gather.argtypes = [vp, i64, i32, vp, sz, P(ctypes.c_double), vp]
        lib.lcrwmd_forms_ran.argtypes = [vp]
        lib.lcrwmd_probe_mfma.argtypes = [vp, i32, i32, i32, ctypes.c_double, vp, sz, P(ctypes.c_double), P(ctypes.c_double), vp]
        lib.lcrwmd_rwmd_quadratic.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), vp, i64, vp, sz, vp]
        lib.lcrwmd_rwmd_quadratic_workspace_bytes.argtypes = [vp, i64, i64, i64, i64, i64, i64, i32, P(sz)]
        lib.lcrwmd_topk.argtypes = [vp, vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]
        lib.lcrwmd_topk_noalloc.argtypes = [vp, vp, i64, i64, i64, i32, vp, vp, vp]
        lib.lcrwmd_wcd.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), vp, i64, vp, sz, vp]
        lib.lcrwmd_wmd_pairs_workspace_bytes.argtypes = [vp, i64, i64, i64, P(sz)]
        lib.lcrwmd_wmd_pairs.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), vp, vp, i64, vp, vp, vp, sz, vp]
        lib.lcrwmd_wmd_topk_workspace_bytes.argtypes = [vp, i64, i64, i64, i64, i64, i64, i32, i32, i64, i64, P(sz)]
        lib.lcrwmd_wmd_topk.argtypes = [vp, P(CsrStruct), P(CsrStruct), P(EmbStruct), i32, vp, vp, vp, vp, sz, vp]
        lib.lcrwmd_profile_begin.argtypes = [vp]
        lib.lcrwmd_profile_end.argtypes = [vp, P(ProfileStruct)]
        for name in EXPORTS:
            if name not in ("lcrwmd_destroy", "lcrwmd_last_error"):
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


class Csr:
    """A histogram set on the device.  Keeps the tensors alive and, optionally, a host copy of row_ptr."""

    def __init__(self, row_ptr: torch.Tensor, col_idx: torch.Tensor, val: torch.Tensor | None, cols: int,
                 row_ptr_host: torch.Tensor | None = None):
        assert row_ptr.dtype == torch.int64 and col_idx.dtype == torch.int32
        assert val is None or val.dtype == torch.float32
        assert row_ptr.is_cuda and col_idx.is_cuda and (val is None or val.is_cuda)
        self.row_ptr, self.col_idx, self.val, self.cols = row_ptr.contiguous(), col_idx.contiguous(), val, cols
        if val is not None:
            self.val = val.contiguous()
        self.row_ptr_host = None
        if row_ptr_host is not None:
            assert row_ptr_host.dtype == torch.int64 and not row_ptr_host.is_cuda
            self.row_ptr_host = row_ptr_host.contiguous()
        self.rows = int(row_ptr.numel()) - 1
        self.nnz = int(col_idx.numel())

    @staticmethod
    def from_numpy(csr, cols: int, device="cuda", host_rows: bool = True) -> "Csr":
        ptr, col, val = csr
        hp = torch.from_numpy(ptr.copy()) if host_rows else None
        return Csr(torch.from_numpy(ptr).to(device), torch.from_numpy(col).to(device),
                   torch.from_numpy(val).to(device), cols, hp)

    def struct(self) -> CsrStruct:
        return CsrStruct(self.rows, self.cols, self.nnz, self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                         self.val.data_ptr() if self.val is not None else None,
                         self.row_ptr_host.data_ptr() if self.row_ptr_host is not None else None)


def _emb_struct(E: torch.Tensor) -> EmbStruct:
    assert E.is_cuda and E.dim() == 2 and E.stride(1) == 1
    if E.dtype == torch.float32:
        dt = F32
    elif E.dtype == torch.bfloat16:
        dt = BF16
    else:
        raise TypeError("E must be float32 or bfloat16")
    return EmbStruct(E.data_ptr(), E.shape[0], E.shape[1], E.stride(0), dt)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Context:
    """Owns an lcrwmd_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        st = self._lib.lcrwmd_create(ctypes.byref(self._h), device)
        if st != OK:
            raise LcrwmdError(st, "lcrwmd_create failed")
        self.device = device

    def close(self):
        if self._h:
            self._lib.lcrwmd_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != OK:
            raise LcrwmdError(st, self._lib.lcrwmd_last_error(self._h).decode())

    def last_error(self) -> str:
        return self._lib.lcrwmd_last_error(self._h).decode()

    def set_options(self, validate: int = 0, compute: int = F32, max_query_batch: int = 0, max_db_batch: int = 0,
                    dedup: int = 0):
        o = OptionsStruct(validate, compute, max_query_batch, max_db_batch, dedup)
        self._check(self._lib.lcrwmd_set_options(self._h, ctypes.byref(o)))

    def get_options(self) -> dict:
        o = OptionsStruct()
        self._check(self._lib.lcrwmd_get_options(self._h, ctypes.byref(o)))
        return {"validate": o.validate, "compute": o.compute, "max_query_batch": o.max_query_batch,
                "max_db_batch": o.max_db_batch, "dedup": o.dedup}

    def workspace_bytes(self, v, m, n, nnz_db, q, nnz_q, emb_dtype=F32, k=0) -> int:
        out = ctypes.c_size_t()
        self._check(self._lib.lcrwmd_workspace_bytes(self._h, v, m, n, nnz_db, q, nnz_q, emb_dtype, k,
                                                     ctypes.byref(out)))
        return int(out.value)

    def profile_begin(self):
        self._check(self._lib.lcrwmd_profile_begin(self._h))

    def profile_end(self) -> dict:
        p = ProfileStruct()
        self._check(self._lib.lcrwmd_profile_end(self._h, ctypes.byref(p)))
        return {name: getattr(p, name) for name, _ in ProfileStruct._fields_}

    @staticmethod
    def _ws(ws: torch.Tensor | None):
        if ws is None:
            return None, 0
        assert ws.is_cuda and ws.dtype == torch.uint8 and ws.is_contiguous()
        return ws.data_ptr(), ws.numel()

    def phase1_mindist(self, E: torch.Tensor, queries: Csr, Z: torch.Tensor, ws: torch.Tensor):
        assert Z.is_cuda and Z.dtype == torch.float32 and Z.stride(1) == 1
        es, qs = _emb_struct(E), queries.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_phase1_mindist(self._h, ctypes.byref(es), ctypes.byref(qs), Z.data_ptr(),
                                                    Z.stride(0), p, nbytes, _stream()))

    def phase2_spmm(self, X: Csr, Z: torch.Tensor, ncols: int, D: torch.Tensor, combine: int = 0):
        assert Z.is_cuda and Z.dtype == torch.float32 and D.is_cuda and D.dtype == torch.float32
        xs = X.struct()
        self._check(self._lib.lcrwmd_phase2_spmm(self._h, ctypes.byref(xs), Z.data_ptr(), Z.stride(0), ncols,
                                                 D.data_ptr(), D.stride(0), combine, _stream()))

    def rwmd(self, queries: Csr, database: Csr, E: torch.Tensor, D: torch.Tensor, ws: torch.Tensor):
        assert D.is_cuda and D.dtype == torch.float32 and D.stride(1) == 1
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_rwmd(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es),
                                          D.data_ptr(), D.stride(0), p, nbytes, _stream()))

    def rwmd_topk(self, queries: Csr, database: Csr, E: torch.Tensor, k: int, R_idx: torch.Tensor,
                  R_dist: torch.Tensor, ws: torch.Tensor):
        assert R_idx.dtype == torch.int32 and R_dist.dtype == torch.float32 and R_idx.is_contiguous() and R_dist.is_contiguous()
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_rwmd_topk(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es), k,
                                               R_idx.data_ptr(), R_dist.data_ptr(), p, nbytes, _stream()))

    def rwmd_reduce(self, queries: Csr, database: Csr, E: torch.Tensor, k: int, R_idx: torch.Tensor | None,
                    R_dist: torch.Tensor | None, col_sum: torch.Tensor | None, ws: torch.Tensor):
        if k > 0:
            assert R_idx.dtype == torch.int32 and R_dist.dtype == torch.float32 and R_idx.is_contiguous() and R_dist.is_contiguous()
        assert col_sum is None or (col_sum.is_cuda and col_sum.dtype == torch.float64 and col_sum.is_contiguous()
                                   and col_sum.numel() >= queries.rows)
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_rwmd_reduce(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es), k,
                                                 R_idx.data_ptr() if k > 0 else None, R_dist.data_ptr() if k > 0 else None,
                                                 col_sum.data_ptr() if col_sum is not None else None, p, nbytes, _stream()))

    def rwmd_self(self, docs: Csr, E: torch.Tensor, batch: int, k: int, R_idx: torch.Tensor | None,
                  R_dist: torch.Tensor | None, dist_sum: torch.Tensor | None, ws: torch.Tensor):
        if k > 0:
            assert R_idx.dtype == torch.int32 and R_dist.dtype == torch.float32 and R_idx.is_contiguous() and R_dist.is_contiguous()
            assert R_idx.numel() >= docs.rows * k and R_dist.numel() >= docs.rows * k
        assert dist_sum is None or (dist_sum.is_cuda and dist_sum.dtype == torch.float64 and dist_sum.is_contiguous()
                                    and dist_sum.numel() >= docs.rows)
        es, ds = _emb_struct(E), docs.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_rwmd_self(self._h, ctypes.byref(ds), ctypes.byref(es), batch, k,
                                               R_idx.data_ptr() if k > 0 else None, R_dist.data_ptr() if k > 0 else None,
                                               dist_sum.data_ptr() if dist_sum is not None else None, p, nbytes, _stream()))

    def probe_gather(self, segments: int, floats_per_lane: int = 4) -> float:
        ws = alloc_workspace(segments * 16384 + 256)
        p, nbytes = self._ws(ws)
        out = ctypes.c_double()
        self._check(self._lib.lcrwmd_probe_gather(self._h, segments, floats_per_lane, p, nbytes, ctypes.byref(out), _stream()))
        return float(out.value)

    def rwmd_quadratic_workspace_bytes(self, v, m, n, nnz_db, q, nnz_q, emb_dtype=F32) -> int:
        out = ctypes.c_size_t()
        self._check(self._lib.lcrwmd_rwmd_quadratic_workspace_bytes(self._h, v, m, n, nnz_db, q, nnz_q, emb_dtype, ctypes.byref(out)))
        return int(out.value)

    def rwmd_quadratic(self, queries: Csr, database: Csr, E: torch.Tensor, D: torch.Tensor, ws: torch.Tensor):
        assert D.is_cuda and D.dtype == torch.float32 and D.stride(1) == 1
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_rwmd_quadratic(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es),
                                                    D.data_ptr(), D.stride(0), p, nbytes, _stream()))

    def probe_mfma(self, dtype: int, random_data: bool, a_from_lds: bool, seconds: float = 0.5):
        """(TFLOP/s, shader MHz) of a bare MFMA loop; see lcrwmd_probe_mfma."""
        ws = alloc_workspace(1 << 20)
        tf, mhz = ctypes.c_double(), ctypes.c_double()
        self._check(self._lib.lcrwmd_probe_mfma(self._h, dtype, int(random_data), int(a_from_lds), seconds, ws.data_ptr(),
                                                ws.numel(), ctypes.byref(tf), ctypes.byref(mhz), _stream()))
        return tf.value, mhz.value

    def forms_ran(self) -> int:
        """Bit 0: the per-entry form ran in the last bound call; bit 1: the table form."""
        return int(self._lib.lcrwmd_forms_ran(self._h))

    def topk(self, D: torch.Tensor, k: int, R_idx: torch.Tensor, R_dist: torch.Tensor, ws: torch.Tensor | None = None):
        assert D.is_cuda and D.dtype == torch.float32 and D.stride(1) == 1
        assert R_idx.dtype == torch.int32 and R_dist.dtype == torch.float32 and R_idx.is_contiguous() and R_dist.is_contiguous()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_topk(self._h, D.data_ptr(), D.shape[0], D.shape[1], D.stride(0), k,
                                          R_idx.data_ptr(), R_dist.data_ptr(), p, nbytes, _stream()))

    def topk_noalloc(self, D: torch.Tensor, k: int, R_idx: torch.Tensor, R_dist: torch.Tensor):
        assert D.is_cuda and D.dtype == torch.float32 and D.stride(1) == 1
        assert R_idx.dtype == torch.int32 and R_dist.dtype == torch.float32 and R_idx.is_contiguous() and R_dist.is_contiguous()
        self._check(self._lib.lcrwmd_topk_noalloc(self._h, D.data_ptr(), D.shape[0], D.shape[1], D.stride(0), k,
                                                  R_idx.data_ptr(), R_dist.data_ptr(), _stream()))

    def wcd(self, queries: Csr, database: Csr, E: torch.Tensor, D: torch.Tensor, ws: torch.Tensor):
        assert D.is_cuda and D.dtype == torch.float32 and D.stride(1) == 1
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_wcd(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es),
                                         D.data_ptr(), D.stride(0), p, nbytes, _stream()))

    def wmd_pairs_workspace_bytes(self, max_h_db: int, max_h_q: int, pairs_in_flight: int) -> int:
        out = ctypes.c_size_t()
        self._check(self._lib.lcrwmd_wmd_pairs_workspace_bytes(self._h, max_h_db, max_h_q, pairs_in_flight, ctypes.byref(out)))
        return int(out.value)

    def wmd_pairs(self, queries: Csr, database: Csr, E: torch.Tensor, pair_db: torch.Tensor, pair_q: torch.Tensor,
                  out: torch.Tensor, ws: torch.Tensor, flags: torch.Tensor | None = None):
        assert pair_db.dtype == torch.int32 and pair_q.dtype == torch.int32 and out.dtype == torch.float32
        assert pair_db.is_cuda and pair_q.is_cuda and out.is_cuda
        assert pair_db.is_contiguous() and pair_q.is_contiguous() and out.is_contiguous()
        assert pair_q.numel() == pair_db.numel() and out.numel() >= pair_db.numel()
        assert flags is None or (flags.is_cuda and flags.dtype == torch.int32 and flags.is_contiguous()
                                 and flags.numel() >= pair_db.numel())
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_wmd_pairs(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es),
                                               pair_db.data_ptr(), pair_q.data_ptr(), pair_db.numel(), out.data_ptr(),
                                               flags.data_ptr() if flags is not None else None, p, nbytes, _stream()))

    def wmd_topk_workspace_bytes(self, v, m, n, nnz_db, q, nnz_q, emb_dtype, k, max_h_db, max_h_q) -> int:
        out = ctypes.c_size_t()
        self._check(self._lib.lcrwmd_wmd_topk_workspace_bytes(self._h, v, m, n, nnz_db, q, nnz_q, emb_dtype, k,
                                                              max_h_db, max_h_q, ctypes.byref(out)))
        return int(out.value)

    def wmd_topk(self, queries: Csr, database: Csr, E: torch.Tensor, k: int, R_idx: torch.Tensor, R_dist: torch.Tensor,
                 ws: torch.Tensor, evaluated: torch.Tensor | None = None):
        """evaluated: optional HOST int64 tensor with one entry per query."""
        assert R_idx.dtype == torch.int32 and R_dist.dtype == torch.float32 and R_idx.is_contiguous() and R_dist.is_contiguous()
        assert evaluated is None or (not evaluated.is_cuda and evaluated.dtype == torch.int64 and evaluated.is_contiguous()
                                     and evaluated.numel() >= queries.rows)
        es, qs, ds = _emb_struct(E), queries.struct(), database.struct()
        p, nbytes = self._ws(ws)
        self._check(self._lib.lcrwmd_wmd_topk(self._h, ctypes.byref(qs), ctypes.byref(ds), ctypes.byref(es), k,
                                              R_idx.data_ptr(), R_dist.data_ptr(),
                                              evaluated.data_ptr() if evaluated is not None else None, p, nbytes, _stream()))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device workspace; torch's allocator returns 512-byte aligned blocks, the library asks for 256."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
