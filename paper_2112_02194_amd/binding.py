"""ctypes binding of libals.so: same names as the C ABI (include/als.h), argument marshalling only.

Tables are torch tensors on the GPU (fp32 or bf16, row-major [rows, d]); sparse
matrices are ``Csr`` triples of device tensors.  Kernels are enqueued on torch's
current stream.  There is no CPU fallback: if the library is missing or no GPU
is visible, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libals.so")

ALS_OK, ALS_EINVAL, ALS_ESHAPE, ALS_EDTYPE, ALS_EALIAS, ALS_ENOTSPD, ALS_ENOMEM, ALS_EHIP = range(8)
ALS_F32, ALS_BF16 = 0, 1
PATH_AUTO, PATH_PRIMAL, PATH_DUAL = 0, 1, 2
SOLVER_DIRECT, SOLVER_CG, SOLVER_CG_FREE = 0, 1, 2

EXPORTS = ["als_create", "als_destroy", "als_gramian", "als_solve_rows", "als_epoch", "als_loss",
           "als_status_sync", "als_check_csr", "als_copy_probe", "als_set_timing", "als_get_timing",
           "als_strerror", "als_last_error", "als_gramian_static", "als_static_last_error", "als_topk"]


class c_als_csr(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("indptr", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("values", ctypes.c_void_p)]


class c_als_table(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("d", ctypes.c_int32),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int)]


class c_als_params(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_float), ("lambda_", ctypes.c_float), ("path", ctypes.c_int32),
                ("dual_max_k", ctypes.c_int32), ("split_nnz", ctypes.c_int32), ("solver", ctypes.c_int32),
                ("cg_max_iters", ctypes.c_int32), ("cg_tol", ctypes.c_float)]


class AlsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libals status {status}: {message}")
        self.status = status


_lib = None


def load_library(path: str = LIB_PATH):
    """Load libals.so (built by ``__graft_entry__.build()``); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(path)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    P = ctypes.POINTER
    lib.als_create.argtypes = [P(vp), i32]
    lib.als_destroy.argtypes = [vp]
    lib.als_gramian.argtypes = [vp, P(c_als_table), vp, vp]
    lib.als_solve_rows.argtypes = [vp, P(c_als_csr), P(c_als_table), vp, P(c_als_params), P(c_als_table), i64, i64, vp]
    lib.als_epoch.argtypes = [vp, P(c_als_csr), P(c_als_csr), P(c_als_table), P(c_als_table), P(c_als_params), vp]
    lib.als_loss.argtypes = [vp, P(c_als_csr), P(c_als_table), P(c_als_table), P(c_als_params), P(ctypes.c_double), vp]
    lib.als_status_sync.argtypes = [vp, vp]
    lib.als_check_csr.argtypes = [vp, P(c_als_csr), vp]
    lib.als_set_timing.argtypes = [vp, i32]
    lib.als_get_timing.argtypes = [vp, P(ctypes.c_double)]
    lib.als_copy_probe.argtypes = [vp, vp, vp, i64, vp]
    for name in EXPORTS[:11]:
        getattr(lib, name).restype = i32
    lib.als_strerror.argtypes = [i32]
    lib.als_strerror.restype = ctypes.c_char_p
    lib.als_last_error.argtypes = [vp]
    lib.als_last_error.restype = ctypes.c_char_p
    lib.als_gramian_static.argtypes = [i32, P(c_als_table), vp, vp]
    lib.als_gramian_static.restype = i32
    lib.als_topk.argtypes = [vp, P(c_als_table), P(c_als_table), P(c_als_csr), i32, vp, vp, vp]
    lib.als_topk.restype = i32
    lib.als_static_last_error.argtypes = []
    lib.als_static_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


@dataclass
class Csr:
    """CSR matrix on the GPU: int64 indptr [rows+1], int32 indices [nnz], optional fp32 values."""
    rows: int
    cols: int
    indptr: torch.Tensor
    indices: torch.Tensor
    values: Optional[torch.Tensor] = None

    @property
    def nnz(self) -> int:
        return int(self.indices.numel())

    def c(self) -> c_als_csr:
        assert self.indptr.dtype == torch.int64 and self.indices.dtype == torch.int32
        assert self.indptr.is_contiguous() and self.indices.is_contiguous()
        assert self.indptr.numel() == self.rows + 1
        vals = None
        if self.values is not None:
            assert self.values.dtype == torch.float32 and self.values.is_contiguous()
            assert self.values.numel() == self.indices.numel()
            vals = self.values.data_ptr()
        return c_als_csr(self.rows, self.cols, self.nnz, self.indptr.data_ptr(),
                         self.indices.data_ptr() if self.nnz else None, vals)


def _table(t: torch.Tensor) -> c_als_table:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("table must be 2-D with unit column stride")
    if t.dtype == torch.float32:
        dt = ALS_F32
    elif t.dtype == torch.bfloat16:
        dt = ALS_BF16
    else:
        raise TypeError("table dtype must be float32 or bfloat16")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])
    return c_als_table(t.data_ptr() if t.numel() else None, t.shape[0], t.shape[1], ld, dt)


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """Owns an ``als_ctx`` (workspace on one GPU)."""

    def __init__(self, device: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("libals needs a GPU: torch.cuda.is_available() is False")
        self.lib = load_library()
        self.handle = ctypes.c_void_p()
        st = self.lib.als_create(ctypes.byref(self.handle), device)
        if st != ALS_OK:
            raise AlsError(st, self.lib.als_strerror(st).decode())
        self.device = torch.device("cuda", device)

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle.value:
            self.lib.als_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != ALS_OK:
            raise AlsError(st, f"{self.lib.als_strerror(st).decode()}: {self.lib.als_last_error(self.handle).decode()}")


def make_params(alpha: float, lam: float, path: int = PATH_AUTO, dual_max_k: int = 0, split_nnz: int = 0,
                solver: int = 0, cg_max_iters: int = 0, cg_tol: float = 0.0) -> c_als_params:
    return c_als_params(alpha, lam, path, dual_max_k, split_nnz, solver, cg_max_iters, cg_tol)


def als_gramian(ctx: Context, V: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    d = V.shape[1]
    G = out if out is not None else torch.empty((d, d), dtype=torch.float32, device=V.device)
    tv = _table(V)
    ctx._check(ctx.lib.als_gramian(ctx.handle, ctypes.byref(tv), G.data_ptr(), _stream()))
    return G


def als_gramian_static(V: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """als_gramian without a context and without any allocation: ``out`` (fp32 [d, d]) is the caller's."""
    lib = load_library()
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == (V.shape[1], V.shape[1])
    tv = _table(V)
    st = lib.als_gramian_static(V.device.index or 0, ctypes.byref(tv), out.data_ptr(), _stream())
    if st != ALS_OK:
        raise AlsError(st, f"{lib.als_strerror(st).decode()}: {lib.als_static_last_error().decode()}")
    return out


def als_solve_rows(ctx: Context, Y: Csr, V: torch.Tensor, G: torch.Tensor, params: c_als_params, X: torch.Tensor,
                   row_begin: int = 0, row_end: Optional[int] = None) -> torch.Tensor:
    cy, tv, tx = Y.c(), _table(V), _table(X)
    assert G.dtype == torch.float32 and G.is_contiguous()
    row_end = Y.rows if row_end is None else row_end
    ctx._check(ctx.lib.als_solve_rows(ctx.handle, ctypes.byref(cy), ctypes.byref(tv), G.data_ptr(),
                                      ctypes.byref(params), ctypes.byref(tx), row_begin, row_end, _stream()))
    return X


def als_epoch(ctx: Context, Y: Csr, Yt: Csr, W: torch.Tensor, H: torch.Tensor, params: c_als_params) -> None:
    cy, cyt, tw, th = Y.c(), Yt.c(), _table(W), _table(H)
    ctx._check(ctx.lib.als_epoch(ctx.handle, ctypes.byref(cy), ctypes.byref(cyt), ctypes.byref(tw),
                                 ctypes.byref(th), ctypes.byref(params), _stream()))


def als_loss(ctx: Context, Y: Csr, W: torch.Tensor, H: torch.Tensor, params: c_als_params) -> float:
    cy, tw, th = Y.c(), _table(W), _table(H)
    out = ctypes.c_double()
    ctx._check(ctx.lib.als_loss(ctx.handle, ctypes.byref(cy), ctypes.byref(tw), ctypes.byref(th),
                                ctypes.byref(params), ctypes.byref(out), _stream()))
    return out.value


def als_topk(ctx: Context, Q: torch.Tensor, H: torch.Tensor, k: int, exclude: Optional[Csr] = None):
    """Best k rows of H per row of Q by inner product -> (ids int32 [nq, k], scores fp32 [nq, k])."""
    tq, th = _table(Q), _table(H)
    ids = torch.empty((Q.shape[0], k), dtype=torch.int32, device=Q.device)
    scores = torch.empty((Q.shape[0], k), dtype=torch.float32, device=Q.device)
    ex = exclude.c() if exclude is not None else None
    ctx._check(ctx.lib.als_topk(ctx.handle, ctypes.byref(tq), ctypes.byref(th), ctypes.byref(ex) if ex is not None else None,
                                k, ids.data_ptr(), scores.data_ptr(), _stream()))
    return ids, scores


def als_status_sync(ctx: Context) -> None:
    ctx._check(ctx.lib.als_status_sync(ctx.handle, _stream()))


def als_check_csr(ctx: Context, Y: Csr) -> None:
    cy = Y.c()
    ctx._check(ctx.lib.als_check_csr(ctx.handle, ctypes.byref(cy), _stream()))


def als_copy_probe(ctx: Context, src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and src.is_contiguous() and dst.is_contiguous()
    ctx._check(ctx.lib.als_copy_probe(ctx.handle, src.data_ptr(), dst.data_ptr(), nbytes, _stream()))


def als_set_timing(ctx: Context, enabled: bool) -> None:
    ctx._check(ctx.lib.als_set_timing(ctx.handle, int(enabled)))


TIMING_SLOTS = (["gramian", "classify", "transform_z", "transform_x", "primal", "segment", "reduce", "dual_k4", "dual_k8"]
                + [f"dual_k{16 * (c + 1)}" for c in range(8)])


def als_get_timing(ctx: Context) -> dict:
    """ms per kernel slot, and under "launches" the number of timed launches of each slot."""
    n = len(TIMING_SLOTS)
    buf = (ctypes.c_double * (2 * n))()
    ctx._check(ctx.lib.als_get_timing(ctx.handle, buf))
    out = dict(zip(TIMING_SLOTS, list(buf)[:n]))
    out["launches"] = dict(zip(TIMING_SLOTS, list(buf)[n:]))
    return out
