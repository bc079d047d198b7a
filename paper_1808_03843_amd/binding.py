"""ctypes binding of libals_gfx950 (declared in include/als.h).

Argument marshalling only: every step of the ALS path runs in the library's HIP
kernels.  torch is used for device memory and the stream.  There is no CPU
fallback: loading fails loudly when the built library is missing.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import build as _build

ALS_OK, ALS_EINVAL, ALS_EHIP, ALS_ENUMERIC, ALS_ENOMEM = 0, -1, -2, -3, -4
SOLVER_CHOLESKY, SOLVER_CG = 0, 1
F32, BF16, F16, F32X3, F32X2 = 0, 1, 2, 3, 4
PEAK_MFMA_F32, PEAK_MFMA_BF16, PEAK_MFMA_F16, PEAK_COPY = 0, 1, 2, 3   # ids of als_measure_peak
K_HERMITIAN, K_SOLVE, K_RMSE, K_PLAN, K_FUSED, K_GRAM, K_SHORT = 0, 1, 2, 3, 4, 5, 6

EXPORTS = [
    "als_create", "als_destroy", "als_last_error", "als_update_rows", "als_update_cols", "als_rmse",
    "als_hermitian", "als_bin_rows", "als_csr_to_csc", "als_synchronize", "als_kernel_time",
    "als_profile_reset", "als_drop_plans", "als_check_matrix", "als_measure_peak", "als_update_rows_implicit", "als_update_cols_implicit", "als_implicit_loss", "als_gram",
    "als_gram_static", "als_workspace_bytes", "als_short_row_limit",
]


class AlsSparse(ctypes.Structure):
    _fields_ = [("nrows", ctypes.c_int64), ("ncols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("ptr", ctypes.c_void_p), ("ptr_is_64", ctypes.c_int32),
                ("idx", ctypes.c_void_p), ("val", ctypes.c_void_p)]


class AlsConfig(ctypes.Structure):
    _fields_ = [("f", ctypes.c_int32), ("solver", ctypes.c_int32), ("cg_iters", ctypes.c_int32),
                ("cg_eps", ctypes.c_float), ("factor_dtype", ctypes.c_int32), ("herm_dtype", ctypes.c_int32),
                ("device", ctypes.c_int32), ("stream", ctypes.c_void_p), ("chunk", ctypes.c_int32),
                ("batch_slots", ctypes.c_int64), ("profile", ctypes.c_int32),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("workspace_max_rows", ctypes.c_int64), ("workspace_max_nnz", ctypes.c_int64),
                ("dense_short_rows", ctypes.c_int32)]


_lib = None


def _declare(lib: ctypes.CDLL) -> ctypes.CDLL:
    vp, i32, i64, fl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    sp = ctypes.POINTER(AlsSparse)
    lib.als_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(AlsConfig)]
    lib.als_workspace_bytes.argtypes = [ctypes.POINTER(AlsConfig), i64, i64]
    lib.als_workspace_bytes.restype = ctypes.c_size_t
    lib.als_destroy.argtypes = [vp]
    lib.als_destroy.restype = None
    lib.als_last_error.argtypes = [vp]
    lib.als_last_error.restype = ctypes.c_char_p
    lib.als_update_rows.argtypes = [vp, sp, vp, fl, ctypes.c_int, vp]
    lib.als_update_cols.argtypes = [vp, sp, vp, fl, ctypes.c_int, vp]
    lib.als_rmse.argtypes = [vp, sp, vp, vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    lib.als_update_rows_implicit.argtypes = [vp, sp, vp, fl, fl, ctypes.c_int, vp]
    lib.als_update_cols_implicit.argtypes = [vp, sp, vp, fl, fl, ctypes.c_int, vp]
    lib.als_implicit_loss.argtypes = [vp, sp, vp, vp, fl, fl, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    lib.als_gram.argtypes = [vp, vp, i64, ctypes.c_int, vp]
    lib.als_gram_static.argtypes = [vp, vp, i64, ctypes.c_int, vp]
    lib.als_hermitian.argtypes = [vp, sp, vp, fl, ctypes.c_int, i64, i64, vp, vp]
    lib.als_bin_rows.argtypes = [vp, sp, ctypes.c_int, vp, ctypes.POINTER(i64)]
    lib.als_csr_to_csc.argtypes = [vp, sp, vp, vp, vp]
    lib.als_synchronize.argtypes = [vp]
    lib.als_kernel_time.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    lib.als_profile_reset.argtypes = [vp]
    lib.als_drop_plans.argtypes = [vp]
    lib.als_check_matrix.argtypes = [vp, sp]
    lib.als_measure_peak.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    lib.als_short_row_limit.argtypes = [vp]
    return lib


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads the in-tree library, building it first only if it was never built.  With `path`: another build of the
    same library (e.g. build.LIB_DRAINED), loaded beside the default one and handed to Als(library=...)."""
    global _lib
    if path is not None:
        if not os.path.exists(path):
            raise FileNotFoundError(path)
        return _declare(ctypes.CDLL(path))
    if _lib is not None:
        return _lib
    path = os.environ.get("ALS_LIBRARY", _build.LIB)   # ALS_LIBRARY: an alternative build, for tuning runs
    if not os.path.exists(path):
        if path != _build.LIB:
            raise FileNotFoundError(path)
        _build.build()
    _lib = _declare(ctypes.CDLL(path))
    return _lib


class AlsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libals_gfx950 error {code}: {text}")
        self.code = code


class SparseMatrix:
    """Device-resident compressed rows (torch tensors own the memory)."""
    _serials = 0

    def __init__(self, nrows: int, ncols: int, ptr: torch.Tensor, idx: torch.Tensor, val: torch.Tensor):
        assert ptr.is_cuda and idx.is_cuda and val.is_cuda
        assert ptr.dtype in (torch.int32, torch.int64) and idx.dtype == torch.int32 and val.dtype == torch.float32
        assert ptr.numel() == nrows + 1 and idx.numel() == val.numel()
        self.nrows, self.ncols = int(nrows), int(ncols)
        self.ptr, self.idx, self.val = ptr.contiguous(), idx.contiguous(), val.contiguous()
        self.nnz = int(idx.numel())
        self.desc = AlsSparse(self.nrows, self.ncols, self.nnz, self.ptr.data_ptr(),
                              1 if ptr.dtype == torch.int64 else 0, self.idx.data_ptr(), self.val.data_ptr())
        SparseMatrix._serials += 1
        self.serial = SparseMatrix._serials   # tells two matrices apart that torch put at the same address

    @staticmethod
    def from_host(nrows, ncols, ptr, idx, val, device="cuda:0", ptr64: Optional[bool] = None) -> "SparseMatrix":
        import numpy as np
        nnz = int(ptr[-1])
        if ptr64 is None:
            ptr64 = nnz >= 2 ** 31
        p = torch.from_numpy(np.ascontiguousarray(ptr, dtype=np.int64 if ptr64 else np.int32)).to(device)
        i = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).to(device)
        v = torch.from_numpy(np.ascontiguousarray(val, dtype=np.float32)).to(device)
        return SparseMatrix(nrows, ncols, p, i, v)


class Als:
    """One library context (als_create .. als_destroy) bound to a device and a stream."""

    def __init__(self, f: int, solver: int = SOLVER_CHOLESKY, cg_iters: int = 6, cg_eps: float = 0.0,
                 device: int = 0, stream: Optional[int] = None, chunk: int = 0, batch_slots: int = 0,
                 profile: bool = False, factor_dtype: int = F32, herm_dtype: int = F32,
                 workspace_rows: int = 0, workspace_nnz: int = 0, library: Optional[ctypes.CDLL] = None,
                 dense_short_rows: bool = False):
        """dense_short_rows: every row builds A_u, also the short ones (see als_config in include/als.h).
        workspace_rows / workspace_nnz > 0: the library works in a torch-allocated workspace sized for matrices of
        at most that many rows and stored entries, and allocates no device memory itself.
        library: another build of the library from load_library(path) (default: the in-tree build)."""
        self._lib = library if library is not None else load_library()
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        self.cfg = AlsConfig(f, solver, cg_iters, cg_eps, factor_dtype, herm_dtype, device, stream, chunk, batch_slots,
                             1 if profile else 0)
        self.cfg.dense_short_rows = 1 if dense_short_rows else 0
        self.workspace = None
        if workspace_rows > 0 or workspace_nnz > 0:
            need = self._lib.als_workspace_bytes(ctypes.byref(self.cfg), workspace_rows, workspace_nnz)
            if need == 0:
                raise AlsError(ALS_EINVAL, "als_workspace_bytes refused the configuration")
            self.workspace = torch.empty(need, dtype=torch.uint8, device=f"cuda:{device}")   # torch owns the memory
            assert self.workspace.data_ptr() % 256 == 0
            self.cfg.workspace, self.cfg.workspace_bytes = self.workspace.data_ptr(), need
            self.cfg.workspace_max_rows, self.cfg.workspace_max_nnz = workspace_rows, workspace_nnz
        self._ctx = ctypes.c_void_p()
        rc = self._lib.als_create(ctypes.byref(self._ctx), ctypes.byref(self.cfg))
        if rc != ALS_OK:
            self._ctx = ctypes.c_void_p()
            raise AlsError(rc, "als_create failed (unsupported f / solver / dtype, or no such device)")
        self.f = f
        self._plan_owner = {}
        self.factor_torch_dtype = {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16, F32X3: torch.float32, F32X2: torch.float32}[factor_dtype]

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx:
            self._lib.als_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _matrix(self, sp: "SparseMatrix"):
        """Descriptor of a matrix for a call that uses its cached plan.  The library keys plans on the address of
        ptr; when torch has handed the address of a freed matrix to a new one, the plans are dropped first."""
        key = sp.desc.ptr
        if self._plan_owner.get(key, sp.serial) != sp.serial:
            self.drop_plans()
            self._plan_owner.clear()
        self._plan_owner[key] = sp.serial
        return ctypes.byref(sp.desc)

    def _check(self, rc: int):
        if rc != ALS_OK:
            raise AlsError(rc, self._lib.als_last_error(self._ctx).decode())

    @staticmethod
    def _factor(t: torch.Tensor, rows: int, f: int, dtype=torch.float32):
        assert t.is_cuda and t.dtype == dtype and t.is_contiguous() and tuple(t.shape) == (rows, f)
        return t.data_ptr()

    def _gathered(self, t: torch.Tensor, rows: int):
        """The factor matrix that is read (config's factor_dtype)."""
        return self._factor(t, rows, self.f, self.factor_torch_dtype)

    def update_rows(self, csr: SparseMatrix, Theta: torch.Tensor, lam: float, X: torch.Tensor):
        self._check(self._lib.als_update_rows(self._ctx, self._matrix(csr), self._gathered(Theta, csr.ncols),
                                              lam, self.f, self._factor(X, csr.nrows, self.f)))

    def update_cols(self, csc: SparseMatrix, X: torch.Tensor, lam: float, Theta: torch.Tensor):
        self._check(self._lib.als_update_cols(self._ctx, self._matrix(csc), self._gathered(X, csc.ncols),
                                              lam, self.f, self._factor(Theta, csc.nrows, self.f)))

    def update_rows_implicit(self, csr: SparseMatrix, Theta: torch.Tensor, lam: float, alpha: float, X: torch.Tensor):
        self._check(self._lib.als_update_rows_implicit(self._ctx, self._matrix(csr),
                                                       self._gathered(Theta, csr.ncols), lam, alpha, self.f,
                                                       self._factor(X, csr.nrows, self.f)))

    def update_cols_implicit(self, csc: SparseMatrix, X: torch.Tensor, lam: float, alpha: float, Theta: torch.Tensor):
        self._check(self._lib.als_update_cols_implicit(self._ctx, self._matrix(csc),
                                                       self._gathered(X, csc.ncols), lam, alpha, self.f,
                                                       self._factor(Theta, csc.nrows, self.f)))

    def implicit_loss(self, csr: SparseMatrix, X: torch.Tensor, Theta: torch.Tensor, lam: float, alpha: float) -> float:
        out = ctypes.c_double()
        self._check(self._lib.als_implicit_loss(self._ctx, self._matrix(csr), self._factor(X, csr.nrows, self.f),
                                                self._factor(Theta, csr.ncols, self.f), lam, alpha, self.f,
                                                ctypes.byref(out)))
        return out.value

    def gram(self, G: torch.Tensor) -> torch.Tensor:
        out = torch.empty((self.f, self.f), dtype=torch.float32, device=G.device)
        self._check(self._lib.als_gram(self._ctx, self._factor(G, G.shape[0], self.f), G.shape[0], self.f,
                                       out.data_ptr()))
        return out

    def gram_static(self, G: torch.Tensor, out: torch.Tensor) -> None:
        """als_gram without allocation: the caller passes the output too (f x f float)."""
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == (self.f, self.f)
        self._check(self._lib.als_gram_static(self._ctx, self._factor(G, G.shape[0], self.f), G.shape[0], self.f,
                                              out.data_ptr()))

    def rmse(self, csr: SparseMatrix, X: torch.Tensor, Theta: torch.Tensor) -> float:
        out = ctypes.c_double()
        self._check(self._lib.als_rmse(self._ctx, self._matrix(csr), self._factor(X, csr.nrows, self.f),
                                       self._factor(Theta, csr.ncols, self.f), self.f, ctypes.byref(out)))
        return out.value

    def hermitian(self, csr: SparseMatrix, Theta: torch.Tensor, lam: float, row0: int, nrows: int):
        A = torch.empty((nrows, self.f, self.f), dtype=torch.float32, device=Theta.device)
        b = torch.empty((nrows, self.f), dtype=torch.float32, device=Theta.device)
        self._check(self._lib.als_hermitian(self._ctx, self._matrix(csr), self._gathered(Theta, csr.ncols),
                                            lam, self.f, row0, nrows, A.data_ptr(), b.data_ptr()))
        return A, b

    def bin_rows(self, csr: SparseMatrix, nclass: int):
        perm = torch.empty(csr.nrows, dtype=torch.int32, device=csr.idx.device)
        start = (ctypes.c_int64 * (nclass + 1))()
        self._check(self._lib.als_bin_rows(self._ctx, ctypes.byref(csr.desc), nclass, perm.data_ptr(), start))
        return perm, list(start)

    def csr_to_csc(self, csr: SparseMatrix) -> SparseMatrix:
        dev = csr.idx.device
        cptr = torch.empty(csr.ncols + 1, dtype=csr.ptr.dtype, device=dev)
        cidx = torch.empty(csr.nnz, dtype=torch.int32, device=dev)
        cval = torch.empty(csr.nnz, dtype=torch.float32, device=dev)
        self._check(self._lib.als_csr_to_csc(self._ctx, ctypes.byref(csr.desc), cptr.data_ptr(), cidx.data_ptr(),
                                             cval.data_ptr()))
        return SparseMatrix(csr.ncols, csr.nrows, cptr, cidx, cval)

    def synchronize(self):
        self._check(self._lib.als_synchronize(self._ctx))

    def kernel_time(self, kernel_id: int):
        ms, n = ctypes.c_double(), ctypes.c_int64()
        self._check(self._lib.als_kernel_time(self._ctx, kernel_id, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def profile_reset(self):
        self._check(self._lib.als_profile_reset(self._ctx))

    def check_matrix(self, sp: "SparseMatrix"):
        """Raise AlsError unless ptr, the range of the column ids and their order inside every row are sound."""
        self._check(self._lib.als_check_matrix(self._ctx, ctypes.byref(sp.desc)))

    def short_row_limit(self) -> int:
        """Rows with fewer stored entries than this run Algorithm 1 on their gathered rows (0: none)."""
        return int(self._lib.als_short_row_limit(self._ctx))

    def measure_peak(self, what: int) -> float:
        """Sustained rate of the device: what = 0 / 1 / 2 MFMA fp32 / bf16 / fp16 (flop/s), 3 streaming copy (B/s)."""
        out = ctypes.c_double()
        self._check(self._lib.als_measure_peak(self._ctx, what, ctypes.byref(out)))
        return out.value

    def drop_plans(self):
        """Forget the cached work plans: needed after a matrix's arrays changed in place or were reallocated."""
        self._check(self._lib.als_drop_plans(self._ctx))
