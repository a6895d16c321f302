"""Thin ctypes binding over the C ABI of libftk.so (declared in include/ftk.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
Function names and argument order follow the header.  numpy arrays are passed as host
pointers; torch CUDA tensors (optional) as device pointers.  There is no CPU fallback: if
the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import importlib.util
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# FTK_LIB points the binding at another build of the library (kernel experiments)
LIB_PATH = os.environ.get("FTK_LIB") or os.path.join(HERE, "libftk.so")

FTK_OK, FTK_EINVAL, FTK_ENOMEM, FTK_EDEVICE, FTK_ESTATE, FTK_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
FTK_PTRS_HOST, FTK_PTRS_DEVICE, FTK_LAYOUT_EXACT = 0, 1, 2
FTK_SYNC, FTK_HOGWILD, FTK_HOGWILD_MODEWISE = 0, 1, 2
FTK_SAMPLE_ENTRIES, FTK_SAMPLE_TILES = 0, 1
FTK_K_SAMPLE, FTK_K_GRAD, FTK_K_APPLY, FTK_K_COUNT = 0, 1, 2, 3
FTK_MAX_ORDER = 10

# every symbol include/ftk.h declares
SYMBOLS = [
    "ftk_create", "ftk_destroy", "ftk_sample", "ftk_get_samples", "ftk_sgd_step", "ftk_sgd_step_noalloc", "ftk_rmse", "ftk_mae",
    "ftk_evaluate", "ftk_step_size", "ftk_set_sampling",
    "ftk_get_factors", "ftk_set_factors", "ftk_set_mode", "ftk_set_stream", "ftk_set_timing",
    "ftk_get_timing", "ftk_set_kernel", "ftk_kernel_name", "ftk_get_table_rows", "ftk_last_error",
]


def ftk_step_size(alpha: float, beta: float, t: int) -> float:
    """alpha / (1 + beta * t^1.5), evaluated by the library (host function, needs no GPU)."""
    return float(load().ftk_step_size(float(alpha), float(beta), int(t)))


class FtkError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("ftk error %d: %s" % (code, message))
        self.code = code


_lib = None


def hip_runtime_path() -> str:
    """The one HIP runtime this process should use.  libftk.so is built without a link-time
    dependency on it, because two copies of the runtime in one process cannot both reach the
    GPU: PyTorch bundles its own, so that one wins whenever PyTorch is installed."""
    override = os.environ.get("FTK_HIP_RUNTIME")
    if override:
        return override
    try:
        spec = importlib.util.find_spec("torch")
    except (ImportError, ValueError):
        spec = None
    if spec is not None and spec.origin:
        bundled = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
        if os.path.exists(bundled):
            return bundled
    return "/opt/rocm/lib/libamdhip64.so"


def load():
    """Load libftk.so (built by `python -m paper_2204_07104_amd.build`).  Raises if missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2204_07104_amd.build` (there is no CPU fallback)" % LIB_PATH)
    C.CDLL(hip_runtime_path(), mode=C.RTLD_GLOBAL)
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    L.ftk_create.argtypes = [C.POINTER(vp), C.c_int32, vp, C.c_int64, vp, vp, vp, C.c_int32, C.c_uint64, C.c_uint32]
    L.ftk_create.restype = C.c_int
    L.ftk_destroy.argtypes = [vp]
    L.ftk_destroy.restype = None
    L.ftk_sample.argtypes = [vp, C.c_uint64, C.c_int64]
    L.ftk_sample.restype = C.c_int
    L.ftk_get_samples.argtypes = [vp, vp]
    L.ftk_get_samples.restype = C.c_int
    L.ftk_sgd_step.argtypes = [vp, C.c_float, C.c_float, C.c_float, C.c_float]
    L.ftk_sgd_step.restype = C.c_int
    L.ftk_sgd_step_noalloc.argtypes = [vp, C.c_float, C.c_float, C.c_float, C.c_float]
    L.ftk_sgd_step_noalloc.restype = C.c_int
    L.ftk_rmse.argtypes = [vp, C.POINTER(C.c_double)]
    L.ftk_rmse.restype = C.c_int
    L.ftk_mae.argtypes = [vp, C.POINTER(C.c_double)]
    L.ftk_mae.restype = C.c_int
    L.ftk_evaluate.argtypes = [vp, C.c_int64, vp, vp, C.c_uint32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.ftk_evaluate.restype = C.c_int
    L.ftk_step_size.argtypes = [C.c_double, C.c_double, C.c_int64]
    L.ftk_step_size.restype = C.c_double
    L.ftk_get_factors.argtypes = [vp, vp, vp]
    L.ftk_get_factors.restype = C.c_int
    L.ftk_set_factors.argtypes = [vp, vp, vp]
    L.ftk_set_factors.restype = C.c_int
    L.ftk_set_sampling.argtypes = [vp, C.c_int]
    L.ftk_set_sampling.restype = C.c_int
    L.ftk_set_mode.argtypes = [vp, C.c_int]
    L.ftk_set_mode.restype = C.c_int
    L.ftk_set_stream.argtypes = [vp, vp]
    L.ftk_set_stream.restype = C.c_int
    L.ftk_set_timing.argtypes = [vp, C.c_int]
    L.ftk_set_timing.restype = C.c_int
    L.ftk_get_timing.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]
    L.ftk_get_timing.restype = C.c_int
    L.ftk_set_kernel.argtypes = [vp, C.c_char_p]
    L.ftk_set_kernel.restype = C.c_int
    L.ftk_kernel_name.argtypes = [vp]
    L.ftk_kernel_name.restype = C.c_char_p
    L.ftk_get_table_rows.argtypes = [vp, vp, vp]
    L.ftk_get_table_rows.restype = C.c_int
    L.ftk_last_error.argtypes = [vp]
    L.ftk_last_error.restype = C.c_char_p
    _lib = L
    return L


def _is_torch_cuda(x) -> bool:
    return hasattr(x, "is_cuda") and bool(x.is_cuda)


def _ptr_list(ptrs: Sequence[Optional[int]]):
    arr = (C.c_void_p * len(ptrs))()
    for k, p in enumerate(ptrs):
        arr[k] = p
    return arr


class FastTucker:
    """One tensor + its parameters + the current sample set (an ftk_ctx)."""

    def __init__(self, dims: Sequence[int], idx: Sequence, vals, J: Sequence[int], R: int, init_seed: int = 1,
                 flags: int = 0):
        L = load()
        self._L = L
        self._ctx = C.c_void_p(None)
        N = len(dims)
        if len(idx) != N or len(J) != N:
            raise ValueError("dims, idx and J must have one entry per mode")
        self.dims = tuple(int(d) for d in dims)
        self.J = tuple(int(j) for j in J)
        self.R = int(R)
        self.order = N
        on_device = _is_torch_cuda(vals)
        if on_device:
            import torch
            for a in idx:
                if not _is_torch_cuda(a) or a.dtype != torch.int32 or not a.is_contiguous():
                    raise ValueError("idx[n] must be contiguous int32 CUDA tensors when vals is one")
            if vals.dtype != torch.float32 or not vals.is_contiguous():
                raise ValueError("vals must be a contiguous float32 tensor")
            nnz = int(vals.numel())
            ptrs = [int(a.data_ptr()) for a in idx]
            vptr = int(vals.data_ptr())
            flags = int(flags) | FTK_PTRS_DEVICE
        else:
            idx = [np.ascontiguousarray(a, dtype=np.int32) for a in idx]
            vals = np.ascontiguousarray(vals, dtype=np.float32)
            nnz = int(vals.shape[0])
            ptrs = [a.ctypes.data for a in idx]
            vptr = vals.ctypes.data
            flags = int(flags) & ~FTK_PTRS_DEVICE
        for a in idx:
            if int(a.shape[0]) != nnz:
                raise ValueError("idx[n] and vals must all have nnz entries")
        self.nnz = nnz
        dims_a = np.asarray(self.dims, dtype=np.int64)
        J_a = np.asarray(self.J, dtype=np.int32)
        idx_ptrs = _ptr_list(ptrs)
        rc = L.ftk_create(C.byref(self._ctx), N, dims_a.ctypes.data, nnz, C.cast(idx_ptrs, C.c_void_p),
                          vptr, J_a.ctypes.data, self.R, int(init_seed), flags)
        if rc != FTK_OK:
            msg = L.ftk_last_error(None)
            self._ctx = C.c_void_p(None)
            raise FtkError(rc, msg.decode() if msg else "")

    # -- helpers -------------------------------------------------------------------------------
    def _check(self, rc: int):
        if rc != FTK_OK:
            msg = self._L.ftk_last_error(self._ctx)
            raise FtkError(rc, msg.decode() if msg else "")

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._L.ftk_destroy(self._ctx)
            self._ctx = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- the ABI, one method per entry point ----------------------------------------------------
    def ftk_sample(self, seed: int, n_samples: int) -> None:
        self._check(self._L.ftk_sample(self._ctx, int(seed), int(n_samples)))
        self._n_samples = int(n_samples)

    def ftk_get_samples(self) -> np.ndarray:
        out = np.empty(getattr(self, "_n_samples", 0) or 1, dtype=np.int64)
        self._check(self._L.ftk_get_samples(self._ctx, out.ctypes.data))
        return out

    def ftk_sgd_step(self, lr_A: float, lr_B: float, lambda_A: float, lambda_B: float) -> None:
        self._check(self._L.ftk_sgd_step(self._ctx, lr_A, lr_B, lambda_A, lambda_B))

    def ftk_sgd_step_noalloc(self, lr_A: float, lr_B: float, lambda_A: float, lambda_B: float) -> None:
        self._check(self._L.ftk_sgd_step_noalloc(self._ctx, lr_A, lr_B, lambda_A, lambda_B))

    def ftk_rmse(self) -> float:
        out = C.c_double(0.0)
        self._check(self._L.ftk_rmse(self._ctx, C.byref(out)))
        return out.value

    def ftk_mae(self) -> float:
        out = C.c_double(0.0)
        self._check(self._L.ftk_mae(self._ctx, C.byref(out)))
        return out.value

    def ftk_evaluate(self, idx: Sequence[np.ndarray], vals: np.ndarray) -> Tuple[float, float]:
        """(RMSE, MAE) of the current parameters on a held-out set given as host arrays."""
        if len(idx) != self.order:
            raise ValueError("idx must hold one array per mode")
        cols = [np.ascontiguousarray(a, dtype=np.int32) for a in idx]
        v = np.ascontiguousarray(vals, dtype=np.float32)
        n_eval = int(v.shape[0])
        if any(a.shape != (n_eval,) for a in cols):
            raise ValueError("idx arrays and vals must have the same length")
        ptrs = (C.c_void_p * self.order)(*[a.ctypes.data for a in cols])
        rmse, mae = C.c_double(0.0), C.c_double(0.0)
        self._check(self._L.ftk_evaluate(self._ctx, n_eval, ptrs, v.ctypes.data, 0, C.byref(rmse), C.byref(mae)))
        return rmse.value, mae.value

    def ftk_get_factors(self) -> Tuple[List[np.ndarray], List[np.ndarray]]:
        A = [np.empty((self.dims[n], self.J[n]), dtype=np.float32) for n in range(self.order)]
        B = [np.empty((self.J[n], self.R), dtype=np.float32) for n in range(self.order)]
        pa = _ptr_list([a.ctypes.data for a in A])
        pb = _ptr_list([b.ctypes.data for b in B])
        self._check(self._L.ftk_get_factors(self._ctx, C.cast(pa, C.c_void_p), C.cast(pb, C.c_void_p)))
        return A, B

    def ftk_set_factors(self, A: Optional[Sequence[np.ndarray]], B: Optional[Sequence[np.ndarray]]) -> None:
        keep = []
        pa = pb = None
        if A is not None:
            A = [np.ascontiguousarray(a, dtype=np.float32) for a in A]
            for n, a in enumerate(A):
                if a.shape != (self.dims[n], self.J[n]):
                    raise ValueError("A[%d] must have shape %r" % (n, (self.dims[n], self.J[n])))
            pa = _ptr_list([a.ctypes.data for a in A])
            keep.append(A)
        if B is not None:
            B = [np.ascontiguousarray(b, dtype=np.float32) for b in B]
            for n, b in enumerate(B):
                if b.shape != (self.J[n], self.R):
                    raise ValueError("B[%d] must have shape %r" % (n, (self.J[n], self.R)))
            pb = _ptr_list([b.ctypes.data for b in B])
            keep.append(B)
        self._check(self._L.ftk_set_factors(self._ctx, C.cast(pa, C.c_void_p) if pa is not None else None,
                                            C.cast(pb, C.c_void_p) if pb is not None else None))

    def ftk_set_sampling(self, rule: int) -> None:
        self._check(self._L.ftk_set_sampling(self._ctx, int(rule)))

    def ftk_set_mode(self, mode: int) -> None:
        self._check(self._L.ftk_set_mode(self._ctx, int(mode)))

    def ftk_set_stream(self, hip_stream: Optional[int]) -> None:
        self._check(self._L.ftk_set_stream(self._ctx, hip_stream))

    def ftk_set_timing(self, enabled: bool) -> None:
        self._check(self._L.ftk_set_timing(self._ctx, 1 if enabled else 0))

    def ftk_get_timing(self, which: int, reset: bool = False) -> Tuple[float, int]:
        ms = C.c_double(0.0)
        cnt = C.c_int64(0)
        self._check(self._L.ftk_get_timing(self._ctx, int(which), C.byref(ms), C.byref(cnt), 1 if reset else 0))
        return ms.value, cnt.value

    def ftk_set_kernel(self, name: str) -> None:
        self._check(self._L.ftk_set_kernel(self._ctx, name.encode()))

    def ftk_kernel_name(self) -> str:
        return self._L.ftk_kernel_name(self._ctx).decode()

    def ftk_get_table_rows(self) -> Tuple[np.ndarray, np.ndarray]:
        """(K, top): per mode, how many of the most frequent rows are summed in the workgroup tables /
        through the one-hot product for the current |Psi|."""
        K = np.zeros(self.order, dtype=np.int32)
        top = np.zeros(self.order, dtype=np.int32)
        self._check(self._L.ftk_get_table_rows(self._ctx, K.ctypes.data, top.ctypes.data))
        return K, top
