"""CPU oracle for the sampled-SGD FastTucker step (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product path never does: it fails
loudly when the HIP library is missing.

The arithmetic lives in ``ftk_oracle.cpp`` (single-threaded C++17, double
accumulators); this file only compiles it with g++ and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# FTK_ORACLE_SOURCE / FTK_ORACLE_LIB redirect the build to another source file: the mutation
# test uses them to check that a planted mistake in the oracle trips one of its pins.
_SRC = os.environ.get("FTK_ORACLE_SOURCE") or os.path.join(_HERE, "ftk_oracle.cpp")
_LIB = os.environ.get("FTK_ORACLE_LIB") or os.path.join(_HERE, "libftk_oracle.so")
ORACLE_CXXFLAGS = ["-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra"]

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle (g++ -O2, no -ffast-math).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", *ORACLE_CXXFLAGS, _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_pp_f = C.POINTER(C.POINTER(C.c_float))
_pp_i = C.POINTER(C.POINTER(C.c_int32))
_pp_d = C.POINTER(C.POINTER(C.c_double))


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.fto_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.fto_philox4x32_10.restype = None
        L.fto_sample_positions.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_void_p]
        L.fto_sample_positions.restype = C.c_int
        L.fto_sample_positions_tiles.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_void_p]
        L.fto_sample_positions_tiles.restype = C.c_int
        L.fto_tile_order_constants.argtypes = [C.c_int64, C.c_void_p, C.c_void_p]
        L.fto_tile_order_constants.restype = C.c_int
        L.fto_init_uniform.argtypes = [C.c_uint64, C.c_int32, C.c_int64, C.c_void_p]
        L.fto_init_uniform.restype = C.c_int
        L.fto_nonzero_terms.argtypes = [C.c_int32, C.c_void_p, C.c_int32, _pp_f, _pp_f,
                                        C.c_void_p, C.c_void_p, C.c_void_p, _pp_d]
        L.fto_nonzero_terms.restype = C.c_int
        L.fto_sgd_step_sync.argtypes = [C.c_int32, C.c_void_p, C.c_int64, _pp_i, C.c_void_p,
                                        C.c_void_p, C.c_int32, _pp_f, _pp_f, C.c_void_p,
                                        C.c_int64, C.c_float, C.c_float, C.c_float, C.c_float]
        L.fto_sgd_step_sync.restype = C.c_int
        L.fto_sgd_step_hogwild.argtypes = L.fto_sgd_step_sync.argtypes
        L.fto_sgd_step_hogwild.restype = C.c_int
        L.fto_errors.argtypes = [C.c_int32, C.c_void_p, C.c_int64, _pp_i, C.c_void_p, C.c_void_p,
                                 C.c_int32, _pp_f, _pp_f, C.c_void_p, C.c_int64, C.c_void_p,
                                 C.c_void_p]
        L.fto_errors.restype = C.c_int
    return _lib


def _ptr_array(arrays: Sequence[np.ndarray], ctype):
    arr = (C.POINTER(ctype) * len(arrays))()
    for k, a in enumerate(arrays):
        arr[k] = a.ctypes.data_as(C.POINTER(ctype))
    return arr


def _check_f32(arrays, shapes):
    out = []
    for a, shp in zip(arrays, shapes):
        if a.dtype != np.float32 or not a.flags.c_contiguous or tuple(a.shape) != tuple(shp):
            raise ValueError("expected C-contiguous float32 array of shape %r, got %r %r"
                             % (shp, a.dtype, a.shape))
        out.append(a)
    return out


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().fto_philox4x32_10(c.ctypes.data, k.ctypes.data, o.ctypes.data)
    return tuple(int(v) for v in o)


def sample_positions(seed: int, n_samples: int, nnz: int) -> np.ndarray:
    pos = np.empty(n_samples, dtype=np.int64)
    rc = lib().fto_sample_positions(seed, n_samples, nnz, pos.ctypes.data)
    if rc:
        raise ValueError("fto_sample_positions failed: %d" % rc)
    return pos


def tile_order_constants(nnz: int) -> Tuple[int, int]:
    """(a, b) of the fixed pseudo-random order pi(q) = (a q + b) mod nnz used by tile sampling."""
    a, b = C.c_int64(0), C.c_int64(0)
    if lib().fto_tile_order_constants(nnz, C.addressof(a), C.addressof(b)):
        raise ValueError("fto_tile_order_constants failed")
    return a.value, b.value


def sample_positions_tiles(seed: int, n_samples: int, nnz: int) -> np.ndarray:
    """Psi under the tile-sampling variant: runs of 64 neighbours in the order pi (caller's positions)."""
    out = np.empty(n_samples, dtype=np.int64)
    if lib().fto_sample_positions_tiles(seed & (2**64 - 1), n_samples, nnz, out.ctypes.data):
        raise ValueError("fto_sample_positions_tiles failed")
    return out


def init_uniform(init_seed: int, array_id: int, shape) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    rc = lib().fto_init_uniform(init_seed, array_id, out.size, out.ctypes.data)
    if rc:
        raise ValueError("fto_init_uniform failed: %d" % rc)
    return out


def init_factors(init_seed: int, dims, J, R) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    N = len(dims)
    A = [init_uniform(init_seed, n, (int(dims[n]), int(J[n]))) for n in range(N)]
    B = [init_uniform(init_seed, N + n, (int(J[n]), int(R))) for n in range(N)]
    return A, B


def nonzero_terms(a_rows: Sequence[np.ndarray], B: Sequence[np.ndarray]):
    """c, w, GS and xhat of one nonzero.  Returns (xhat, c[N,R], w[N,R], [gs_n])."""
    N = len(a_rows)
    R = int(B[0].shape[1])
    J = np.asarray([b.shape[0] for b in B], dtype=np.int32)
    a_rows = _check_f32(a_rows, [(int(j),) for j in J])
    B = _check_f32(B, [(int(j), R) for j in J])
    xhat = C.c_double(0.0)
    c = np.zeros((N, R))
    w = np.zeros((N, R))
    gs = [np.zeros(int(j)) for j in J]
    rc = lib().fto_nonzero_terms(N, J.ctypes.data, R, _ptr_array(a_rows, C.c_float),
                                 _ptr_array(B, C.c_float), C.addressof(xhat), c.ctypes.data,
                                 w.ctypes.data, _ptr_array(gs, C.c_double))
    if rc:
        raise ValueError("fto_nonzero_terms failed: %d" % rc)
    return xhat.value, c, w, gs


def _tensor_args(dims, idx, vals, A, B):
    N = len(dims)
    dims_a = np.asarray(dims, dtype=np.int64)
    nnz = int(vals.shape[0])
    for n in range(N):
        if idx[n].dtype != np.int32 or not idx[n].flags.c_contiguous or idx[n].shape != (nnz,):
            raise ValueError("idx[%d] must be contiguous int32[nnz]" % n)
    if vals.dtype != np.float32 or not vals.flags.c_contiguous:
        raise ValueError("vals must be contiguous float32")
    R = int(B[0].shape[1])
    J = np.asarray([b.shape[0] for b in B], dtype=np.int32)
    A = _check_f32(A, [(int(dims[n]), int(J[n])) for n in range(N)])
    B = _check_f32(B, [(int(J[n]), R) for n in range(N)])
    return N, dims_a, nnz, J, R, A, B


def sgd_step_sync(dims, idx, vals, A, B, pos, lr_A, lr_B, lambda_A, lambda_B) -> None:
    """One synchronous step over Psi = pos; A and B (lists of float32 arrays) change in place."""
    N, dims_a, nnz, J, R, A, B = _tensor_args(dims, idx, vals, A, B)
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    rc = lib().fto_sgd_step_sync(N, dims_a.ctypes.data, nnz, _ptr_array(idx, C.c_int32),
                                 vals.ctypes.data, J.ctypes.data, R, _ptr_array(A, C.c_float),
                                 _ptr_array(B, C.c_float), pos.ctypes.data, int(pos.shape[0]),
                                 lr_A, lr_B, lambda_A, lambda_B)
    if rc:
        raise ValueError("fto_sgd_step_sync failed: %d" % rc)


def sgd_step_hogwild(dims, idx, vals, A, B, pos, lr_A, lr_B, lambda_A, lambda_B) -> None:
    """One step in the order Algorithm 1 prints (rows overwritten sample by sample, mode by mode;
    core factors from the accumulated gradient afterwards), run sequentially.  In place."""
    N, dims_a, nnz, J, R, A, B = _tensor_args(dims, idx, vals, A, B)
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    rc = lib().fto_sgd_step_hogwild(N, dims_a.ctypes.data, nnz, _ptr_array(idx, C.c_int32),
                                    vals.ctypes.data, J.ctypes.data, R, _ptr_array(A, C.c_float),
                                    _ptr_array(B, C.c_float), pos.ctypes.data, int(pos.shape[0]),
                                    lr_A, lr_B, lambda_A, lambda_B)
    if rc:
        raise ValueError("fto_sgd_step_hogwild failed: %d" % rc)


def errors(dims, idx, vals, A, B, positions: Optional[np.ndarray] = None) -> Tuple[float, float]:
    """(RMSE, MAE) over the given stored positions (default: all stored nonzeros)."""
    N, dims_a, nnz, J, R, A, B = _tensor_args(dims, idx, vals, A, B)
    rmse = C.c_double(0.0)
    mae = C.c_double(0.0)
    if positions is not None:
        positions = np.ascontiguousarray(positions, dtype=np.int64)
        p_ptr, cnt = positions.ctypes.data, int(positions.shape[0])
    else:
        p_ptr, cnt = None, 0
    rc = lib().fto_errors(N, dims_a.ctypes.data, nnz, _ptr_array(idx, C.c_int32), vals.ctypes.data,
                          J.ctypes.data, R, _ptr_array(A, C.c_float), _ptr_array(B, C.c_float),
                          p_ptr, cnt, C.addressof(rmse), C.addressof(mae))
    if rc:
        raise ValueError("fto_errors failed: %d" % rc)
    return rmse.value, mae.value


def rmse(dims, idx, vals, A, B) -> float:
    return errors(dims, idx, vals, A, B)[0]
