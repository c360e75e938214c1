"""ctypes wrapper around the CPU oracle (oracle/rtopk_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module.
All arrays are host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_rtopk.so")
_lib = None


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "rtopk_oracle.cpp")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(
            ["g++", "-O2", "-std=c++17", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
             "-shared", "-fPIC", src, "-o", _LIB_PATH]
        )
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        f32p = ctypes.POINTER(ctypes.c_float)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_topk_exact.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, f32p, i32p]
        lib.oracle_topk_exact.restype = ctypes.c_int
        lib.oracle_topk_earlystop_ex.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                 ctypes.c_int32, ctypes.c_int32, f32p, i32p, i32p]
        lib.oracle_topk_earlystop_ex.restype = ctypes.c_int
        lib.oracle_topk_exact_smallest.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, f32p, i32p]
        lib.oracle_topk_exact_smallest.restype = ctypes.c_int
        lib.oracle_topk_earlystop_smallest.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                       ctypes.c_int32, f32p, i32p]
        lib.oracle_topk_earlystop_smallest.restype = ctypes.c_int
        lib.oracle_alg1.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                    ctypes.c_int32, f32p, i32p, i32p]
        lib.oracle_alg1.restype = ctypes.c_int
        lib.oracle_maxk_backward.argtypes = [f32p, i32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, f32p]
        lib.oracle_maxk_backward.restype = ctypes.c_int
        lib.oracle_maxk_backward_gather.argtypes = [f32p, i32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, f32p]
        lib.oracle_maxk_backward_gather.restype = ctypes.c_int
        lib.oracle_mean_overlap.argtypes = [i32p, i32p, ctypes.c_int64, ctypes.c_int32]
        lib.oracle_mean_overlap.restype = ctypes.c_double
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _f32(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _check_in(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim != 2:
        raise ValueError("input must be 2-D [N, M]")
    return x


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def topk_exact(x: np.ndarray, k: int):
    """Plain-definition top-k per row.  Returns (vals [N,k] f32, idx [N,k] i32), columns ascending."""
    x = _check_in(x)
    N, M = x.shape
    vals = np.empty((N, k), dtype=np.float32)
    idx = np.empty((N, k), dtype=np.int32)
    rc = _load().oracle_topk_exact(_f32(x), N, M, k, _f32(vals), _i32(idx))
    if rc != 0:
        raise ValueError("oracle_topk_exact: bad arguments")
    return vals, idx


def topk_earlystop(x: np.ndarray, k: int, max_iter: int, stop_on_equal: bool = False, return_hit_iter: bool = False):
    """Algorithm 2, literal (stop_on_equal=False).  stop_on_equal=True is the diagnostic variant."""
    x = _check_in(x)
    N, M = x.shape
    vals = np.empty((N, k), dtype=np.float32)
    idx = np.empty((N, k), dtype=np.int32)
    hit = np.empty((N,), dtype=np.int32) if return_hit_iter else None
    rc = _load().oracle_topk_earlystop_ex(_f32(x), N, M, k, max_iter, 1 if stop_on_equal else 0,
                                          _f32(vals), _i32(idx), _i32(hit) if hit is not None else None)
    if rc != 0:
        raise ValueError("oracle_topk_earlystop: bad arguments")
    return (vals, idx, hit) if return_hit_iter else (vals, idx)


def topk_exact_smallest(x: np.ndarray, k: int):
    """Plain-definition k smallest per row (value ascending, then column ascending), columns ascending."""
    x = _check_in(x)
    N, M = x.shape
    vals = np.empty((N, k), dtype=np.float32)
    idx = np.empty((N, k), dtype=np.int32)
    if _load().oracle_topk_exact_smallest(_f32(x), N, M, k, _f32(vals), _i32(idx)) != 0:
        raise ValueError("oracle_topk_exact_smallest: bad arguments")
    return vals, idx


def topk_earlystop_smallest(x: np.ndarray, k: int, max_iter: int):
    """Algorithm 2 on the negated row, original values returned."""
    x = _check_in(x)
    N, M = x.shape
    vals = np.empty((N, k), dtype=np.float32)
    idx = np.empty((N, k), dtype=np.int32)
    if _load().oracle_topk_earlystop_smallest(_f32(x), N, M, k, max_iter, _f32(vals), _i32(idx)) != 0:
        raise ValueError("oracle_topk_earlystop_smallest: bad arguments")
    return vals, idx


def alg1(x: np.ndarray, k: int, eps_rel: float = 0.0, collect: int = 1, want_select: bool = True,
         want_iters: bool = True):
    """Algorithm 1.  Returns (vals, idx, iters); entries not asked for are None."""
    x = _check_in(x)
    N, M = x.shape
    vals = np.empty((N, k), dtype=np.float32) if want_select else None
    idx = np.empty((N, k), dtype=np.int32) if want_select else None
    iters = np.empty((N,), dtype=np.int32) if want_iters else None
    rc = _load().oracle_alg1(_f32(x), N, M, k, eps_rel, collect,
                             _f32(vals) if want_select else None, _i32(idx) if want_select else None,
                             _i32(iters) if want_iters else None)
    if rc != 0:
        raise ValueError("oracle_alg1: bad arguments")
    return vals, idx, iters


def mean_overlap(idx_a: np.ndarray, idx_b: np.ndarray) -> float:
    """Mean over rows of |A ∩ B| / k for two [N,k] ascending index arrays (Table 2's Hit)."""
    a = np.ascontiguousarray(idx_a, dtype=np.int32)
    b = np.ascontiguousarray(idx_b, dtype=np.int32)
    assert a.shape == b.shape and a.ndim == 2
    return float(_load().oracle_mean_overlap(_i32(a), _i32(b), a.shape[0], a.shape[1]))


# ---------------------------------------------------------------------------------------------
# 16-bit storage (IEEE half "f16", bfloat16 "bf16").  The paper works in fp32 throughout; for rows
# stored in 16 bits the selection is DEFINED as the fp32 method applied to the exactly widened row
# (every half and bfloat16 value is an fp32 value), and the values written out are the row's own
# 16-bit patterns at the chosen columns.  Inputs and outputs here are raw uint16 bit patterns.
# ---------------------------------------------------------------------------------------------
def widen16(bits16: np.ndarray, kind: str) -> np.ndarray:
    """Exact conversion of uint16 bit patterns to fp32."""
    b = np.ascontiguousarray(bits16, dtype=np.uint16)
    if kind == "f16":
        return b.view(np.float16).astype(np.float32)
    if kind == "bf16":
        return (b.astype(np.uint32) << 16).view(np.float32)
    raise KeyError(kind)


def _gather16(bits16: np.ndarray, idx: np.ndarray) -> np.ndarray:
    return np.take_along_axis(np.ascontiguousarray(bits16, dtype=np.uint16), idx.astype(np.int64), axis=1)


def topk_exact_16(bits16: np.ndarray, kind: str, k: int):
    """Plain-definition top-k of rows stored in 16 bits.  Returns (value bits [N,k] u16, idx [N,k] i32)."""
    _, idx = topk_exact(widen16(bits16, kind), k)
    return _gather16(bits16, idx), idx


def topk_earlystop_16(bits16: np.ndarray, kind: str, k: int, max_iter: int):
    """Algorithm 2 in fp32 on the widened row.  Returns (value bits [N,k] u16, idx [N,k] i32)."""
    _, idx = topk_earlystop(widen16(bits16, kind), k, max_iter)
    return _gather16(bits16, idx), idx


# ---------------------------------------------------------------------------------------------
# Dense form of the selection (the MaxK non-linearity, Section 1 / Fig. 1): the selected values in
# place, +0 everywhere else.  Written out from the column lists the functions above return.
# ---------------------------------------------------------------------------------------------
def maxk_dense(x: np.ndarray, k: int, max_iter: int = -1) -> np.ndarray:
    """max_iter < 0: exact top-k; otherwise Algorithm 2 with max_iter steps.  Returns [N, M] fp32."""
    x = _check_in(x)
    _, idx = topk_exact(x, k) if max_iter < 0 else topk_earlystop(x, k, max_iter)
    out = np.zeros_like(x)
    rows = np.arange(x.shape[0])[:, None]
    out[rows, idx] = x[rows, idx]
    return out


# ---------------------------------------------------------------------------------------------
# Backward edge of the MaxK non-linearity (Section 1 / Fig. 1, Section 4.3): the derivative of "keep
# the k selected columns, zero the rest" with respect to the row is the 0/1 selection mask.
# ---------------------------------------------------------------------------------------------
def maxk_backward(grad_vals: np.ndarray, idx: np.ndarray, M: int) -> np.ndarray:
    """Scatter form: gradients of the k kept values [N, k] -> gradient of the dense row [N, M]
    (zero except at the saved columns idx [N, k])."""
    g = np.ascontiguousarray(grad_vals, dtype=np.float32)
    i = np.ascontiguousarray(idx, dtype=np.int32)
    assert g.ndim == 2 and g.shape == i.shape
    N, k = g.shape
    out = np.empty((N, M), dtype=np.float32)
    if _load().oracle_maxk_backward(_f32(g), _i32(i), N, M, k, _f32(out)) != 0:
        raise ValueError("oracle_maxk_backward: bad arguments")
    return out


def maxk_backward_gather(grad_out: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Gather form: dense gradient rows [N, M] -> their entries at the saved columns idx [N, k]."""
    g = _check_in(grad_out)
    i = np.ascontiguousarray(idx, dtype=np.int32)
    N, M = g.shape
    assert i.ndim == 2 and i.shape[0] == N
    k = i.shape[1]
    out = np.empty((N, k), dtype=np.float32)
    if _load().oracle_maxk_backward_gather(_f32(g), _i32(i), N, M, k, _f32(out)) != 0:
        raise ValueError("oracle_maxk_backward_gather: bad arguments")
    return out
