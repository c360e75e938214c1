"""Seeded synthetic inputs for the row-wise top-k workloads.

Shared by the CPU oracle's tests, the GPU parity tests and the benchmark.  It
holds none of the selection method's arithmetic: it only produces N x M fp32
matrices (host numpy arrays) whose shapes and value distributions follow the
paper's workloads (Section 3.1: normally distributed rows; Section 4.3:
MaxK-GNN hidden features with M = 256, k = 32, N = number of graph nodes;
Appendix B: N = 65536 rows of width up to 8192).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libworkloads.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the generator with g++ (host only)."""
    src = os.path.join(_HERE, "gen.cpp")
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(
            ["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c++17", src, "-o", _LIB_PATH]
        )
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.wl_fill_normal.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                                       ctypes.c_int32, ctypes.c_double, ctypes.c_double]
        lib.wl_fill_uniform.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                                        ctypes.c_double, ctypes.c_double]
        lib.wl_fill_laplace.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64]
        lib.wl_fill_normal_ties.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64,
                                            ctypes.c_double, ctypes.c_int32, ctypes.c_double, ctypes.c_double]
        for fn in (lib.wl_fill_normal, lib.wl_fill_uniform, lib.wl_fill_laplace, lib.wl_fill_normal_ties):
            fn.restype = ctypes.c_int
        _lib = lib
    return _lib


def _alloc(N: int, M: int) -> np.ndarray:
    return np.empty((N, M), dtype=np.float32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def normal(N: int, M: int, seed: int, row_scale: tuple[float, float] | None = None) -> np.ndarray:
    """i.i.d. N(0,1) entries; optionally each row multiplied by s_r ~ U(row_scale)."""
    out = _alloc(N, M)
    lo, hi = row_scale if row_scale else (1.0, 1.0)
    rc = _load().wl_fill_normal(_ptr(out), N, M, seed, 1 if row_scale else 0, lo, hi)
    assert rc == 0
    return out


def uniform(N: int, M: int, seed: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    out = _alloc(N, M)
    assert _load().wl_fill_uniform(_ptr(out), N, M, seed, lo, hi) == 0
    return out


def laplace(N: int, M: int, seed: int) -> np.ndarray:
    out = _alloc(N, M)
    assert _load().wl_fill_laplace(_ptr(out), N, M, seed) == 0
    return out


def normal_ties(N: int, M: int, seed: int, p: float = 0.05, levels: int = 16,
                level0: float = -3.0, step: float = 0.4) -> np.ndarray:
    """N(0,1) with a fraction p of entries snapped to `levels` shared values (forces ties)."""
    out = _alloc(N, M)
    assert _load().wl_fill_normal_ties(_ptr(out), N, M, seed, p, levels, level0, step) == 0
    return out


# A pool of awkward fp32 values: signed zeros, subnormals, adjacent floats,
# large magnitudes (still far below FLT_MAX/2 so that a sum of two cannot
# overflow), and a few ordinary ones.
def awkward_pool() -> np.ndarray:
    one = np.float32(1.0)
    vals = [
        0.0, -0.0, 1.0, -1.0, 0.5, -0.5, 2.0, -2.0, 3.0,
        float(np.nextafter(one, np.float32(2.0))), float(np.nextafter(one, np.float32(0.0))),
        float(np.nextafter(-one, np.float32(-2.0))), float(np.nextafter(-one, np.float32(0.0))),
        1e-45, -1e-45, 2.8e-45, 1e-40, -1e-40, 1.17549435e-38, -1.17549435e-38,
        1e30, -1e30, 9.999999e29, 1e-30, -1e-30, 123.456, -123.456,
    ]
    return np.array(vals, dtype=np.float32)


def from_pool(N: int, M: int, seed: int, pool_size: int | None = None) -> np.ndarray:
    """Rows drawn with replacement from a small random subset of `awkward_pool()`:
    heavy ties, including ties that straddle the k-th position."""
    rng = np.random.Generator(np.random.Philox(seed))
    pool = awkward_pool()
    out = np.empty((N, M), dtype=np.float32)
    for r in range(N):
        sz = pool_size if pool_size else int(rng.integers(1, 6))
        sub = rng.choice(pool, size=min(sz, pool.size), replace=False)
        out[r] = rng.choice(sub, size=M, replace=True)
    return out


def small_ints(N: int, M: int, seed: int, span: int = 16) -> np.ndarray:
    """Rows of small integers in [-span, span] as fp32: every midpoint the search forms
    is exactly representable, and ties are frequent."""
    rng = np.random.Generator(np.random.Philox(seed))
    return rng.integers(-span, span + 1, size=(N, M)).astype(np.float32)


# ----------------------------------------------------------------------------
# The five benchmark/parity configurations (shape, distribution, k, modes).
# ----------------------------------------------------------------------------
CONFIGS = {
    # small parity gate: finishes in well under a second on the CPU
    "c0_small": dict(N=4096, M=256, seed=0, dist="normal", ks=(32,), max_iters=(8,), idx="int32"),
    # MaxK-GNN hidden-layer shape (headline): N = 2^20, M = 256
    "c1_maxk": dict(N=1 << 20, M=256, seed=1, dist="normal_rowscale", ks=(16, 32, 64, 128),
                    max_iters=(4, 8, 16), idx="int32"),
    # width sweep, k = M/8
    "c2_w128": dict(N=1 << 20, M=128, seed=2, dist="uniform", ks=(16,), max_iters=(), idx="int32"),
    "c2_w512": dict(N=1 << 20, M=512, seed=2, dist="uniform", ks=(64,), max_iters=(), idx="int32"),
    "c2_w1024": dict(N=1 << 20, M=1024, seed=2, dist="uniform", ks=(128,), max_iters=(), idx="int32"),
    # large graph-feature matrix with forced ties, uint8 indices
    "c3_ties": dict(N=2_400_000, M=256, seed=3, dist="normal_ties", ks=(32,), max_iters=(8,), idx="uint8"),
    # wide rows
    "c4_wide": dict(N=65536, M=4096, seed=4, dist="laplace", ks=(64, 256), max_iters=(), idx="int32"),
    # the paper's widest row (Appendix B: M = 8192), 128 values per lane of one wavefront
    "x_wide8k": dict(N=32768, M=8192, seed=8, dist="laplace", ks=(256,), max_iters=(), idx="int32"),
    # beyond the paper's widest row: one workgroup per row
    "x_wide32k": dict(N=8192, M=32768, seed=5, dist="laplace", ks=(256, 2048), max_iters=(), idx="int32"),
    "x_wide64k": dict(N=4096, M=65536, seed=6, dist="laplace", ks=(512,), max_iters=(), idx="int32"),
    # rows that no longer fit a workgroup's registers: streamed from memory
    "x_stream256k": dict(N=1024, M=262144, seed=7, dist="laplace", ks=(512,), max_iters=(), idx="int32"),
}


def make(name: str, N: int | None = None) -> np.ndarray:
    """Input matrix of configuration `name`; `N` overrides the row count (the first N rows
    of the full matrix are reproduced exactly, because values depend only on (seed, index))."""
    cfg = CONFIGS[name]
    n = cfg["N"] if N is None else N
    M, seed, dist = cfg["M"], cfg["seed"], cfg["dist"]
    if dist == "normal":
        return normal(n, M, seed)
    if dist == "normal_rowscale":
        return normal(n, M, seed, row_scale=(0.5, 2.0))
    if dist == "uniform":
        return uniform(n, M, seed)
    if dist == "normal_ties":
        return normal_ties(n, M, seed)
    if dist == "laplace":
        return laplace(n, M, seed)
    raise KeyError(dist)


# ----------------------------------------------------------------------------
# 16-bit storage: the same matrices rounded to IEEE half or bfloat16 (round to
# nearest even), returned as their raw uint16 bit patterns.  Rounding N(0,1)
# rows to 8 or 11 significant bits makes ties frequent, which is wanted.
# ----------------------------------------------------------------------------
def to_f16_bits(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def to_bits16(x: np.ndarray, kind: str) -> np.ndarray:
    if kind == "f16":
        return to_f16_bits(x)
    if kind == "bf16":
        return to_bf16_bits(x)
    raise KeyError(kind)
