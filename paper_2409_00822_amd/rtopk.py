"""ctypes binding with the same names as the C ABI (include/rtopk.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librtopk.so")
_lib = None


class RTopKError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"rtopk status {status}: {text}")
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load librtopk.so (built by `python -m paper_2409_00822_amd.build` or __graft_entry__.build()).
    Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} not found: build it with `python -m paper_2409_00822_amd.build`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.rtopk_rowwise.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
        lib.rtopk_rowwise_u8.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
        lib.rtopk_rowwise_smallest.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
        lib.rtopk_rowwise_exact_smallest.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        lib.rtopk_rowwise_exact.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        lib.rtopk_rowwise_exact_u8.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        lib.rtopk_rowwise_eps.argtypes = [vp, i64, i32, i32, ctypes.c_float, vp, vp, vp, vp]
        for name in ("rtopk_rowwise_f16", "rtopk_rowwise_bf16"):
            getattr(lib, name).argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
            getattr(lib, name).restype = ctypes.c_int
        for name in ("rtopk_rowwise_exact_f16", "rtopk_rowwise_exact_bf16"):
            getattr(lib, name).argtypes = [vp, i64, i32, i32, vp, vp, vp]
            getattr(lib, name).restype = ctypes.c_int
        lib.rtopk_maxk_dense.argtypes = [vp, i64, i32, i32, i32, vp, vp]
        lib.rtopk_maxk_dense.restype = ctypes.c_int
        for fn in (lib.rtopk_rowwise, lib.rtopk_rowwise_u8, lib.rtopk_rowwise_exact, lib.rtopk_rowwise_exact_u8,
                   lib.rtopk_rowwise_eps, lib.rtopk_rowwise_smallest, lib.rtopk_rowwise_exact_smallest,
                   lib.rtopk_version, lib.rtopk_max_m):
            fn.restype = ctypes.c_int
        for name in ("rtopk_maxk_backward", "rtopk_maxk_backward_u8", "rtopk_maxk_backward_gather",
                     "rtopk_maxk_backward_gather_u8"):
            getattr(lib, name).argtypes = [vp, vp, i64, i32, i32, vp, vp]
            getattr(lib, name).restype = ctypes.c_int
        lib.rtopk_status_string.argtypes = [ctypes.c_int]
        lib.rtopk_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def rtopk_status_string(status: int) -> str:
    return load_library().rtopk_status_string(int(status)).decode()


def rtopk_version() -> int:
    return int(load_library().rtopk_version())


def rtopk_max_m() -> int:
    return int(load_library().rtopk_max_m())


def _check(status: int) -> None:
    if status != 0:
        raise RTopKError(status, rtopk_status_string(status))


def _prepare(x, k: int, out_vals, out_idx, idx_dtype, val_dtype=None):
    import torch

    val_dtype = torch.float32 if val_dtype is None else val_dtype
    if not (x.is_cuda and x.dtype == val_dtype and x.dim() == 2 and x.is_contiguous()):
        raise ValueError(f"x must be a contiguous 2-D {val_dtype} tensor on the GPU")
    N, M = x.shape
    if out_vals is None:
        out_vals = torch.empty((N, k), dtype=val_dtype, device=x.device)
    if out_idx is None:
        out_idx = torch.empty((N, k), dtype=idx_dtype, device=x.device)
    for t, dt in ((out_vals, val_dtype), (out_idx, idx_dtype)):
        if not (t.is_cuda and t.dtype == dt and t.is_contiguous() and tuple(t.shape) == (N, k)):
            raise ValueError("outputs must be contiguous [N, k] GPU tensors of the right dtype")
    stream = torch.cuda.current_stream(x.device).cuda_stream
    return N, M, out_vals, out_idx, stream


def rtopk_rowwise(x, k: int, max_iter: int, out_vals=None, out_idx=None):
    """Algorithm 2 (early stopping).  Returns (values [N,k] f32, columns [N,k] i32)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.int32)
    _check(load_library().rtopk_rowwise(x.data_ptr(), N, M, k, max_iter, out_vals.data_ptr(), out_idx.data_ptr(),
                                        stream))
    return out_vals, out_idx


def rtopk_rowwise_exact(x, k: int, out_vals=None, out_idx=None):
    """Algorithm 1 at epsilon = 0 (exact top-k).  Returns (values [N,k] f32, columns [N,k] i32)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.int32)
    _check(load_library().rtopk_rowwise_exact(x.data_ptr(), N, M, k, out_vals.data_ptr(), out_idx.data_ptr(), stream))
    return out_vals, out_idx


def rtopk_rowwise_u8(x, k: int, max_iter: int, out_vals=None, out_idx=None):
    """Algorithm 2 with uint8 columns (M <= 256)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.uint8)
    _check(load_library().rtopk_rowwise_u8(x.data_ptr(), N, M, k, max_iter, out_vals.data_ptr(), out_idx.data_ptr(),
                                           stream))
    return out_vals, out_idx


def rtopk_rowwise_exact_u8(x, k: int, out_vals=None, out_idx=None):
    """Exact top-k with uint8 columns (M <= 256)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.uint8)
    _check(load_library().rtopk_rowwise_exact_u8(x.data_ptr(), N, M, k, out_vals.data_ptr(), out_idx.data_ptr(),
                                                 stream))
    return out_vals, out_idx


def rtopk_rowwise_eps(x, k: int, eps_rel: float, out_vals=None, out_idx=None, out_iters=None, want_iters: bool = False):
    """Algorithm 1 with precision epsilon = eps_rel * |max(row)|.  Returns (values, columns) or, when
    `want_iters` is set or `out_iters` is given, (values, columns, exit iterations [N] i32)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.int32)
    if out_iters is None and want_iters:
        out_iters = torch.empty((N,), dtype=torch.int32, device=x.device)
    if out_iters is not None and not (out_iters.is_cuda and out_iters.dtype == torch.int32
                                      and out_iters.is_contiguous() and tuple(out_iters.shape) == (N,)):
        raise ValueError("out_iters must be a contiguous [N] int32 GPU tensor")
    _check(load_library().rtopk_rowwise_eps(x.data_ptr(), N, M, k, float(eps_rel), out_vals.data_ptr(),
                                            out_idx.data_ptr(), out_iters.data_ptr() if out_iters is not None else None,
                                            stream))
    return (out_vals, out_idx, out_iters) if out_iters is not None else (out_vals, out_idx)


def rtopk_rowwise_smallest(x, k: int, max_iter: int, out_vals=None, out_idx=None):
    """Algorithm 2 for the k smallest values per row.  Returns (values [N,k] f32, columns [N,k] i32)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.int32)
    _check(load_library().rtopk_rowwise_smallest(x.data_ptr(), N, M, k, max_iter, out_vals.data_ptr(),
                                                 out_idx.data_ptr(), stream))
    return out_vals, out_idx


def rtopk_rowwise_exact_smallest(x, k: int, out_vals=None, out_idx=None):
    """Exact k smallest values per row.  Returns (values [N,k] f32, columns [N,k] i32)."""
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.int32)
    _check(load_library().rtopk_rowwise_exact_smallest(x.data_ptr(), N, M, k, out_vals.data_ptr(), out_idx.data_ptr(),
                                                       stream))
    return out_vals, out_idx


def _rowwise_16(name: str, val_dtype, x, k, max_iter, out_vals, out_idx):
    import torch

    N, M, out_vals, out_idx, stream = _prepare(x, k, out_vals, out_idx, torch.int32, val_dtype)
    fn = getattr(load_library(), name)
    if max_iter is None:
        _check(fn(x.data_ptr(), N, M, k, out_vals.data_ptr(), out_idx.data_ptr(), stream))
    else:
        _check(fn(x.data_ptr(), N, M, k, max_iter, out_vals.data_ptr(), out_idx.data_ptr(), stream))
    return out_vals, out_idx


def rtopk_rowwise_f16(x, k: int, max_iter: int, out_vals=None, out_idx=None):
    """Algorithm 2 on float16 rows (fp32 arithmetic on the widened row).  Returns (values f16, columns i32)."""
    import torch

    return _rowwise_16("rtopk_rowwise_f16", torch.float16, x, k, max_iter, out_vals, out_idx)


def rtopk_rowwise_exact_f16(x, k: int, out_vals=None, out_idx=None):
    """Exact top-k of float16 rows.  Returns (values f16, columns i32)."""
    import torch

    return _rowwise_16("rtopk_rowwise_exact_f16", torch.float16, x, k, None, out_vals, out_idx)


def rtopk_rowwise_bf16(x, k: int, max_iter: int, out_vals=None, out_idx=None):
    """Algorithm 2 on bfloat16 rows (fp32 arithmetic on the widened row).  Returns (values bf16, columns i32)."""
    import torch

    return _rowwise_16("rtopk_rowwise_bf16", torch.bfloat16, x, k, max_iter, out_vals, out_idx)


def rtopk_rowwise_exact_bf16(x, k: int, out_vals=None, out_idx=None):
    """Exact top-k of bfloat16 rows.  Returns (values bf16, columns i32)."""
    import torch

    return _rowwise_16("rtopk_rowwise_exact_bf16", torch.bfloat16, x, k, None, out_vals, out_idx)


def rtopk_maxk_dense(x, k: int, max_iter: int = -1, out=None):
    """MaxK non-linearity, dense form: the k selected values of each row in place, zero elsewhere.
    max_iter < 0: exact selection; max_iter >= 0: Algorithm 2 with that many steps.  Returns out [N,M] f32."""
    import torch

    if not (x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.is_contiguous()):
        raise ValueError("x must be a contiguous 2-D float32 tensor on the GPU")
    N, M = x.shape
    if out is None:
        out = torch.empty_like(x)
    if not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == (N, M)):
        raise ValueError("out must be a contiguous [N, M] float32 GPU tensor")
    stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(load_library().rtopk_maxk_dense(x.data_ptr(), N, M, k, max_iter, out.data_ptr(), stream))
    return out


def _backward_args(idx, M: int):
    import torch

    if not (idx.is_cuda and idx.dim() == 2 and idx.is_contiguous() and idx.dtype in (torch.int32, torch.uint8)):
        raise ValueError("idx must be a contiguous [N, k] int32 or uint8 GPU tensor")
    if idx.dtype == torch.uint8 and M > 256:
        raise ValueError("uint8 columns need M <= 256")
    return idx.dtype == torch.uint8, torch.cuda.current_stream(idx.device).cuda_stream


def rtopk_maxk_backward(grad_vals, idx, M: int, grad_in=None):
    """Backward of the MaxK non-linearity, scatter form: gradients of the k kept values [N, k] and the
    saved columns [N, k] (int32 or uint8) -> gradient of the dense row [N, M], zero elsewhere."""
    import torch

    u8, stream = _backward_args(idx, M)
    N, k = idx.shape
    if not (grad_vals.is_cuda and grad_vals.dtype == torch.float32 and grad_vals.is_contiguous()
            and tuple(grad_vals.shape) == (N, k)):
        raise ValueError("grad_vals must be a contiguous [N, k] float32 GPU tensor")
    if grad_in is None:
        grad_in = torch.empty((N, M), dtype=torch.float32, device=idx.device)
    if not (grad_in.is_cuda and grad_in.dtype == torch.float32 and grad_in.is_contiguous()
            and tuple(grad_in.shape) == (N, M)):
        raise ValueError("grad_in must be a contiguous [N, M] float32 GPU tensor")
    fn = load_library().rtopk_maxk_backward_u8 if u8 else load_library().rtopk_maxk_backward
    _check(fn(grad_vals.data_ptr(), idx.data_ptr(), N, M, k, grad_in.data_ptr(), stream))
    return grad_in


def rtopk_maxk_backward_gather(grad_out, idx, grad_vals=None):
    """Backward of the MaxK non-linearity, gather form: dense gradient rows [N, M] and the saved columns
    [N, k] (int32 or uint8) -> the gradient entries at those columns [N, k]."""
    import torch

    if not (grad_out.is_cuda and grad_out.dtype == torch.float32 and grad_out.dim() == 2 and grad_out.is_contiguous()):
        raise ValueError("grad_out must be a contiguous [N, M] float32 GPU tensor")
    N, M = grad_out.shape
    u8, stream = _backward_args(idx, M)
    if idx.shape[0] != N:
        raise ValueError("idx must have one row per row of grad_out")
    k = idx.shape[1]
    if grad_vals is None:
        grad_vals = torch.empty((N, k), dtype=torch.float32, device=idx.device)
    if not (grad_vals.is_cuda and grad_vals.dtype == torch.float32 and grad_vals.is_contiguous()
            and tuple(grad_vals.shape) == (N, k)):
        raise ValueError("grad_vals must be a contiguous [N, k] float32 GPU tensor")
    fn = load_library().rtopk_maxk_backward_gather_u8 if u8 else load_library().rtopk_maxk_backward_gather
    _check(fn(grad_out.data_ptr(), idx.data_ptr(), N, M, k, grad_vals.data_ptr(), stream))
    return grad_vals
