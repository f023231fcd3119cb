"""Thin Python binding of the C-ABI library ``libna2d.so`` (see ``include/na2d.h``).

Argument marshalling only: every function takes torch tensors that already live on the GPU
(PyTorch is used for device memory and streams, nothing else), checks dtype / shape /
contiguity, passes raw device pointers and the current HIP stream through ctypes and raises
``Na2dError`` on a non-zero status.  There is no fallback: if the library has not been built
(``python -m paper_2204_07143_amd.build``) loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libna2d.so")

DTYPE_CODES = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}
WS_QK_BWD_RPB, WS_BWD, WS_FUSED_BWD = 0, 1, 2

EXPORTS = (
    "na2d_qk_rpb", "na2d_softmax", "na2d_av", "na2d_fused_fwd", "na2d_av_bwd_p", "na2d_av_bwd_v",
    "na2d_softmax_bwd", "na2d_qk_bwd_q", "na2d_qk_bwd_k", "na2d_qk_bwd_rpb", "na2d_qk_bwd_rpb_noalloc", "na2d_bwd", "na2d_fused_bwd",
    "na2d_fused_bwd_is_fused",
    "na2d_workspace_bytes", "na2d_debug_indices", "na2d_host_axis_tables", "na2d_validate_problem",
    "na2d_strerror", "na2d_version",
)


EXPORTS_1D = (
    "na1d_validate_problem", "na1d_qk_rpb", "na1d_softmax", "na1d_av", "na1d_fused_fwd", "na1d_av_bwd_p", "na1d_av_bwd_v",
    "na1d_softmax_bwd", "na1d_qk_bwd_q", "na1d_qk_bwd_k", "na1d_qk_bwd_rpb", "na1d_workspace_bytes",
    "na1d_fused_bwd", "na1d_fused_bwd_workspace_bytes",
)


class Na2dError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"na2d status {status}: {message}")
        self.status = status


class Na2dProblem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "heads", "H", "W", "D", "k", "dtype")]


class Na1dProblem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "heads", "L", "D", "k", "dtype")]


_lib = None


def load(path: str | None = None) -> ctypes.CDLL:
    """Load libna2d.so (once). Raises if it has not been built.  ``path`` (first call only) names another build of
    the same library, e.g. the benchmark's memory-only measurement build."""
    global _lib
    if _lib is None:
        lib_path = LIB_PATH if path is None else path
        if not os.path.exists(lib_path):
            raise FileNotFoundError(
                f"{lib_path} is missing: build it with `python -m paper_2204_07143_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        lib = ctypes.CDLL(lib_path)
        vp, pp, f = ctypes.c_void_p, ctypes.POINTER(Na2dProblem), ctypes.c_float
        sigs = {
            "na2d_qk_rpb": [pp, vp, vp, vp, f, vp, vp],
            "na2d_softmax": [pp, vp, vp, vp],
            "na2d_av": [pp, vp, vp, vp, vp],
            "na2d_fused_fwd": [pp, vp, vp, vp, vp, f, vp, vp, vp],
            "na2d_av_bwd_p": [pp, vp, vp, vp, vp],
            "na2d_av_bwd_v": [pp, vp, vp, vp, vp],
            "na2d_softmax_bwd": [pp, vp, vp, vp, vp],
            "na2d_qk_bwd_q": [pp, vp, vp, f, vp, vp],
            "na2d_qk_bwd_k": [pp, vp, vp, f, vp, vp],
            "na2d_qk_bwd_rpb": [pp, vp, vp, vp, ctypes.c_size_t, vp],
            "na2d_qk_bwd_rpb_noalloc": [pp, vp, vp, vp],
            "na2d_bwd": [pp, vp, vp, vp, vp, vp, f, vp, vp, vp, vp, vp, ctypes.c_size_t, vp],
            "na2d_fused_bwd": [pp, vp, vp, vp, vp, f, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp],
            "na2d_debug_indices": [pp, vp, vp, vp],
            "na2d_host_axis_tables": [ctypes.c_int32, ctypes.c_int32, vp, vp, vp],
            "na2d_validate_problem": [pp],
            "na2d_fused_bwd_is_fused": [pp],
        }
        for name, argtypes in sigs.items():
            fn = getattr(lib, name)
            fn.argtypes = argtypes
            fn.restype = ctypes.c_int
        p1 = ctypes.POINTER(Na1dProblem)
        sigs_1d = {
            "na1d_validate_problem": [p1],
            "na1d_qk_rpb": [p1, vp, vp, vp, f, vp, vp],
            "na1d_softmax": [p1, vp, vp, vp],
            "na1d_av": [p1, vp, vp, vp, vp],
            "na1d_fused_fwd": [p1, vp, vp, vp, vp, f, vp, vp, vp],
            "na1d_av_bwd_p": [p1, vp, vp, vp, vp],
            "na1d_av_bwd_v": [p1, vp, vp, vp, vp],
            "na1d_softmax_bwd": [p1, vp, vp, vp, vp],
            "na1d_qk_bwd_q": [p1, vp, vp, f, vp, vp],
            "na1d_qk_bwd_k": [p1, vp, vp, f, vp, vp],
            "na1d_qk_bwd_rpb": [p1, vp, vp, vp, ctypes.c_size_t, vp],
            "na1d_fused_bwd": [p1, vp, vp, vp, vp, f, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp],
        }
        for name, argtypes in sigs_1d.items():
            fn = getattr(lib, name)
            fn.argtypes = argtypes
            fn.restype = ctypes.c_int
        lib.na1d_workspace_bytes.argtypes = [p1]
        lib.na1d_workspace_bytes.restype = ctypes.c_size_t
        lib.na1d_fused_bwd_workspace_bytes.argtypes = [p1]
        lib.na1d_fused_bwd_workspace_bytes.restype = ctypes.c_size_t
        lib.na2d_workspace_bytes.argtypes = [pp, ctypes.c_int]
        lib.na2d_workspace_bytes.restype = ctypes.c_size_t
        lib.na2d_strerror.argtypes = [ctypes.c_int]
        lib.na2d_strerror.restype = ctypes.c_char_p
        lib.na2d_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load().na2d_strerror(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        raise Na2dError(status, strerror(status))


def problem(B: int, heads: int, H: int, W: int, D: int, k: int, dtype) -> Na2dProblem:
    code = DTYPE_CODES[dtype] if dtype in DTYPE_CODES else int(dtype)
    return Na2dProblem(B, heads, H, W, D, k, code)


def _problem_of(x: torch.Tensor, k: int) -> Na2dProblem:
    if x.dim() != 5:
        raise ValueError("expected a [B, heads, H, W, D] tensor")
    B, heads, H, W, D = x.shape
    return problem(B, heads, H, W, D, k, x.dtype)


def _ptr(t, dtype=None, shape=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("na2d takes GPU tensors only")
    if not t.is_contiguous():
        raise ValueError("na2d takes contiguous tensors only")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _attn_shape(x: torch.Tensor, k: int):
    return (*x.shape[:4], k * k)


def _rpb_shape(x: torch.Tensor, k: int):
    return (x.shape[1], 2 * k - 1, 2 * k - 1)


# ---- the C ABI, one Python function per export, same names ---------------------------------

def na2d_qk_rpb(q, k_, rpb, scale: float, kernel: int, logits):
    p = _problem_of(q, kernel)
    _check(load().na2d_qk_rpb(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape),
                              _ptr(rpb, q.dtype, _rpb_shape(q, kernel)) if rpb is not None else None,
                              scale, _ptr(logits, q.dtype, _attn_shape(q, kernel)), _stream()))
    return logits


def na2d_softmax(logits, kernel: int, like, out):
    p = _problem_of(like, kernel)
    _check(load().na2d_softmax(ctypes.byref(p), _ptr(logits, like.dtype, _attn_shape(like, kernel)),
                               _ptr(out, like.dtype, _attn_shape(like, kernel)), _stream()))
    return out


def na2d_av(attn, v, kernel: int, out):
    p = _problem_of(v, kernel)
    _check(load().na2d_av(ctypes.byref(p), _ptr(attn, v.dtype, _attn_shape(v, kernel)), _ptr(v),
                          _ptr(out, v.dtype, v.shape), _stream()))
    return out


def na2d_fused_fwd(q, k_, v, rpb, scale: float, kernel: int, out, lse=None):
    p = _problem_of(q, kernel)
    _check(load().na2d_fused_fwd(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape), _ptr(v, q.dtype, q.shape),
                                 _ptr(rpb, q.dtype, _rpb_shape(q, kernel)) if rpb is not None else None, scale,
                                 _ptr(out, q.dtype, q.shape),
                                 _ptr(lse, torch.float32, q.shape[:4]) if lse is not None else None, _stream()))
    return out


def na2d_av_bwd_p(dout, v, kernel: int, dp):
    p = _problem_of(v, kernel)
    _check(load().na2d_av_bwd_p(ctypes.byref(p), _ptr(dout, v.dtype, v.shape), _ptr(v),
                                _ptr(dp, v.dtype, _attn_shape(v, kernel)), _stream()))
    return dp


def na2d_av_bwd_v(attn, dout, kernel: int, dv):
    p = _problem_of(dout, kernel)
    _check(load().na2d_av_bwd_v(ctypes.byref(p), _ptr(attn, dout.dtype, _attn_shape(dout, kernel)), _ptr(dout),
                                _ptr(dv, dout.dtype, dout.shape), _stream()))
    return dv


def na2d_softmax_bwd(attn, dp, kernel: int, like, ds):
    p = _problem_of(like, kernel)
    shape = _attn_shape(like, kernel)
    _check(load().na2d_softmax_bwd(ctypes.byref(p), _ptr(attn, like.dtype, shape), _ptr(dp, like.dtype, shape),
                                   _ptr(ds, like.dtype, shape), _stream()))
    return ds


def na2d_qk_bwd_q(ds, k_, scale: float, kernel: int, dq):
    p = _problem_of(k_, kernel)
    _check(load().na2d_qk_bwd_q(ctypes.byref(p), _ptr(ds, k_.dtype, _attn_shape(k_, kernel)), _ptr(k_), scale,
                                _ptr(dq, k_.dtype, k_.shape), _stream()))
    return dq


def na2d_qk_bwd_k(ds, q, scale: float, kernel: int, dk):
    p = _problem_of(q, kernel)
    _check(load().na2d_qk_bwd_k(ctypes.byref(p), _ptr(ds, q.dtype, _attn_shape(q, kernel)), _ptr(q), scale,
                                _ptr(dk, q.dtype, q.shape), _stream()))
    return dk


def na2d_workspace_bytes(p: Na2dProblem, kind: int) -> int:
    return int(load().na2d_workspace_bytes(ctypes.byref(p), int(kind)))


def na2d_qk_bwd_rpb(ds, kernel: int, like, d_rpb, workspace):
    p = _problem_of(like, kernel)
    _check(load().na2d_qk_bwd_rpb(ctypes.byref(p), _ptr(ds, like.dtype, _attn_shape(like, kernel)),
                                  _ptr(d_rpb, torch.float32, _rpb_shape(like, kernel)), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()))
    return d_rpb


NOALLOC_SCRATCH_BYTES = 4 << 20   # NA2D_NOALLOC_SCRATCH_BYTES of na2d.h


def na2d_qk_bwd_rpb_noalloc(ds, kernel: int, like, d_rpb):
    """na2d_qk_bwd_rpb with the partials in the library's own device array: no workspace argument."""
    p = _problem_of(like, kernel)
    _check(load().na2d_qk_bwd_rpb_noalloc(ctypes.byref(p), _ptr(ds, like.dtype, _attn_shape(like, kernel)),
                                          _ptr(d_rpb, torch.float32, _rpb_shape(like, kernel)), _stream()))
    return d_rpb


def na2d_bwd(q, k_, v, attn, dout, scale: float, kernel: int, dq, dk, dv, d_rpb, workspace):
    p = _problem_of(q, kernel)
    _check(load().na2d_bwd(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape), _ptr(v, q.dtype, q.shape),
                           _ptr(attn, q.dtype, _attn_shape(q, kernel)), _ptr(dout, q.dtype, q.shape), scale,
                           _ptr(dq, q.dtype, q.shape), _ptr(dk, q.dtype, q.shape), _ptr(dv, q.dtype, q.shape),
                           _ptr(d_rpb, torch.float32, _rpb_shape(q, kernel)) if d_rpb is not None else None,
                           _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
    return dq, dk, dv, d_rpb


def na2d_fused_bwd(q, k_, v, rpb, scale: float, lse, dout, kernel: int, dq, dk, dv, d_rpb, workspace):
    p = _problem_of(q, kernel)
    _check(load().na2d_fused_bwd(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape), _ptr(v, q.dtype, q.shape),
                                 _ptr(rpb, q.dtype, _rpb_shape(q, kernel)) if rpb is not None else None, scale,
                                 _ptr(lse, torch.float32, q.shape[:4]), _ptr(dout, q.dtype, q.shape),
                                 _ptr(dq, q.dtype, q.shape), _ptr(dk, q.dtype, q.shape), _ptr(dv, q.dtype, q.shape),
                                 _ptr(d_rpb, torch.float32, _rpb_shape(q, kernel)) if d_rpb is not None else None,
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
    return dq, dk, dv, d_rpb


def na2d_fused_bwd_is_fused(p: Na2dProblem) -> int:
    return int(load().na2d_fused_bwd_is_fused(ctypes.byref(p)))


def na2d_debug_indices(H: int, W: int, kernel: int, key_index, rpb_index):
    p = problem(1, 1, H, W, 32, kernel, torch.float32)
    shape = (H, W, kernel * kernel)
    _check(load().na2d_debug_indices(ctypes.byref(p),
                                     _ptr(key_index, torch.int32, shape) if key_index is not None else None,
                                     _ptr(rpb_index, torch.int32, shape) if rpb_index is not None else None,
                                     _stream()))
    return key_index, rpb_index


def na2d_host_axis_tables(L: int, kernel: int):
    """(start, qs, qe) int32 numpy arrays of length L, computed on the host by the library."""
    import numpy as np
    start, qs, qe = (np.empty(L, dtype=np.int32) for _ in range(3))
    _check(load().na2d_host_axis_tables(L, kernel, start.ctypes.data, qs.ctypes.data, qe.ctypes.data))
    return start, qs, qe


def na2d_validate_problem(p: Na2dProblem) -> int:
    return int(load().na2d_validate_problem(ctypes.byref(p)))


def na2d_version() -> int:
    return int(load().na2d_version())


# ---- 1D entry points (include/na1d.h): tensors are [B, heads, L, D], [B, heads, L, k], [heads, 2k-1] ----------

def problem_1d(B: int, heads: int, L: int, D: int, k: int, dtype) -> Na1dProblem:
    code = DTYPE_CODES[dtype] if dtype in DTYPE_CODES else int(dtype)
    return Na1dProblem(B, heads, L, D, k, code)


def _p1(x: torch.Tensor, k: int) -> Na1dProblem:
    if x.dim() != 4:
        raise ValueError("expected a [B, heads, L, D] tensor")
    B, heads, L, D = x.shape
    return problem_1d(B, heads, L, D, k, x.dtype)


def _attn1(x, k):
    return (*x.shape[:3], k)


def _rpb1(x, k):
    return (x.shape[1], 2 * k - 1)


def na1d_validate_problem(p: Na1dProblem) -> int:
    return int(load().na1d_validate_problem(ctypes.byref(p)))


def na1d_qk_rpb(q, k_, rpb, scale: float, kernel: int, logits):
    p = _p1(q, kernel)
    _check(load().na1d_qk_rpb(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape),
                              _ptr(rpb, q.dtype, _rpb1(q, kernel)) if rpb is not None else None, scale,
                              _ptr(logits, q.dtype, _attn1(q, kernel)), _stream()))
    return logits


def na1d_softmax(logits, kernel: int, like, out):
    p = _p1(like, kernel)
    _check(load().na1d_softmax(ctypes.byref(p), _ptr(logits, like.dtype, _attn1(like, kernel)),
                               _ptr(out, like.dtype, _attn1(like, kernel)), _stream()))
    return out


def na1d_av(attn, v, kernel: int, out):
    p = _p1(v, kernel)
    _check(load().na1d_av(ctypes.byref(p), _ptr(attn, v.dtype, _attn1(v, kernel)), _ptr(v), _ptr(out, v.dtype, v.shape),
                          _stream()))
    return out


def na1d_fused_fwd(q, k_, v, rpb, scale: float, kernel: int, out, lse=None):
    p = _p1(q, kernel)
    _check(load().na1d_fused_fwd(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape), _ptr(v, q.dtype, q.shape),
                                 _ptr(rpb, q.dtype, _rpb1(q, kernel)) if rpb is not None else None, scale,
                                 _ptr(out, q.dtype, q.shape),
                                 _ptr(lse, torch.float32, q.shape[:3]) if lse is not None else None, _stream()))
    return out


def na1d_av_bwd_p(dout, v, kernel: int, dp):
    p = _p1(v, kernel)
    _check(load().na1d_av_bwd_p(ctypes.byref(p), _ptr(dout, v.dtype, v.shape), _ptr(v), _ptr(dp, v.dtype, _attn1(v, kernel)),
                                _stream()))
    return dp


def na1d_av_bwd_v(attn, dout, kernel: int, dv):
    p = _p1(dout, kernel)
    _check(load().na1d_av_bwd_v(ctypes.byref(p), _ptr(attn, dout.dtype, _attn1(dout, kernel)), _ptr(dout),
                                _ptr(dv, dout.dtype, dout.shape), _stream()))
    return dv


def na1d_softmax_bwd(attn, dp, kernel: int, like, ds):
    p = _p1(like, kernel)
    shape = _attn1(like, kernel)
    _check(load().na1d_softmax_bwd(ctypes.byref(p), _ptr(attn, like.dtype, shape), _ptr(dp, like.dtype, shape),
                                   _ptr(ds, like.dtype, shape), _stream()))
    return ds


def na1d_qk_bwd_q(ds, k_, scale: float, kernel: int, dq):
    p = _p1(k_, kernel)
    _check(load().na1d_qk_bwd_q(ctypes.byref(p), _ptr(ds, k_.dtype, _attn1(k_, kernel)), _ptr(k_), scale,
                                _ptr(dq, k_.dtype, k_.shape), _stream()))
    return dq


def na1d_qk_bwd_k(ds, q, scale: float, kernel: int, dk):
    p = _p1(q, kernel)
    _check(load().na1d_qk_bwd_k(ctypes.byref(p), _ptr(ds, q.dtype, _attn1(q, kernel)), _ptr(q), scale,
                                _ptr(dk, q.dtype, q.shape), _stream()))
    return dk


def na1d_workspace_bytes(p: Na1dProblem) -> int:
    return int(load().na1d_workspace_bytes(ctypes.byref(p)))


def na1d_qk_bwd_rpb(ds, kernel: int, like, d_rpb, workspace):
    p = _p1(like, kernel)
    _check(load().na1d_qk_bwd_rpb(ctypes.byref(p), _ptr(ds, like.dtype, _attn1(like, kernel)),
                                  _ptr(d_rpb, torch.float32, _rpb1(like, kernel)), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()))
    return d_rpb


def na1d_fused_bwd_workspace_bytes(p: Na1dProblem) -> int:
    return int(load().na1d_fused_bwd_workspace_bytes(ctypes.byref(p)))


def na1d_fused_bwd(q, k_, v, rpb, scale: float, lse, dout, kernel: int, dq, dk, dv, d_rpb, workspace):
    p = _p1(q, kernel)
    _check(load().na1d_fused_bwd(ctypes.byref(p), _ptr(q), _ptr(k_, q.dtype, q.shape), _ptr(v, q.dtype, q.shape),
                                 _ptr(rpb, q.dtype, _rpb1(q, kernel)) if rpb is not None else None, scale,
                                 _ptr(lse, torch.float32, q.shape[:3]), _ptr(dout, q.dtype, q.shape),
                                 _ptr(dq, q.dtype, q.shape), _ptr(dk, q.dtype, q.shape), _ptr(dv, q.dtype, q.shape),
                                 _ptr(d_rpb, torch.float32, _rpb1(q, kernel)) if d_rpb is not None else None,
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))
    return dq, dk, dv, d_rpb
