"""ctypes front end of the fp64 CPU oracle (``na2d_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this module.  It never touches the GPU library and the GPU library never
touches it.  Everything goes in and comes out as C-contiguous ``numpy.float64`` arrays
in the layouts documented at the top of ``na2d_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "na2d_oracle.c")
_LIB = os.path.join(_HERE, "libna2d_oracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ctypes.CDLL(_LIB)
        _lib.na2d_oracle_window_start.restype = ctypes.c_int
        _lib.na2d_oracle_num_threads.restype = ctypes.c_int
    return _lib


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float64)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_dp)


def num_threads() -> int:
    return int(_load().na2d_oracle_num_threads())


def set_threads(n: int) -> None:
    _load().na2d_oracle_set_threads(ctypes.c_int(int(n)))


def window_start(i: int, L: int, k: int) -> int:
    return int(_load().na2d_oracle_window_start(int(i), int(L), int(k)))


def indices(H: int, W: int, k: int):
    """(key_index, rpb_index), both int32 [H, W, k*k]."""
    key_index = np.empty((H, W, k * k), dtype=np.int32)
    rpb_index = np.empty((H, W, k * k), dtype=np.int32)
    _load().na2d_oracle_indices(int(H), int(W), int(k),
                                key_index.ctypes.data_as(_ip), rpb_index.ctypes.data_as(_ip))
    return key_index, rpb_index


def _dims(x, k):
    B, heads, H, W, D = x.shape
    return (ctypes.c_int(B), ctypes.c_int(heads), ctypes.c_int(H), ctypes.c_int(W),
            ctypes.c_int(D), ctypes.c_int(int(k)))


def qk_rpb(q, key, rpb, scale: float, k: int) -> np.ndarray:
    q, key = _f64(q), _f64(key)
    rpb = None if rpb is None else _f64(rpb)
    B, heads, H, W, D = q.shape
    logits = np.empty((B, heads, H, W, k * k), dtype=np.float64)
    _load().na2d_oracle_qk_rpb(*_dims(q, k), _ptr(q), _ptr(key), _ptr(rpb),
                               ctypes.c_double(scale), _ptr(logits))
    return logits


def softmax(logits, return_lse: bool = False):
    logits = _f64(logits)
    kk = logits.shape[-1]
    rows = logits.size // kk
    p = np.empty_like(logits)
    lse = np.empty(logits.shape[:-1], dtype=np.float64) if return_lse else None
    _load().na2d_oracle_softmax(ctypes.c_size_t(rows), ctypes.c_int(kk), _ptr(logits), _ptr(p), _ptr(lse))
    return (p, lse) if return_lse else p


def av(p, v, k: int) -> np.ndarray:
    p, v = _f64(p), _f64(v)
    out = np.empty_like(v)
    _load().na2d_oracle_av(*_dims(v, k), _ptr(p), _ptr(v), _ptr(out))
    return out


def fwd(q, key, v, rpb, scale: float, k: int, return_lse: bool = False):
    q, key, v = _f64(q), _f64(key), _f64(v)
    rpb = None if rpb is None else _f64(rpb)
    out = np.empty_like(q)
    lse = np.empty(q.shape[:-1], dtype=np.float64) if return_lse else None
    _load().na2d_oracle_fwd(*_dims(q, k), _ptr(q), _ptr(key), _ptr(v), _ptr(rpb),
                            ctypes.c_double(scale), _ptr(out), _ptr(lse))
    return (out, lse) if return_lse else out


def av_bwd_p(dout, v, k: int) -> np.ndarray:
    dout, v = _f64(dout), _f64(v)
    B, heads, H, W, D = v.shape
    dp = np.empty((B, heads, H, W, k * k), dtype=np.float64)
    _load().na2d_oracle_av_bwd_p(*_dims(v, k), _ptr(dout), _ptr(v), _ptr(dp))
    return dp


def av_bwd_v(p, dout, k: int) -> np.ndarray:
    p, dout = _f64(p), _f64(dout)
    dv = np.empty_like(dout)
    _load().na2d_oracle_av_bwd_v(*_dims(dout, k), _ptr(p), _ptr(dout), _ptr(dv))
    return dv


def softmax_bwd(p, dp) -> np.ndarray:
    p, dp = _f64(p), _f64(dp)
    kk = p.shape[-1]
    ds = np.empty_like(p)
    _load().na2d_oracle_softmax_bwd(ctypes.c_size_t(p.size // kk), ctypes.c_int(kk), _ptr(p), _ptr(dp), _ptr(ds))
    return ds


def qk_bwd_q(ds, key, scale: float, k: int) -> np.ndarray:
    ds, key = _f64(ds), _f64(key)
    dq = np.empty_like(key)
    _load().na2d_oracle_qk_bwd_q(*_dims(key, k), _ptr(ds), _ptr(key), ctypes.c_double(scale), _ptr(dq))
    return dq


def qk_bwd_k(ds, q, scale: float, k: int) -> np.ndarray:
    ds, q = _f64(ds), _f64(q)
    dk = np.empty_like(q)
    _load().na2d_oracle_qk_bwd_k(*_dims(q, k), _ptr(ds), _ptr(q), ctypes.c_double(scale), _ptr(dk))
    return dk


def qk_bwd_rpb(ds, k: int) -> np.ndarray:
    ds = _f64(ds)
    B, heads, H, W, _ = ds.shape
    d_rpb = np.empty((heads, 2 * k - 1, 2 * k - 1), dtype=np.float64)
    _load().na2d_oracle_qk_bwd_rpb(ctypes.c_int(B), ctypes.c_int(heads), ctypes.c_int(H), ctypes.c_int(W),
                                   ctypes.c_int(int(k)), _ptr(ds), _ptr(d_rpb))
    return d_rpb


def bwd(q, key, v, rpb, scale: float, dout, k: int):
    """(dq, dk, dv, d_rpb) of sum(out * dout); d_rpb is None when rpb is None."""
    q, key, v, dout = _f64(q), _f64(key), _f64(v), _f64(dout)
    rpb = None if rpb is None else _f64(rpb)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    heads = q.shape[1]
    d_rpb = None if rpb is None else np.empty((heads, 2 * k - 1, 2 * k - 1), dtype=np.float64)
    _load().na2d_oracle_bwd(*_dims(q, k), _ptr(q), _ptr(key), _ptr(v), _ptr(rpb), ctypes.c_double(scale),
                            _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(d_rpb))
    return dq, dk, dv, d_rpb
