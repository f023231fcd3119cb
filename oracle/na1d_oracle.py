"""fp64 CPU oracle for 1D Neighborhood Attention -- TEST INFRASTRUCTURE ONLY.

The operation of "Neighborhood Attention Transformer" (arXiv 2204.07143), Section 3.1, Eq. 2-4,
on a sequence instead of a feature map (the paper's package also ships a 1D module, Appendix A,
"Implementation notes"): every token attends to its k nearest tokens; at the two ends the window
is shifted, never shrunk, so each query keeps exactly k keys; a relative positional bias B(i, j)
is added to the logits.  Plain numpy in double precision: one loop over query positions and one
over window slots per definition, vectorised over (batch, head) only; the gradients of keys, values
and bias are scatter-adds in query order.  No blocking, fusion or reordering.

Only tests and the smoke check may import this module; it shares no code with the HIP path.

Parity pins (tests/test_oracle_na1d.py): dense self attention at k = L (brute force and torch's
scaled_dot_product_attention), brute-force k-nearest neighbourhoods, the box-mean special case
(avg_pool1d), an independent gather + batched-matmul formulation differentiated by autograd,
central finite differences, the adjoint identity, the closed-form bias-gradient counts, translation
equivariance away from the ends.  No function here is "parity unpinned".

Layouts (C order):  q, k, v, out, dout, dq, dk, dv : [B, heads, L, D]
                    logits, p, dp, ds             : [B, heads, L, k]   (slot a = key s(i) + a)
                    rpb, d_rpb                    : [heads, 2k-1]
                    lse                           : [B, heads, L]
Readings (the same as for the 2D operator): s(i) = clamp(i - (k-1)/2, 0, L - k); logit =
scale * <q_i, k_j> + rpb[head, j - i + k - 1] (bias unscaled).
"""
from __future__ import annotations

import numpy as np


def window_start(i: int, L: int, k: int) -> int:
    """First key position seen by query position i (Section 3.1: the k nearest, shifted at the ends)."""
    return min(max(i - (k - 1) // 2, 0), L - k)


def _f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def _check(L: int, k: int):
    if k % 2 == 0 or k < 1 or k > L:
        raise ValueError("k must be odd and at most L")


def qk_rpb(q, key, rpb, scale: float, k: int) -> np.ndarray:
    """Eq. 2: logits[i, a] = scale * <q_i, k_{s(i)+a}> + B(i, s(i)+a)."""
    q, key = _f64(q), _f64(key)
    B, heads, L, D = q.shape
    _check(L, k)
    logits = np.empty((B, heads, L, k))
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            j = s + a
            logits[:, :, i, a] = scale * np.sum(q[:, :, i, :] * key[:, :, j, :], axis=-1)
            if rpb is not None:
                logits[:, :, i, a] += _f64(rpb)[None, :, j - i + k - 1]
    return logits


def softmax(logits, return_lse: bool = False):
    """Eq. 4: softmax over the k window slots (max-subtracted)."""
    logits = _f64(logits)
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    z = e.sum(axis=-1, keepdims=True)
    p = e / z
    return (p, (m + np.log(z))[..., 0]) if return_lse else p


def av(p, v, k: int) -> np.ndarray:
    """Eq. 3-4: out_i = sum_a p[i, a] * v_{s(i)+a}."""
    p, v = _f64(p), _f64(v)
    B, heads, L, D = v.shape
    _check(L, k)
    out = np.zeros_like(v)
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            out[:, :, i, :] += p[:, :, i, a, None] * v[:, :, s + a, :]
    return out


def fwd(q, key, v, rpb, scale: float, k: int, return_lse: bool = False):
    p, lse = softmax(qk_rpb(q, key, rpb, scale, k), return_lse=True)
    out = av(p, v, k)
    return (out, lse) if return_lse else out


# ---- backward: the chain rule on the three steps above ------------------------------------

def av_bwd_p(dout, v, k: int) -> np.ndarray:
    """dp[i, a] = <dout_i, v_{s(i)+a}>."""
    dout, v = _f64(dout), _f64(v)
    B, heads, L, D = v.shape
    _check(L, k)
    dp = np.empty((B, heads, L, k))
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            dp[:, :, i, a] = np.sum(dout[:, :, i, :] * v[:, :, s + a, :], axis=-1)
    return dp


def av_bwd_v(p, dout, k: int) -> np.ndarray:
    """dv_j = sum over the queries i that see j of p[i, j - s(i)] * dout_i (scatter-add in query order)."""
    p, dout = _f64(p), _f64(dout)
    B, heads, L, D = dout.shape
    _check(L, k)
    dv = np.zeros_like(dout)
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            dv[:, :, s + a, :] += p[:, :, i, a, None] * dout[:, :, i, :]
    return dv


def softmax_bwd(p, dp) -> np.ndarray:
    """ds = p * (dp - <p, dp>) per row."""
    p, dp = _f64(p), _f64(dp)
    return p * (dp - np.sum(p * dp, axis=-1, keepdims=True))


def qk_bwd_q(ds, key, scale: float, k: int) -> np.ndarray:
    ds, key = _f64(ds), _f64(key)
    B, heads, L, D = key.shape
    _check(L, k)
    dq = np.zeros_like(key)
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            dq[:, :, i, :] += scale * ds[:, :, i, a, None] * key[:, :, s + a, :]
    return dq


def qk_bwd_k(ds, q, scale: float, k: int) -> np.ndarray:
    ds, q = _f64(ds), _f64(q)
    B, heads, L, D = q.shape
    _check(L, k)
    dk = np.zeros_like(q)
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            dk[:, :, s + a, :] += scale * ds[:, :, i, a, None] * q[:, :, i, :]
    return dk


def qk_bwd_rpb(ds, k: int) -> np.ndarray:
    """d_rpb[h, u] = sum over batch, queries and slots whose bias cell is u of ds."""
    ds = _f64(ds)
    B, heads, L, _ = ds.shape
    _check(L, k)
    d_rpb = np.zeros((heads, 2 * k - 1))
    for i in range(L):
        s = window_start(i, L, k)
        for a in range(k):
            d_rpb[:, (s + a) - i + k - 1] += ds[:, :, i, a].sum(axis=0)
    return d_rpb


def bwd(q, key, v, rpb, scale: float, dout, k: int):
    """(dq, dk, dv, d_rpb) of sum(out * dout); d_rpb is None when rpb is None."""
    p = softmax(qk_rpb(q, key, rpb, scale, k))
    dp = av_bwd_p(dout, v, k)
    dv = av_bwd_v(p, dout, k)
    ds = softmax_bwd(p, dp)
    return (qk_bwd_q(ds, key, scale, k), qk_bwd_k(ds, q, scale, k), dv,
            None if rpb is None else qk_bwd_rpb(ds, k))
