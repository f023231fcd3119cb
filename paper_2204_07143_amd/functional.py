"""Differentiable wrappers around the C-ABI calls (``torch.autograd.Function``), for drop-in use.

The paper's extension exposes two differentiable functions, QK+RPB and AV, with the softmax
between them left to the framework (arXiv 2204.07143, Appendix A, "Implementation notes");
``na2d_qk_rpb`` and ``na2d_av`` below are that split.  ``na2d`` is the whole operator (Eq. 2-4)
through the fused forward and the fused backward, which keep the attention tensor out of memory.

Only argument marshalling and buffer allocation happen here: every gradient comes from the
library's kernels.  Tensors are ``[B, heads, H, W, D]`` (q, k, v, out), ``[B, heads, H, W, k*k]``
(logits / attention weights) and ``[heads, 2k-1, 2k-1]`` (bias), contiguous, on the GPU; the
library is loaded on first use and a missing library raises.
"""
from __future__ import annotations

import torch

from . import binding as na


def _workspace(x: torch.Tensor, kernel_size: int, kind: int) -> torch.Tensor:
    B, heads, H, W, D = x.shape
    p = na.problem(B, heads, H, W, D, kernel_size, x.dtype)
    return torch.empty(max(16, na.na2d_workspace_bytes(p, kind)), dtype=torch.uint8, device=x.device)


def _bias_grad(d_rpb_f32, rpb):
    return None if d_rpb_f32 is None else d_rpb_f32.to(rpb.dtype)


class _NA2DQKRPB(torch.autograd.Function):
    """logits = scale * <q, k over the neighbourhood> + bias (Eq. 2)."""

    @staticmethod
    def forward(ctx, q, k, rpb, kernel_size, scale):
        q, k = q.contiguous(), k.contiguous()
        rpb_c = None if rpb is None else rpb.contiguous()
        logits = torch.empty((*q.shape[:4], kernel_size * kernel_size), dtype=q.dtype, device=q.device)
        na.na2d_qk_rpb(q, k, rpb_c, scale, kernel_size, logits)
        ctx.save_for_backward(q, k)
        ctx.kernel_size, ctx.scale, ctx.has_rpb = kernel_size, scale, rpb is not None
        ctx.rpb_dtype = None if rpb is None else rpb.dtype
        return logits

    @staticmethod
    def backward(ctx, dlogits):
        q, k = ctx.saved_tensors
        ks, scale = ctx.kernel_size, ctx.scale
        dlogits = dlogits.contiguous()
        dq, dk, d_rpb = None, None, None
        if ctx.needs_input_grad[0]:
            dq = na.na2d_qk_bwd_q(dlogits, k, scale, ks, torch.empty_like(q))
        if ctx.needs_input_grad[1]:
            dk = na.na2d_qk_bwd_k(dlogits, q, scale, ks, torch.empty_like(k))
        if ctx.has_rpb and ctx.needs_input_grad[2]:
            d32 = torch.empty((q.shape[1], 2 * ks - 1, 2 * ks - 1), dtype=torch.float32, device=q.device)
            na.na2d_qk_bwd_rpb(dlogits, ks, q, d32, _workspace(q, ks, na.WS_QK_BWD_RPB))
            d_rpb = d32.to(ctx.rpb_dtype)
        return dq, dk, d_rpb, None, None


class _NA2DAV(torch.autograd.Function):
    """out = attention weights times the neighbourhood's values (Eq. 3-4)."""

    @staticmethod
    def forward(ctx, attn, v, kernel_size):
        attn, v = attn.contiguous(), v.contiguous()
        out = na.na2d_av(attn, v, kernel_size, torch.empty_like(v))
        ctx.save_for_backward(attn, v)
        ctx.kernel_size = kernel_size
        return out

    @staticmethod
    def backward(ctx, dout):
        attn, v = ctx.saved_tensors
        ks = ctx.kernel_size
        dout = dout.contiguous()
        dattn, dv = None, None
        if ctx.needs_input_grad[0]:
            dattn = na.na2d_av_bwd_p(dout, v, ks, torch.empty_like(attn))
        if ctx.needs_input_grad[1]:
            dv = na.na2d_av_bwd_v(attn, dout, ks, torch.empty_like(v))
        return dattn, dv, None


class _NA2D(torch.autograd.Function):
    """The whole operator: softmax(scale * QK + bias) V over each query's neighbourhood."""

    @staticmethod
    def forward(ctx, q, k, v, rpb, kernel_size, scale):
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        rpb_c = None if rpb is None else rpb.contiguous()
        out = torch.empty_like(q)
        lse = torch.empty(q.shape[:4], dtype=torch.float32, device=q.device)
        na.na2d_fused_fwd(q, k, v, rpb_c, scale, kernel_size, out, lse)
        ctx.save_for_backward(q, k, v, lse) if rpb_c is None else ctx.save_for_backward(q, k, v, lse, rpb_c)
        ctx.kernel_size, ctx.scale, ctx.has_rpb = kernel_size, scale, rpb is not None
        return out

    @staticmethod
    def backward(ctx, dout):
        if ctx.has_rpb:
            q, k, v, lse, rpb = ctx.saved_tensors
        else:
            (q, k, v, lse), rpb = ctx.saved_tensors, None
        ks = ctx.kernel_size
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        want_bias = ctx.has_rpb and ctx.needs_input_grad[3]
        d32 = torch.empty((q.shape[1], 2 * ks - 1, 2 * ks - 1), dtype=torch.float32, device=q.device) if want_bias else None
        na.na2d_fused_bwd(q, k, v, rpb, ctx.scale, lse, dout.contiguous(), ks, dq, dk, dv, d32,
                          _workspace(q, ks, na.WS_FUSED_BWD))
        return dq, dk, dv, (d32.to(rpb.dtype) if want_bias else None), None, None


class _NA1D(torch.autograd.Function):
    """The 1D operator on [B, heads, L, D] tensors (bias [heads, 2k-1]): fused forward, fused backward."""

    @staticmethod
    def forward(ctx, q, k, v, rpb, kernel_size, scale):
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        rpb_c = None if rpb is None else rpb.contiguous()
        out = torch.empty_like(q)
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
        na.na1d_fused_fwd(q, k, v, rpb_c, scale, kernel_size, out, lse)
        ctx.save_for_backward(q, k, v, lse) if rpb_c is None else ctx.save_for_backward(q, k, v, lse, rpb_c)
        ctx.kernel_size, ctx.scale, ctx.has_rpb = kernel_size, scale, rpb is not None
        return out

    @staticmethod
    def backward(ctx, dout):
        if ctx.has_rpb:
            q, k, v, lse, rpb = ctx.saved_tensors
        else:
            (q, k, v, lse), rpb = ctx.saved_tensors, None
        ks = ctx.kernel_size
        B, heads, L, D = q.shape
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        want_bias = ctx.has_rpb and ctx.needs_input_grad[3]
        d32 = torch.empty((heads, 2 * ks - 1), dtype=torch.float32, device=q.device) if want_bias else None
        ws = torch.empty(max(16, na.na1d_fused_bwd_workspace_bytes(na.problem_1d(B, heads, L, D, ks, q.dtype))),
                         dtype=torch.uint8, device=q.device)
        na.na1d_fused_bwd(q, k, v, rpb, ctx.scale, lse, dout.contiguous(), ks, dq, dk, dv, d32, ws)
        return dq, dk, dv, (d32.to(rpb.dtype) if want_bias else None), None, None


class _NA2DSoftmax(torch.autograd.Function):
    """attn = softmax(logits) over the k*k axis (Eq. 4), forward and backward by the library's kernels."""

    @staticmethod
    def forward(ctx, logits, like, kernel_size):
        logits = logits.contiguous()
        attn = na.na2d_softmax(logits, kernel_size, like, torch.empty_like(logits))
        ctx.save_for_backward(attn)
        ctx.kernel_size, ctx.like_shape = kernel_size, like.shape
        return attn

    @staticmethod
    def backward(ctx, dattn):
        (attn,) = ctx.saved_tensors
        like = torch.empty(ctx.like_shape, dtype=attn.dtype, device="meta")   # shape and dtype only
        ds = na.na2d_softmax_bwd(attn, dattn.contiguous(), ctx.kernel_size, like, torch.empty_like(attn))
        return ds, None, None


def _scale_of(q, scale):
    return float(q.shape[-1]) ** -0.5 if scale is None else float(scale)


def na2d_qk_rpb(q, k, rpb, kernel_size: int, scale: float | None = None):
    """Neighbourhood logits ``[B, heads, H, W, k*k]``; differentiable in q, k and rpb (rpb may be None)."""
    return _NA2DQKRPB.apply(q, k, rpb, int(kernel_size), _scale_of(q, scale))


def na2d_av(attn, v, kernel_size: int):
    """Weighted sum of the neighbourhood's values ``[B, heads, H, W, D]``; differentiable in attn and v."""
    return _NA2DAV.apply(attn, v, int(kernel_size))


def na2d(q, k, v, rpb=None, kernel_size: int = 7, scale: float | None = None):
    """2D neighbourhood attention, fused; differentiable in q, k, v and rpb."""
    return _NA2D.apply(q, k, v, rpb, int(kernel_size), _scale_of(q, scale))


def na1d(q, k, v, rpb=None, kernel_size: int = 7, scale: float | None = None):
    """1D neighbourhood attention ([B, heads, L, D]), fused; differentiable in q, k, v and rpb."""
    return _NA1D.apply(q, k, v, rpb, int(kernel_size), _scale_of(q, scale))


def na2d_softmax(logits, like, kernel_size: int):
    """Softmax over the k*k axis of neighbourhood logits; ``like`` is any [B, heads, H, W, D] tensor of the
    problem (its shape and dtype describe it to the library).  Differentiable in logits."""
    return _NA2DSoftmax.apply(logits, like, int(kernel_size))


def na2d_unfused(q, k, v, rpb=None, kernel_size: int = 7, scale: float | None = None):
    """The same operator as the paper composes it: QK+RPB, softmax, AV; every step, forward and backward, is a
    library kernel."""
    logits = na2d_qk_rpb(q, k, rpb, kernel_size, scale)
    return na2d_av(na2d_softmax(logits, q, kernel_size), v, kernel_size)
