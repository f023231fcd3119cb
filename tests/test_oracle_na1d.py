"""Pins for the 1D oracle (CPU only).  Expected values come from what the paper and the mathematics
fix, never from the oracle itself:
  * Section 3.1: the k nearest neighbours (brute force), and NA at its maximum neighbourhood
    (k = L) is self attention (dense numpy brute force, torch's scaled_dot_product_attention);
  * an independent formulation (gather the windows by index, two batched matmuls: the plain
    PyTorch route the Appendix describes) differentiated by autograd, for every gradient;
  * special cases that reduce to library routines (box mean = avg_pool1d), closed forms (bias
    gradient counts), finite differences, the adjoint identity, translation equivariance.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import na1d_oracle as o


def rng(seed):
    return np.random.default_rng(seed)


def make(seed, B, heads, L, D, k, bias_std=0.5):
    g = rng(seed)
    q, key, v, dout = (g.standard_normal((B, heads, L, D)) for _ in range(4))
    rpb = bias_std * g.standard_normal((heads, 2 * k - 1))
    return q, key, v, rpb, dout


@pytest.mark.parametrize("k", [1, 3, 5, 7, 9, 13, 31])
def test_window_is_the_k_nearest(k):
    for L in range(k, min(3 * k + 4, 60)):
        for i in range(L):
            # the k positions closest to i (ties cannot occur for odd k inside the sequence; at the
            # ends the one-sided candidates have distinct distances)
            order = sorted(range(L), key=lambda j: (abs(j - i), j))
            near = sorted(order[:k])
            # where the nearest-k set is not unique (a tie for the last place) the shifted window is one of them
            s = o.window_start(i, L, k)
            window = list(range(s, s + k))
            kth = abs(order[k - 1] - i)
            assert all(abs(j - i) <= kth for j in window), (L, i, k)
            if k < L and abs(order[k] - i) > kth:
                assert window == near, (L, i, k)
            assert 0 <= s and s + k <= L and s <= i < s + k


@pytest.mark.parametrize("L", [3, 7, 13])
def test_maximum_neighbourhood_is_self_attention(L):
    k = L
    q, key, v, rpb, _ = make(10 + L, 2, 3, L, 8, k)
    scale = 0.31
    out, lse = o.fwd(q, key, v, rpb, scale, k, return_lse=True)
    bias = np.empty((3, L, L))
    for i in range(L):
        for j in range(L):
            bias[:, i, j] = rpb[:, j - i + k - 1]
    s = scale * np.einsum("bhid,bhjd->bhij", q, key) + bias[None]
    e = np.exp(s - s.max(-1, keepdims=True))
    want = np.einsum("bhij,bhjd->bhid", e / e.sum(-1, keepdims=True), v)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, np.log(np.exp(s).sum(-1)), rtol=1e-12)
    t = lambda a: torch.from_numpy(a)
    sdpa = F.scaled_dot_product_attention(t(q), t(key), t(v), attn_mask=t(np.broadcast_to(bias[None], s.shape).copy()), scale=scale)
    np.testing.assert_allclose(out, sdpa.numpy(), rtol=1e-10, atol=1e-12)


def gather_formulation(q, key, v, rpb, scale, k):
    """Windows gathered by an index tensor, then two batched matmuls; torch fp64, differentiable."""
    B, heads, L, D = q.shape
    r = (k - 1) // 2
    start = torch.clamp(torch.arange(L) - r, 0, L - k)
    idx = start[:, None] + torch.arange(k)[None, :]                      # [L, k] key positions
    kw = key[:, :, idx]                                                  # [B, heads, L, k, D]
    vw = v[:, :, idx]
    logits = scale * torch.matmul(kw, q[..., None])[..., 0]
    if rpb is not None:
        rel = idx - torch.arange(L)[:, None] + (k - 1)
        logits = logits + rpb[:, rel][None]
    p = torch.softmax(logits, dim=-1)
    return torch.matmul(p[..., None, :], vw)[..., 0, :], logits, p


@pytest.mark.parametrize("L,k", [(9, 3), (12, 5), (20, 7), (16, 13), (40, 31)])
def test_forward_and_every_gradient_against_gather_matmul_autograd(L, k):
    q, key, v, rpb, dout = make(100 + L, 2, 2, L, 6, k)
    scale = 6 ** -0.5
    tq, tk, tv, tb = (torch.from_numpy(a).requires_grad_(True) for a in (q, key, v, rpb))
    out, logits, p = gather_formulation(tq, tk, tv, tb, scale, k)
    out.backward(torch.from_numpy(dout))
    np.testing.assert_allclose(o.qk_rpb(q, key, rpb, scale, k), logits.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(o.softmax(logits.detach().numpy()), p.detach().numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(o.av(p.detach().numpy(), v, k), out.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(o.fwd(q, key, v, rpb, scale, k), out.detach().numpy(), rtol=1e-12, atol=1e-13)
    dq, dk, dv, d_rpb = o.bwd(q, key, v, rpb, scale, dout, k)
    for got, want in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad), (d_rpb, tb.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)
    # the stage functions one by one, against autograd through the matching part of the formulation
    pn = p.detach().numpy()
    dp = o.av_bwd_p(dout, v, k)
    tp = torch.from_numpy(pn).requires_grad_(True)
    idx = torch.clamp(torch.arange(L) - (k - 1) // 2, 0, L - k)[:, None] + torch.arange(k)[None, :]
    (torch.matmul(tp[..., None, :], torch.from_numpy(v)[:, :, idx])[..., 0, :] * torch.from_numpy(dout)).sum().backward()
    np.testing.assert_allclose(dp, tp.grad.numpy(), rtol=1e-12, atol=1e-13)
    tl = logits.detach().clone().requires_grad_(True)
    (torch.softmax(tl, -1) * torch.from_numpy(dp)).sum().backward()
    np.testing.assert_allclose(o.softmax_bwd(pn, dp), tl.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_no_bias_and_bias_gradient_absent():
    q, key, v, _, dout = make(7, 1, 2, 11, 4, 5)
    out = o.fwd(q, key, v, None, 0.5, 5)
    want = gather_formulation(*(torch.from_numpy(a) for a in (q, key, v)), None, 0.5, 5)[0].numpy()
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    assert o.bwd(q, key, v, None, 0.5, dout, 5)[3] is None


def test_box_mean_special_case():
    """q = 0, no bias: uniform weights, so out is the k-wide box mean of v (avg_pool1d inside, the
    value at the nearest fully-inside position at the ends)."""
    L, k, r = 23, 7, 3
    g = rng(5)
    v = g.standard_normal((2, 2, L, 5))
    out = o.fwd(np.zeros_like(v), g.standard_normal(v.shape), v, None, 1.0, k)
    pooled = F.avg_pool1d(torch.from_numpy(v).permute(0, 1, 3, 2).reshape(4, 5, L), k, stride=1).reshape(2, 2, 5, L - k + 1)
    pooled = pooled.permute(0, 1, 3, 2).numpy()
    for i in range(L):
        c = min(max(i, r), L - 1 - r)
        np.testing.assert_allclose(out[:, :, i], pooled[:, :, c - r], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("L,k", [(56, 7), (10, 3), (13, 13), (40, 9)])
def test_bias_gradient_closed_form_counts(L, k):
    """ds == 1 everywhere: d_rpb[h, u] = B * (number of (query, key) pairs at relative offset u - (k-1))."""
    B, heads = 3, 2
    got = o.qk_bwd_rpb(np.ones((B, heads, L, k)), k)
    cnt = np.zeros(2 * k - 1)
    for i in range(L):
        for j in sorted(range(L), key=lambda j: (abs(j - i), j))[:k]:   # brute-force k nearest (unique for odd k)
            cnt[j - i + k - 1] += 1
    np.testing.assert_array_equal(got, np.broadcast_to(B * cnt, (heads, 2 * k - 1)))
    if (L, k) == (56, 7):   # the per-axis counts of a 56-long axis at k = 7
        assert list(cnt) == [1, 2, 3, 53, 54, 55, 56, 55, 54, 53, 3, 2, 1]
    assert cnt.sum() == L * k and cnt[k - 1] == L


def test_finite_differences_and_adjoint():
    L, k, scale = 8, 3, 0.7
    q, key, v, rpb, dout = make(77, 1, 2, L, 3, k)
    f = lambda q_, k_, v_, b_: float(np.sum(o.fwd(q_, k_, v_, b_, scale, k) * dout))
    grads = o.bwd(q, key, v, rpb, scale, dout, k)
    args = [q, key, v, rpb]
    eps = 1e-6
    g = rng(3)
    for n, (x, gx) in enumerate(zip(args, grads)):
        for _ in range(12):
            i = tuple(g.integers(0, s) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[i] += eps
            xm[i] -= eps
            a = list(args)
            a[n] = xp
            fp = f(*a)
            a[n] = xm
            fm = f(*a)
            assert abs((fp - fm) / (2 * eps) - gx[i]) < 1e-7, (n, i)
    # adjoint identity for the two linear maps: <av(p, v), dout> = <p, av_bwd_p(dout, v)> = <v, av_bwd_v(p, dout)>
    p = g.standard_normal((1, 2, L, k))
    lhs = np.sum(o.av(p, v, k) * dout)
    assert abs(lhs - np.sum(p * o.av_bwd_p(dout, v, k))) < 1e-12
    assert abs(lhs - np.sum(v * o.av_bwd_v(p, dout, k))) < 1e-12
    ds = g.standard_normal((1, 2, L, k))
    lhs = np.sum(o.qk_rpb(q, key, None, scale, k) * ds)
    assert abs(lhs - np.sum(q * o.qk_bwd_q(ds, key, scale, k))) < 1e-12
    assert abs(lhs - np.sum(key * o.qk_bwd_k(ds, q, scale, k))) < 1e-12
    # rows of ds from a softmax backward sum to zero
    assert np.abs(o.softmax_bwd(o.softmax(p), ds).sum(-1)).max() < 1e-14


def test_translation_equivariance_away_from_the_ends():
    L, k, r, shift = 30, 5, 2, 4
    q, key, v, rpb, _ = make(91, 1, 1, L, 4, k)
    out = o.fwd(q, key, v, rpb, 0.4, k)
    crop = slice(shift, shift + 18)
    out_c = o.fwd(q[:, :, crop], key[:, :, crop], v[:, :, crop], rpb, 0.4, k)
    # queries whose window is centred in both the sequence and its crop
    np.testing.assert_allclose(out_c[:, :, r:18 - r], out[:, :, shift + r:shift + 18 - r], rtol=1e-12, atol=1e-14)


def test_bias_is_unscaled_and_indexed_by_key_minus_query():
    L, k = 9, 3
    q, key, v, rpb, _ = make(5, 1, 2, L, 4, k)
    scale = 0.25
    # scaling the whole logit (the literal form of Eq. 4) is the same function with the table divided by the scale
    a = o.qk_rpb(q, key, rpb, scale, k)
    b = scale * (o.qk_rpb(q, key, None, 1.0, k) + o.qk_rpb(np.zeros_like(q), key, rpb / scale, 1.0, k))
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    # sequence reversal: the same operator with the bias table flipped
    rev = lambda t: t[:, :, ::-1].copy()
    out = o.fwd(q, key, v, rpb, scale, k)
    out_r = o.fwd(rev(q), rev(key), rev(v), rpb[:, ::-1].copy(), scale, k)
    np.testing.assert_allclose(rev(out_r), out, rtol=1e-12, atol=1e-14)
    # an interior query only uses the central k cells; cell k-1+d belongs to key = query + d
    only = np.zeros_like(rpb)
    only[:, k - 1 + 1] = 1.0   # key one to the right of the query
    lg = o.qk_rpb(np.zeros_like(q), key, only, 1.0, k)
    assert np.all(lg[:, :, 4, :] == np.array([0.0, 0.0, 1.0]))
    assert np.all(lg[:, :, 0, :] == np.array([0.0, 1.0, 0.0]))   # query 0 sees keys 0, 1, 2
