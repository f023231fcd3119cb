"""Pins for the oracle's backward functions (CPU only).

The paper (Appendix A) says which gradients its package computes -- for q, k, the bias b,
the attention weights a and v -- but prints no formulas, so the pins are mathematical:
central finite differences of the oracle's own forward (already pinned elsewhere), the
adjoint identity of each linear stage, torch autograd through the independent
gather + batched-matmul formulation, and a closed form for the bias gradient.
"""
import numpy as np
import pytest
import torch

from test_oracle_forward import gather_matmul_reference, rng


def bias_cell_counts(L, k):
    """cnt[u] = number of (query i, slot a) pairs on one axis whose bias row is u, by brute force
    over nearest-k windows."""
    cnt = np.zeros(2 * k - 1, dtype=np.int64)
    for i in range(L):
        order = sorted(range(L), key=lambda j: abs(j - i))
        for j in order[:k]:
            cnt[j - i + k - 1] += 1
    return cnt


def test_bias_cell_counts_examples():
    # worked examples: every query contributes k slots, so the counts sum to L * k
    assert bias_cell_counts(56, 7).tolist() == [1, 2, 3, 53, 54, 55, 56, 55, 54, 53, 3, 2, 1]
    assert bias_cell_counts(7, 7).tolist() == [1, 2, 3, 4, 5, 6, 7, 6, 5, 4, 3, 2, 1]
    assert bias_cell_counts(14, 3).tolist() == [1, 13, 14, 13, 1]


@pytest.mark.parametrize("B,heads,H,W,k", [(3, 2, 9, 12, 5), (2, 1, 7, 7, 7), (1, 2, 14, 14, 3), (1, 1, 13, 20, 13), (2, 1, 18, 25, 15),
                                           (1, 2, 21, 24, 21)])
def test_bias_gradient_closed_form_for_constant_ds(oracle, B, heads, H, W, k):
    ds = np.ones((B, heads, H, W, k * k))
    want = B * np.outer(bias_cell_counts(H, k), bias_cell_counts(W, k))
    got = oracle.qk_bwd_rpb(ds, k)
    for h in range(heads):
        np.testing.assert_array_equal(got[h], want)


def test_bias_gradient_separates_heads_and_slots(oracle):
    # one hot ds: a single (query, slot) must land in exactly one cell of its own head
    B, heads, H, W, k = 2, 3, 8, 9, 5
    key_index, rpb_index = oracle.indices(H, W, k)
    g = rng(1)
    for _ in range(20):
        b, h, qy, qx, j = g.integers(B), g.integers(heads), g.integers(H), g.integers(W), g.integers(k * k)
        ds = np.zeros((B, heads, H, W, k * k))
        ds[b, h, qy, qx, j] = 2.5
        got = oracle.qk_bwd_rpb(ds, k)
        want = np.zeros_like(got)
        want[h].reshape(-1)[rpb_index[qy, qx, j]] = 2.5
        np.testing.assert_array_equal(got, want)


def loss(oracle, q, key, v, rpb, scale, k, dout):
    return float((oracle.fwd(q, key, v, rpb, scale, k) * dout).sum())


@pytest.mark.parametrize("H,W,k", [(5, 6, 3), (7, 5, 5)])
def test_gradients_by_central_finite_differences(oracle, H, W, k):
    g = rng(20 + k)
    B, heads, D = 1, 2, 4
    q, key, v, dout = (g.standard_normal((B, heads, H, W, D)) for _ in range(4))
    rpb = g.standard_normal((heads, 2 * k - 1, 2 * k - 1))
    scale = 0.6
    dq, dk, dv, d_rpb = oracle.bwd(q, key, v, rpb, scale, dout, k)
    eps = 1e-6
    for name, x, grad in (("q", q, dq), ("k", key, dk), ("v", v, dv), ("rpb", rpb, d_rpb)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            up = loss(oracle, q, key, v, rpb, scale, k, dout)
            x[idx] = old - eps
            dn = loss(oracle, q, key, v, rpb, scale, k, dout)
            x[idx] = old
            num[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=2e-6, atol=2e-8, err_msg=name)


@pytest.mark.parametrize("B,heads,H,W,D,k", [(2, 2, 9, 11, 8, 5), (1, 2, 10, 8, 4, 7), (1, 1, 14, 14, 32, 3), (1, 1, 16, 17, 4, 15)])
def test_gradients_match_autograd_of_gather_matmul(oracle, B, heads, H, W, D, k):
    g = rng(40 + k)
    q, key, v, dout = (g.standard_normal((B, heads, H, W, D)) for _ in range(4))
    rpb = 0.3 * g.standard_normal((heads, 2 * k - 1, 2 * k - 1))
    scale = D ** -0.5
    tq, tk, tv, tb = (torch.from_numpy(x).clone().requires_grad_(True) for x in (q, key, v, rpb))
    _, _, out = gather_matmul_reference(tq, tk, tv, tb, scale, k)
    (out * torch.from_numpy(dout)).sum().backward()
    dq, dk, dv, d_rpb = oracle.bwd(q, key, v, rpb, scale, dout, k)
    for got, want in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad), (d_rpb, tb.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)
    # without a bias table the other three gradients are unchanged and d_rpb is absent
    dq0, dk0, dv0, none = oracle.bwd(q, key, v, None, scale, dout, k)
    assert none is None
    dq1, dk1, dv1, _ = oracle.bwd(q, key, v, np.zeros_like(rpb), scale, dout, k)
    for a, b in ((dq0, dq1), (dk0, dk1), (dv0, dv1)):
        np.testing.assert_array_equal(a, b)


def test_stagewise_backward_composes_and_is_adjoint(oracle):
    g = rng(60)
    B, heads, H, W, D, k = 2, 2, 8, 10, 6, 5
    kk = k * k
    q, key, v, dout = (g.standard_normal((B, heads, H, W, D)) for _ in range(4))
    rpb = g.standard_normal((heads, 2 * k - 1, 2 * k - 1))
    scale = 0.41
    p = oracle.softmax(oracle.qk_rpb(q, key, rpb, scale, k))
    dp = oracle.av_bwd_p(dout, v, k)
    dv = oracle.av_bwd_v(p, dout, k)
    ds = oracle.softmax_bwd(p, dp)
    dq = oracle.qk_bwd_q(ds, key, scale, k)
    dk = oracle.qk_bwd_k(ds, q, scale, k)
    d_rpb = oracle.qk_bwd_rpb(ds, k)
    cq, ck, cv, cb = oracle.bwd(q, key, v, rpb, scale, dout, k)
    for a, b in ((dq, cq), (dk, ck), (dv, cv), (d_rpb, cb)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-15)
    # rows of ds sum to zero (softmax weights sum to a constant)
    np.testing.assert_allclose(ds.sum(-1), 0.0, atol=1e-14)
    # adjoint identities <y, A x> = <A^T y, x> of the two bilinear stages, with random probes
    w = g.standard_normal((B, heads, H, W, kk))       # a probe in attention-weight space
    x = g.standard_normal((B, heads, H, W, D))        # a probe in value/key space
    # AV is linear in p and in v
    lhs = (dout * oracle.av(w, v, k)).sum()
    np.testing.assert_allclose(lhs, (oracle.av_bwd_p(dout, v, k) * w).sum(), rtol=1e-12)
    lhs = (dout * oracle.av(p, x, k)).sum()
    np.testing.assert_allclose(lhs, (oracle.av_bwd_v(p, dout, k) * x).sum(), rtol=1e-12)
    # QK+RPB is linear in q, in k and in rpb
    lin = lambda qq, kk_, bb: oracle.qk_rpb(qq, kk_, bb, scale, k)
    zero_b = np.zeros_like(rpb)
    np.testing.assert_allclose((w * lin(x, key, zero_b)).sum(), (oracle.qk_bwd_q(w, key, scale, k) * x).sum(), rtol=1e-12)
    np.testing.assert_allclose((w * lin(q, x, zero_b)).sum(), (oracle.qk_bwd_k(w, q, scale, k) * x).sum(), rtol=1e-12)
    pb = g.standard_normal(rpb.shape)
    np.testing.assert_allclose((w * lin(np.zeros_like(q), key, pb)).sum(), (oracle.qk_bwd_rpb(w, k) * pb).sum(), rtol=1e-12)


def test_softmax_backward_against_jacobian(oracle):
    g = rng(61)
    x = g.standard_normal((3, 9))
    dp = g.standard_normal((3, 9))
    p = oracle.softmax(x)
    ds = oracle.softmax_bwd(p, dp)
    for n in range(3):
        jac = np.diag(p[n]) - np.outer(p[n], p[n])
        np.testing.assert_allclose(ds[n], jac @ dp[n], rtol=1e-12, atol=1e-15)
