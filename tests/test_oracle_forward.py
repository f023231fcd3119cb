"""Pins for the oracle's forward functions (CPU only).

Expected values come from what the paper and the mathematics fix, never from the oracle:
  * Section 3.1 (after Eq. 4): with the neighbourhood at its maximum (k = H = W) NA is
    self attention (Eq. 1) -- checked against a dense numpy brute force and against
    torch's scaled_dot_product_attention in fp64;
  * Appendix "Notes on translational equivariance": NA is translation-equivariant away
    from the borders;
  * Eq. 4: softmax weights are a convex combination;
  * special cases that reduce to library routines (box mean = avg_pool2d; gather +
    batched matmul, the plain-PyTorch formulation the Appendix describes).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F


def rng(seed):
    return np.random.default_rng(seed)


def dense_self_attention(q, k, v, bias, scale):
    """Eq. 1 with an additive bias: softmax(scale * Q K^T + bias) V, per (batch, head)."""
    B, Hh, N, D = q.shape
    out = np.empty_like(q)
    for b in range(B):
        for h in range(Hh):
            s = scale * q[b, h] @ k[b, h].T + bias[h]
            s = s - s.max(axis=1, keepdims=True)
            e = np.exp(s)
            out[b, h] = (e / e.sum(axis=1, keepdims=True)) @ v[b, h]
    return out


def full_bias_matrix(rpb, L, k):
    """Bias[h, i, j] = rpb[h, jy - iy + k - 1, jx - ix + k - 1] on an L x L map."""
    heads = rpb.shape[0]
    bias = np.empty((heads, L * L, L * L))
    for iy in range(L):
        for ix in range(L):
            for jy in range(L):
                for jx in range(L):
                    bias[:, iy * L + ix, jy * L + jx] = rpb[:, jy - iy + k - 1, jx - ix + k - 1]
    return bias


@pytest.mark.parametrize("L", [3, 5, 7])
def test_na_equals_self_attention_at_max_neighbourhood(oracle, L):
    g = rng(10 + L)
    B, heads, D, k = 2, 3, 8, L
    q, kk_, v = (g.standard_normal((B, heads, L, L, D)) for _ in range(3))
    rpb = 0.5 * g.standard_normal((heads, 2 * k - 1, 2 * k - 1))
    scale = D ** -0.5
    got = oracle.fwd(q, kk_, v, rpb, scale, k)
    flat = lambda x: x.reshape(B, heads, L * L, D)
    bias = full_bias_matrix(rpb, L, k)
    want = dense_self_attention(flat(q), flat(kk_), flat(v), bias, scale).reshape(q.shape)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    # library cross-check: torch SDPA with a float mask, fp64
    t = lambda x: torch.from_numpy(flat(x))
    sd = F.scaled_dot_product_attention(t(q), t(kk_), t(v), attn_mask=torch.from_numpy(bias)[None], scale=scale)
    np.testing.assert_allclose(got, sd.numpy().reshape(q.shape), rtol=1e-10, atol=1e-11)


def brute_nearest_window(i, L, k):
    order = sorted(range(L), key=lambda j: abs(j - i))
    return sorted(order[:k])


def gather_matmul_reference(q, key, v, rpb, scale, k):
    """The plain-PyTorch formulation (Appendix A, 'Background'): gather every query's
    neighbourhood (chosen here by brute-force nearest-k), then two batched matmuls.
    Written with torch fp64 ops so autograd can also give gradients."""
    B, heads, H, W, D = q.shape
    ky = torch.tensor([brute_nearest_window(i, H, k) for i in range(H)])  # [H, k]
    kx = torch.tensor([brute_nearest_window(i, W, k) for i in range(W)])  # [W, k]
    yy = ky[:, None, :, None].expand(H, W, k, k)
    xx = kx[None, :, None, :].expand(H, W, k, k)
    flat_idx = (yy * W + xx).reshape(H * W, k * k)  # [HW, kk]
    qy = torch.arange(H)[:, None, None, None].expand(H, W, k, k)
    qx = torch.arange(W)[None, :, None, None].expand(H, W, k, k)
    bu = (yy - qy + k - 1).reshape(H * W, k * k)
    bv = (xx - qx + k - 1).reshape(H * W, k * k)
    kf = key.reshape(B, heads, H * W, D)
    vf = v.reshape(B, heads, H * W, D)
    kn = kf[:, :, flat_idx]  # [B, heads, HW, kk, D]
    vn = vf[:, :, flat_idx]
    logits = scale * torch.einsum("bhnd,bhnjd->bhnj", q.reshape(B, heads, H * W, D), kn)
    if rpb is not None:
        logits = logits + rpb[:, bu, bv][None]
    p = torch.softmax(logits, dim=-1)
    out = torch.einsum("bhnj,bhnjd->bhnd", p, vn).reshape(B, heads, H, W, D)
    return logits.reshape(B, heads, H, W, k * k), p.reshape(B, heads, H, W, k * k), out


@pytest.mark.parametrize("B,heads,H,W,D,k", [(1, 1, 14, 14, 32, 3), (2, 2, 9, 11, 8, 5), (1, 2, 10, 8, 4, 7), (1, 1, 15, 13, 4, 13),
                                               (1, 2, 17, 19, 4, 15), (1, 1, 23, 21, 4, 21)])
def test_stages_match_gather_matmul_formulation(oracle, B, heads, H, W, D, k):
    g = rng(100 + H + k)
    q, key, v = (g.standard_normal((B, heads, H, W, D)) for _ in range(3))
    rpb = 0.3 * g.standard_normal((heads, 2 * k - 1, 2 * k - 1))
    scale = 0.37
    t = torch.from_numpy
    logits_ref, p_ref, out_ref = gather_matmul_reference(t(q), t(key), t(v), t(rpb), scale, k)
    logits = oracle.qk_rpb(q, key, rpb, scale, k)
    np.testing.assert_allclose(logits, logits_ref.numpy(), rtol=1e-12, atol=1e-12)
    p, lse = oracle.softmax(logits, return_lse=True)
    np.testing.assert_allclose(p, p_ref.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, torch.logsumexp(logits_ref, dim=-1).numpy(), rtol=1e-12)
    out = oracle.av(p, v, k)
    np.testing.assert_allclose(out, out_ref.numpy(), rtol=1e-12, atol=1e-13)
    # the composed forward is the same three steps
    out2, lse2 = oracle.fwd(q, key, v, rpb, scale, k, return_lse=True)
    np.testing.assert_allclose(out2, out, rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse2, lse, rtol=0, atol=1e-15)
    # no bias == zero bias
    np.testing.assert_allclose(oracle.qk_rpb(q, key, None, scale, k),
                               oracle.qk_rpb(q, key, np.zeros_like(rpb), scale, k), rtol=0, atol=0)


def test_softmax_is_a_convex_combination(oracle):
    g = rng(5)
    B, heads, H, W, D, k = 1, 2, 12, 9, 6, 5
    q, key, v = (g.standard_normal((B, heads, H, W, D)) for _ in range(3))
    rpb = g.standard_normal((heads, 9, 9))
    p = oracle.softmax(oracle.qk_rpb(q, key, rpb, 0.4, k))
    assert np.all(p > 0)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-13)
    out = oracle.av(p, v, k)
    key_index, _ = oracle.indices(H, W, k)
    vf = v.reshape(B, heads, H * W, D)
    win = vf[:, :, key_index.reshape(H * W, k * k)]  # [B, heads, HW, kk, D]
    lo, hi = win.min(axis=3).reshape(out.shape), win.max(axis=3).reshape(out.shape)
    assert np.all(out >= lo - 1e-12) and np.all(out <= hi + 1e-12)


def test_translation_equivariance_in_the_interior(oracle):
    # Appendix 'Notes on translational equivariance': NA keeps it except where windows are
    # repeated at the borders.  Shift the content by (dy, dx) inside a larger map and compare
    # queries whose windows are unclamped in both maps.
    g = rng(7)
    heads, D, k, r = 2, 5, 5, 2
    H, W, dy, dx = 15, 17, 3, 4
    big = {n: g.standard_normal((1, heads, H + dy, W + dx, D)) for n in "qkv"}
    rpb = g.standard_normal((heads, 9, 9))
    a = oracle.fwd(big["q"][:, :, :H, :W], big["k"][:, :, :H, :W], big["v"][:, :, :H, :W], rpb, 0.3, k)
    b = oracle.fwd(big["q"][:, :, dy:, dx:], big["k"][:, :, dy:, dx:], big["v"][:, :, dy:, dx:], rpb, 0.3, k)
    # pixel (y, x) of crop b is pixel (y + dy, x + dx) of crop a
    ya = slice(dy + r, H - r)
    xa = slice(dx + r, W - r)
    yb = slice(r, H - dy - r)
    xb = slice(r, W - dx - r)
    np.testing.assert_allclose(a[:, :, ya, xa], b[:, :, yb, xb], rtol=0, atol=1e-14)
    # and it is *not* kept at the corner, where the window is repeated
    assert not np.allclose(a[:, :, dy, dx], b[:, :, 0, 0])


@pytest.mark.parametrize("k", [3, 7])
def test_zero_query_gives_box_mean(oracle, k):
    g = rng(3)
    B, heads, H, W, D = 1, 2, 12, 15, 3
    r = k // 2
    v = g.standard_normal((B, heads, H, W, D))
    key = g.standard_normal(v.shape)
    out = oracle.fwd(np.zeros_like(v), key, v, None, 1.0, k)
    vt = torch.from_numpy(v).permute(0, 1, 4, 2, 3).reshape(B * heads * D, 1, H, W)
    pooled = F.avg_pool2d(vt, k, stride=1).reshape(B, heads, D, H - 2 * r, W - 2 * r).permute(0, 1, 3, 4, 2).numpy()
    np.testing.assert_allclose(out[:, :, r:H - r, r:W - r], pooled, rtol=1e-12, atol=1e-13)
    # a border query has the window of the nearest interior centre
    for qy in range(H):
        for qx in range(W):
            cy, cx = min(max(qy, r), H - 1 - r), min(max(qx, r), W - 1 - r)
            np.testing.assert_allclose(out[:, :, qy, qx], out[:, :, cy, cx], rtol=0, atol=1e-15)


def test_zero_query_gives_softmax_of_the_bias_block(oracle):
    g = rng(4)
    heads, H, W, D, k = 2, 9, 10, 4, 5
    r = k // 2
    rpb = g.standard_normal((heads, 2 * k - 1, 2 * k - 1))
    key = g.standard_normal((1, heads, H, W, D))
    p = oracle.softmax(oracle.qk_rpb(np.zeros_like(key), key, rpb, 1.0, k))
    for h in range(heads):
        for qy in range(H):
            for qx in range(W):
                fy = min(max(qy - r, 0), H - k)
                fx = min(max(qx - r, 0), W - k)
                uy, ux = fy - qy + k - 1, fx - qx + k - 1
                block = rpb[h, uy:uy + k, ux:ux + k].reshape(-1)
                e = np.exp(block - block.max())
                np.testing.assert_allclose(p[0, h, qy, qx], e / e.sum(), rtol=1e-12)


def test_bias_identities(oracle):
    g = rng(8)
    heads, H, W, D, k = 2, 8, 9, 4, 3
    q, key, v = (g.standard_normal((1, heads, H, W, D)) for _ in range(3))
    rpb = g.standard_normal((heads, 5, 5))
    scale = D ** -0.5
    ours = oracle.fwd(q, key, v, rpb, scale, k)
    # Eq. 2 + Eq. 4 read literally, softmax((QK^T + B) / sqrt(d)), is the same function with B * sqrt(d) passed in
    literal_logits = scale * oracle.qk_rpb(q, key, rpb / scale, 1.0, k)
    np.testing.assert_allclose(oracle.av(oracle.softmax(literal_logits), v, k), ours, rtol=1e-12, atol=1e-13)
    # opposite sign convention for the relative offset == flipping the table and the map
    flip = lambda x: x[:, :, ::-1, ::-1].copy()
    flipped = oracle.fwd(flip(q), flip(key), flip(v), rpb[:, ::-1, ::-1].copy(), scale, k)
    np.testing.assert_allclose(flip(flipped), ours, rtol=1e-12, atol=1e-13)


def test_softmax_shift_invariance_and_extremes(oracle):
    g = rng(9)
    x = g.standard_normal((4, 49))
    np.testing.assert_allclose(oracle.softmax(x + 1000.0), oracle.softmax(x), rtol=1e-10)
    one_hot = np.full((1, 9), -1e4)
    one_hot[0, 4] = 0.0
    p = oracle.softmax(one_hot)
    assert p[0, 4] == 1.0 and p.sum() == 1.0


# ---- SASA through zero padding (Section 3.1: SASA's sliding window can run on the NA kernels if
# the input is zero-padded; the windows of the un-padded positions are then all centred) ----------

def sasa_brute_force(q, k, v, bias_centre, scale, ks):
    """Stand-alone self attention with a centred ks x ks window and zero padding: keys outside the
    map are zero vectors that still take part in the softmax.  bias_centre[h, dy + r, dx + r]."""
    B, Hh, H, W, D = q.shape
    r = ks // 2
    out = np.zeros_like(q)
    for b in range(B):
        for h in range(Hh):
            for y in range(H):
                for x in range(W):
                    logit = np.empty(ks * ks)
                    vals = np.zeros((ks * ks, D))
                    for dy in range(-r, r + 1):
                        for dx in range(-r, r + 1):
                            s = (dy + r) * ks + dx + r
                            yy, xx = y + dy, x + dx
                            inside = 0 <= yy < H and 0 <= xx < W
                            kv = k[b, h, yy, xx] if inside else np.zeros(D)
                            if inside:
                                vals[s] = v[b, h, yy, xx]
                            logit[s] = scale * float(q[b, h, y, x] @ kv) + bias_centre[h, dy + r, dx + r]
                    e = np.exp(logit - logit.max())
                    out[b, h, y, x] = (e / e.sum()) @ vals
    return out


@pytest.mark.parametrize("H,W,ks", [(5, 6, 3), (6, 7, 5), (4, 9, 7)])
def test_sasa_equals_na_on_zero_padded_input(oracle, H, W, ks):
    g = rng(300 + ks)
    B, Hh, D, r = 2, 2, 4, ks // 2
    q, k, v = (g.standard_normal((B, Hh, H, W, D)) for _ in range(3))
    rpb = 0.5 * g.standard_normal((Hh, 2 * ks - 1, 2 * ks - 1))
    scale = 0.37
    pad = lambda t: np.pad(t, ((0, 0), (0, 0), (r, r), (r, r), (0, 0)))
    na_out = oracle.fwd(pad(q), pad(k), pad(v), rpb, scale, ks)[:, :, r:r + H, r:r + W]
    # a centred window uses the central ks x ks block of the relative bias table
    want = sasa_brute_force(q, k, v, rpb[:, r:r + ks, r:r + ks], scale, ks)
    np.testing.assert_allclose(na_out, want, rtol=1e-12, atol=1e-13)
