"""GPU tests of the differentiable wrappers (paper_2204_07143_amd.functional): the gradients autograd
returns are the library's, bit for bit, and the operator as a whole matches the fp64 oracle to the
tolerances of gpu_util.py.  Also the zero-padding route to SASA (Section 3.1) through the HIP path.
"""
import numpy as np
import pytest
import torch

from paper_2204_07143_amd import binding as na
from paper_2204_07143_amd import functional as F
from paper_2204_07143_amd import synth

from gpu_util import Stages, assert_close, assert_close_rpb, to_np

pytestmark = pytest.mark.gpu


def leaves(p, host):
    dev = lambda n: synth.to_device(host[n], p.dtype).requires_grad_(True)
    return dev("q"), dev("k"), dev("v"), dev("rpb"), synth.to_device(host["dout"], p.dtype)


@pytest.mark.parametrize("dtype,k", [("f16", 7), ("bf16", 5), ("f32", 3), ("f16", 9)])
def test_fused_operator_gradients(oracle, dtype, k):
    p = synth.Problem(2, 2, 20, 23, 32, k, dtype)
    host = synth.make_inputs(p, 7100 + k)
    q, key, v, rpb, dout = leaves(p, host)
    out = F.na2d(q, key, v, rpb, kernel_size=k)
    out.backward(dout)
    torch.cuda.synchronize()
    # the same calls made directly through the binding give the same bits
    st = Stages(p, host)
    st.forward_fused()
    dq, dk, dv, d_rpb = st.backward_fused()
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), st.out_fused)
    assert torch.equal(q.grad, dq) and torch.equal(key.grad, dk) and torch.equal(v.grad, dv)
    assert torch.equal(rpb.grad, d_rpb.to(rpb.dtype))
    # and the operator matches the oracle end to end where the backward is computed from the inputs alone
    h64 = {n: host[n].astype(np.float64) for n in host}
    o_out = oracle.fwd(h64["q"], h64["k"], h64["v"], h64["rpb"], p.default_scale, k)
    assert_close("na2d out", out, o_out, dtype)
    prob = na.problem(p.B, p.heads, p.H, p.W, p.D, k, synth.TORCH_DTYPES[dtype])
    if na.na2d_fused_bwd_is_fused(prob):
        o_dq, o_dk, o_dv, o_drpb = oracle.bwd(h64["q"], h64["k"], h64["v"], h64["rpb"], p.default_scale, h64["dout"], k)
        assert_close("na2d dq", q.grad, o_dq, dtype)
        assert_close("na2d dk", key.grad, o_dk, dtype)
        assert_close("na2d dv", v.grad, o_dv, dtype)
        assert_close_rpb("na2d d_rpb", d_rpb, o_drpb)


def test_fused_operator_without_bias_and_partial_grads():
    p = synth.Problem(1, 2, 17, 16, 32, 7, "f16")
    host = synth.make_inputs(p, 7200)
    q, key, v, _, dout = leaves(p, host)
    v2 = v.detach().clone()   # no gradient wanted for v
    out = F.na2d(q, key, v2, None, kernel_size=7, scale=0.2)
    out.backward(dout)
    torch.cuda.synchronize()
    st = Stages(p, host, scale=0.2, use_rpb=False)
    st.forward_fused()
    dq, dk, _, _ = st.backward_fused(with_rpb_grad=False)
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), st.out_fused) and torch.equal(q.grad, dq) and torch.equal(key.grad, dk)


def test_two_function_split_matches_stage_calls_and_oracle(oracle):
    """QK+RPB and AV as two differentiable functions with torch's softmax between them (fp32)."""
    k = 5
    p = synth.Problem(2, 2, 18, 21, 32, k, "f32")
    host = synth.make_inputs(p, 7300)
    q, key, v, rpb, dout = leaves(p, host)
    logits = F.na2d_qk_rpb(q, key, rpb, k)
    attn = torch.softmax(logits, dim=-1)
    out = F.na2d_av(attn, v, k)
    out.backward(dout)
    torch.cuda.synchronize()
    # gradients of the two functions are the stage kernels' outputs, bit for bit
    with torch.no_grad():
        dattn = na.na2d_av_bwd_p(dout, v, k, torch.empty_like(attn))
        dv = na.na2d_av_bwd_v(attn, dout, k, torch.empty_like(v))
    assert torch.equal(v.grad, dv)
    assert dattn.shape == attn.shape   # (grad-a itself is covered by the stage tests; torch's softmax backward follows it here)
    # end to end against the oracle: four fp32 stages in a row, each within 1e-5 of its exact result
    h64 = {n: host[n].astype(np.float64) for n in host}
    o_out = oracle.fwd(h64["q"], h64["k"], h64["v"], h64["rpb"], p.default_scale, k)
    o_dq, o_dk, o_dv, o_drpb = oracle.bwd(h64["q"], h64["k"], h64["v"], h64["rpb"], p.default_scale, h64["dout"], k)
    for name, g, o in (("out", out, o_out), ("dq", q.grad, o_dq), ("dk", key.grad, o_dk), ("dv", v.grad, o_dv)):
        err = np.abs(to_np(g) - o)
        tol = 4e-5 * np.maximum(np.abs(o), np.sqrt(np.mean(o * o)))
        assert (err <= tol).all(), f"{name}: max err / tol {np.max(err / tol):.2f}"
    assert_close_rpb("d_rpb", rpb.grad, o_drpb)
    # the convenience composition runs the library's softmax instead of torch's: same result to fp32 rounding
    with torch.no_grad():
        assert torch.allclose(F.na2d_unfused(q, key, v, rpb, k), out, rtol=2e-5, atol=2e-6)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_unfused_composition_is_library_kernels_end_to_end(oracle, dtype):
    """na2d_unfused = QK+RPB, softmax, AV with every step (and every gradient) a library call: forward and all
    four gradients are the stage kernels' outputs bit for bit, and within the bounds of the oracle's."""
    k = 7
    p = synth.Problem(2, 2, 19, 23, 32, k, dtype)
    host = synth.make_inputs(p, 7400)
    q, key, v, rpb, dout = leaves(p, host)
    out = F.na2d_unfused(q, key, v, rpb, k)
    out.backward(dout)
    torch.cuda.synchronize()
    st = Stages(p, host)
    st.forward_unfused()
    st.backward_unfused()
    torch.cuda.synchronize()
    assert torch.equal(out.detach(), st.out)
    assert torch.equal(v.grad, st.dv) and torch.equal(q.grad, st.dq) and torch.equal(key.grad, st.dk)
    assert torch.equal(rpb.grad, st.d_rpb.to(rpb.dtype))
    if dtype == "f32":
        h64 = {n: host[n].astype(np.float64) for n in host}
        o_dq, o_dk, o_dv, o_drpb = oracle.bwd(h64["q"], h64["k"], h64["v"], h64["rpb"], p.default_scale, h64["dout"], k)
        for name, g, o in (("dq", q.grad, o_dq), ("dk", key.grad, o_dk), ("dv", v.grad, o_dv)):
            err = np.abs(to_np(g) - o)
            tol = 4e-5 * np.maximum(np.abs(o), np.sqrt(np.mean(o * o)))
            assert (err <= tol).all(), f"{name}: max err / tol {np.max(err / tol):.2f}"
        assert_close_rpb("d_rpb", rpb.grad, o_drpb)


def test_1d_operator_gradients():
    from oracle import na1d_oracle as o1
    p = synth.Problem1D(2, 2, 300, 32, 9, "f16")
    host = synth.make_inputs_1d(p, 7500)
    dev = lambda n: synth.to_device(host[n], p.dtype).requires_grad_(True)
    q, key, v, rpb = dev("q"), dev("k"), dev("v"), dev("rpb")
    dout = synth.to_device(host["dout"], p.dtype)
    out = F.na1d(q, key, v, rpb, kernel_size=9)
    out.backward(dout)
    torch.cuda.synchronize()
    h = {n: host[n].astype(np.float64) for n in host}
    assert_close("na1d out", out, o1.fwd(h["q"], h["k"], h["v"], h["rpb"], p.default_scale, 9), "f16")
    o_dq, o_dk, o_dv, o_db = o1.bwd(h["q"], h["k"], h["v"], h["rpb"], p.default_scale, h["dout"], 9)
    assert_close("na1d dq", q.grad, o_dq, "f16")
    assert_close("na1d dk", key.grad, o_dk, "f16")
    assert_close("na1d dv", v.grad, o_dv, "f16")
    # the wrapper hands the fp32 bias gradient back in the bias's dtype: half an ulp of that on top
    err = np.abs(to_np(rpb.grad) - o_db)
    assert (err <= 1e-4 * np.abs(o_db).max() + np.abs(o_db) * 2.0 ** -11).all()


@pytest.mark.parametrize("dtype,ks", [("f16", 7), ("f32", 3)])
def test_sasa_through_zero_padding(dtype, ks):
    """Section 3.1: a centred sliding window with zero padding (SASA) is NA on the zero-padded map, read at the
    un-padded positions.  The expected values are a plain fp64 evaluation of the centred window."""
    B, heads, H, W, D, r = 1, 2, 9, 11, 32, ks // 2
    p = synth.Problem(B, heads, H, W, D, ks, dtype)
    host = synth.make_inputs(p, 7400 + ks, with_dout=False)
    td = synth.TORCH_DTYPES[dtype]
    pad = lambda t: torch.nn.functional.pad(torch.from_numpy(t), (0, 0, r, r, r, r)).to(td).cuda().contiguous()
    rpb = torch.from_numpy(host["rpb"]).to(td).cuda()
    out = F.na2d(pad(host["q"]), pad(host["k"]), pad(host["v"]), rpb, kernel_size=ks)[:, :, r:r + H, r:r + W]
    torch.cuda.synchronize()
    q, k, v = (host[n].astype(np.float64) for n in ("q", "k", "v"))
    bias = host["rpb"].astype(np.float64)[:, r:r + ks, r:r + ks]
    kp, vp = (np.pad(t, ((0, 0), (0, 0), (r, r), (r, r), (0, 0))) for t in (k, v))
    want = np.empty_like(q)
    for y in range(H):
        for x in range(W):
            kw = kp[:, :, y:y + ks, x:x + ks].reshape(B, heads, ks * ks, D)
            vw = vp[:, :, y:y + ks, x:x + ks].reshape(B, heads, ks * ks, D)
            s = p.default_scale * np.einsum("bhd,bhsd->bhs", q[:, :, y, x], kw) + bias.reshape(1, heads, ks * ks)
            e = np.exp(s - s.max(-1, keepdims=True))
            want[:, :, y, x] = np.einsum("bhs,bhsd->bhd", e / e.sum(-1, keepdims=True), vw)
    assert_close("sasa", out.contiguous(), want, dtype)
