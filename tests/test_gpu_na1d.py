"""GPU parity of the 1D entry points (through the C ABI) against the fp64 1D oracle on the same seeded
inputs: every stage element by element with the oracle stage fed what the GPU stored as that stage's
input, the fused forward end to end.  Tolerances as in gpu_util.py (fp32 rel 1e-5 with an rms floor;
16-bit 2e-3 + half an ulp of the storage type; bias gradient 1e-4 of its largest entry)."""
import numpy as np
import pytest
import torch

from oracle import na1d_oracle as o1
from paper_2204_07143_amd import binding as na
from paper_2204_07143_amd import synth

from gpu_util import assert_close, assert_close_rpb, to_np

pytestmark = pytest.mark.gpu


def run_1d(p: synth.Problem1D, seed: int, planes=None, use_rpb=True, scale=None, rpb_std=0.02):
    host = synth.make_inputs_1d(p, seed, rpb_std=rpb_std)
    k, dt = p.k, p.dtype
    scale = p.default_scale if scale is None else scale
    td = synth.TORCH_DTYPES[dt]
    dev = lambda n: synth.to_device(host[n], dt)
    q, key, v, dout = dev("q"), dev("k"), dev("v"), dev("dout")
    rpb = dev("rpb") if use_rpb else None
    attn_like = lambda: torch.empty((p.B, p.heads, p.L, k), dtype=td, device="cuda")
    logits = na.na1d_qk_rpb(q, key, rpb, scale, k, attn_like())
    attn = na.na1d_softmax(logits, k, q, attn_like())
    out = na.na1d_av(attn, v, k, torch.empty_like(q))
    lse = torch.empty((p.B, p.heads, p.L), dtype=torch.float32, device="cuda")
    out_f = na.na1d_fused_fwd(q, key, v, rpb, scale, k, torch.empty_like(q), lse)
    out_f2 = na.na1d_fused_fwd(q, key, v, rpb, scale, k, torch.empty_like(q), None)
    dp = na.na1d_av_bwd_p(dout, v, k, attn_like())
    dv = na.na1d_av_bwd_v(attn, dout, k, torch.empty_like(q))
    ds = na.na1d_softmax_bwd(attn, dp, k, q, attn_like())
    dq = na.na1d_qk_bwd_q(ds, key, scale, k, torch.empty_like(q))
    dk = na.na1d_qk_bwd_k(ds, q, scale, k, torch.empty_like(q))
    prob = na.problem_1d(p.B, p.heads, p.L, p.D, k, td)
    ws = torch.empty(na.na1d_workspace_bytes(prob), dtype=torch.uint8, device="cuda")
    d_rpb = na.na1d_qk_bwd_rpb(ds, k, q, torch.empty((p.heads, 2 * k - 1), dtype=torch.float32, device="cuda"), ws)
    d_rpb2 = na.na1d_qk_bwd_rpb(ds, k, q, torch.empty((p.heads, 2 * k - 1), dtype=torch.float32, device="cuda"), ws)
    # in-place forms: softmax over its input, softmax backward over dp
    logits_c, dp_c = logits.clone(), dp.clone()
    na.na1d_softmax(logits_c, k, q, logits_c)
    na.na1d_softmax_bwd(attn, dp_c, k, q, dp_c)
    torch.cuda.synchronize()
    assert torch.equal(logits_c, attn) and torch.equal(dp_c, ds)
    assert torch.equal(out_f, out_f2) and torch.equal(d_rpb, d_rpb2)
    # fused backward (from the fused forward's lse): everything is computed in fp32 from the inputs, so it is
    # compared with the all-double oracle; a run without the bias gradient and a repeat give the same bits
    ws_f = torch.empty(na.na1d_fused_bwd_workspace_bytes(prob), dtype=torch.uint8, device="cuda")
    fdq, fdk, fdv = (torch.empty_like(q) for _ in range(3))
    fd_rpb = torch.empty((p.heads, 2 * k - 1), dtype=torch.float32, device="cuda")
    na.na1d_fused_bwd(q, key, v, rpb, scale, lse, dout, k, fdq, fdk, fdv, fd_rpb, ws_f)
    fdq2, fdk2, fdv2 = (torch.empty_like(q) for _ in range(3))
    na.na1d_fused_bwd(q, key, v, rpb, scale, lse, dout, k, fdq2, fdk2, fdv2, None, ws_f)
    fdq3, fdk3, fdv3, fd_rpb3 = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), torch.empty_like(fd_rpb)
    na.na1d_fused_bwd(q, key, v, rpb, scale, lse, dout, k, fdq3, fdk3, fdv3, fd_rpb3, ws_f)
    torch.cuda.synchronize()
    assert torch.equal(fdq, fdq2) and torch.equal(fdk, fdk2) and torch.equal(fdv, fdv2)
    assert torch.equal(fdq, fdq3) and torch.equal(fdk, fdk3) and torch.equal(fdv, fdv3) and torch.equal(fd_rpb, fd_rpb3)

    if planes is None:
        planes = [(b, h) for b in range(p.B) for h in range(p.heads)]
    for (b, h) in planes:
        sl = lambda x: x[b:b + 1, h:h + 1]
        f64 = lambda n: sl(host[n]).astype(np.float64)
        tag = f"1d plane({b},{h})"
        r = host["rpb"][h:h + 1].astype(np.float64) if use_rpb else None
        assert_close(f"{tag} logits", sl(logits), o1.qk_rpb(f64("q"), f64("k"), r, scale, k), dt)
        assert_close(f"{tag} softmax", sl(attn), o1.softmax(to_np(sl(logits))), dt)
        assert_close(f"{tag} av", sl(out), o1.av(to_np(sl(attn)), f64("v"), k), dt)
        o_out, o_lse = o1.fwd(f64("q"), f64("k"), f64("v"), r, scale, k, return_lse=True)
        assert_close(f"{tag} fused", sl(out_f), o_out, dt)
        assert_close(f"{tag} lse", sl(lse), o_lse, "f32")
        if dt != "bf16":
            assert_close(f"{tag} unfused chain", sl(out), o_out, dt)
        assert_close(f"{tag} grad-a", sl(dp), o1.av_bwd_p(f64("dout"), f64("v"), k), dt)
        assert_close(f"{tag} grad-v", sl(dv), o1.av_bwd_v(to_np(sl(attn)), f64("dout"), k), dt)
        assert_close(f"{tag} softmax-bwd", sl(ds), o1.softmax_bwd(to_np(sl(attn)), to_np(sl(dp))), dt)
        assert_close(f"{tag} grad-q", sl(dq), o1.qk_bwd_q(to_np(sl(ds)), f64("k"), scale, k), dt)
        assert_close(f"{tag} grad-k", sl(dk), o1.qk_bwd_k(to_np(sl(ds)), f64("q"), scale, k), dt)
        o_dq, o_dk, o_dv, _ = o1.bwd(f64("q"), f64("k"), f64("v"), r, scale, f64("dout"), k)
        assert_close(f"{tag} fused dq", sl(fdq), o_dq, dt)
        assert_close(f"{tag} fused dk", sl(fdk), o_dk, dt)
        assert_close(f"{tag} fused dv", sl(fdv), o_dv, dt)
    assert_close_rpb("1d grad-b", d_rpb, o1.qk_bwd_rpb(to_np(ds), k))
    # the bias gradient sums over the batch: the whole tensors (a table of zeros stands in where there is no bias)
    h64 = {n: host[n].astype(np.float64) for n in ("q", "k", "v", "dout")}
    rpb_all = host["rpb"].astype(np.float64) if use_rpb else np.zeros_like(host["rpb"], dtype=np.float64)
    want_b = o1.bwd(h64["q"], h64["k"], h64["v"], rpb_all, scale, h64["dout"], k)[3]
    assert_close_rpb("1d fused grad-b", fd_rpb, want_b)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("L,k", [(300, 3), (777, 7), (515, 13), (600, 31), (263, 33), (450, 63)])
def test_1d_small_ragged_all_elements(dtype, L, k):
    """Several tiles and a ragged last tile, every window size class, every element."""
    run_1d(synth.Problem1D(2, 3, L, 32, k, dtype), seed=8000 + L + k)


@pytest.mark.parametrize("L,k", [(3, 3), (7, 7), (9, 7), (63, 63), (64, 63), (256, 5), (257, 5), (128, 33), (129, 33), (31, 31)])
def test_1d_degenerate_lengths(L, k):
    """k = L (self attention), L just above k (every query at an end), exact and one-over tile multiples."""
    run_1d(synth.Problem1D(3, 2, L, 32, k, "f16"), seed=8100 + L + k)
    run_1d(synth.Problem1D(1, 1, L, 32, k, "f32"), seed=8200 + L + k)


def test_1d_no_bias_custom_scale_large_bias():
    run_1d(synth.Problem1D(2, 2, 400, 32, 9, "f16"), seed=8300, use_rpb=False, scale=0.3)
    run_1d(synth.Problem1D(2, 2, 400, 32, 9, "bf16"), seed=8301, rpb_std=1.5)
    run_1d(synth.Problem1D(2, 2, 400, 32, 9, "f32"), seed=8302, rpb_std=1.5, scale=0.05)


@pytest.mark.parametrize("name", list(synth.CONFIGS_1D))
def test_1d_full_size_sampled_planes(name):
    """The benchmark shapes in the launch configuration bench.py times: four sampled planes element by element,
    the bias gradient (a sum over everything) on the whole tensor."""
    p = synth.CONFIGS_1D[name]
    run_1d(p, seed=8400, planes=[(0, 0), (17, 1), (p.B - 1, 0), (p.B // 2, p.heads - 1)])
