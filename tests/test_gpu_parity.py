"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded
inputs.  Every stage is compared element by element with the oracle stage fed exactly what
the GPU stored as that stage's input (so storage rounding does not compound), plus
end-to-end comparisons of the fused forward and of the unfused chain against the all-double
oracle.  Tolerances: see gpu_util.py.
"""
import numpy as np
import pytest
import torch

from paper_2204_07143_amd import binding as na
from paper_2204_07143_amd import synth

from gpu_util import Stages, assert_close, assert_close_rpb, plane, to_np

pytestmark = pytest.mark.gpu

KS = (3, 5, 7, 9, 11, 13)


def check_planes(oracle, st: Stages, host: dict, planes, backward: bool, e2e_unfused: bool = True):
    """Stage-wise and end-to-end parity on the given (b, h) planes."""
    p, k, scale = st.p, st.k, st.scale
    flat = {}
    for (b, h) in planes:
        tag = f"plane({b},{h})"
        q, key, v = (plane(host[n], b, h).astype(np.float64) for n in ("q", "k", "v"))
        rpb = host["rpb"][h:h + 1].astype(np.float64) if st.rpb is not None else None
        # forward, stage by stage
        flat["logits"] = assert_close(f"{tag} logits", plane(st.logits, b, h), oracle.qk_rpb(q, key, rpb, scale, k), p.dtype)
        g_logits = to_np(plane(st.logits, b, h))
        flat["attn"] = assert_close(f"{tag} softmax", plane(st.attn, b, h), oracle.softmax(g_logits), p.dtype)
        g_attn = to_np(plane(st.attn, b, h))
        flat["out"] = assert_close(f"{tag} av", plane(st.out, b, h), oracle.av(g_attn, v, k), p.dtype)
        # forward, end to end against the all-double oracle
        o_out, o_lse = oracle.fwd(q, key, v, rpb, scale, k, return_lse=True)
        flat["fused"] = assert_close(f"{tag} fused", plane(st.out_fused, b, h), o_out, p.dtype)
        assert_close(f"{tag} lse", plane(st.lse, b, h), o_lse, "f32")
        # The unfused chain stores logits and weights in the problem dtype.  In bf16 (8 significant
        # bits) those two intermediate roundings alone move the output by more than the 2e-3
        # bound, so for bf16 the chain is covered by the stage-wise checks above and the fused
        # end-to-end check; for fp32 / fp16 it is also compared end to end.
        if e2e_unfused and p.dtype != "bf16":
            assert_close(f"{tag} unfused chain", plane(st.out, b, h), o_out, p.dtype)
        if not backward:
            continue
        dout = plane(host["dout"], b, h).astype(np.float64)
        assert_close(f"{tag} grad-a", plane(st.dp, b, h), oracle.av_bwd_p(dout, v, k), p.dtype)
        assert_close(f"{tag} grad-v", plane(st.dv, b, h), oracle.av_bwd_v(g_attn, dout, k), p.dtype)
        g_dp = to_np(plane(st.dp, b, h))
        assert_close(f"{tag} softmax-bwd", plane(st.ds, b, h), oracle.softmax_bwd(g_attn, g_dp), p.dtype)
        g_ds = to_np(plane(st.ds, b, h))
        assert_close(f"{tag} grad-q", plane(st.dq, b, h), oracle.qk_bwd_q(g_ds, key, scale, k), p.dtype)
        assert_close(f"{tag} grad-k", plane(st.dk, b, h), oracle.qk_bwd_k(g_ds, q, scale, k), p.dtype)
    return flat


def run_all(oracle, p: synth.Problem, seed: int, planes=None, backward=True, use_rpb=True, scale=None):
    host = synth.make_inputs(p, seed)
    st = Stages(p, host, scale=scale, use_rpb=use_rpb)
    st.forward_unfused()
    st.forward_fused()
    if backward:
        st.backward_unfused()
    torch.cuda.synchronize()
    if planes is None:
        planes = [(b, h) for b in range(p.B) for h in range(p.heads)]
    flat = check_planes(oracle, st, host, planes, backward)
    if backward and use_rpb:
        # grad-b sums over the batch: needs the whole ds tensor
        assert_close_rpb("grad-b", st.d_rpb, oracle.qk_bwd_rpb(to_np(st.ds), p.k))
        # The composed backward either runs the same kernels as the stages (then everything is bitwise
        # equal to them) or fuses grad-a with the softmax backward (16-bit types, k <= 7: dp is never
        # rounded to the storage type).  The fused result is checked like the stages: its ds (left in
        # the workspace) against the oracle's softmax backward of the exact dp, and grad-q / grad-k /
        # grad-b against the oracle fed that ds.  grad-v does not depend on ds: always bitwise equal.
        dq, dk, dv, d_rpb, ds_c = st.backward_composed()
        torch.cuda.synchronize()
        assert torch.equal(dv, st.dv), "na2d_bwd dv differs from the stage-by-stage result"
        if torch.equal(ds_c, st.ds):
            for a, b_, n in ((dq, st.dq, "dq"), (dk, st.dk, "dk"), (d_rpb, st.d_rpb, "d_rpb")):
                assert torch.equal(a, b_), f"na2d_bwd {n} differs from the stage-by-stage result"
        else:
            assert p.dtype != "f32" and p.k <= 7, "only the 16-bit small-window backward is fused"
            for (b, h) in planes:
                tag = f"na2d_bwd plane({b},{h})"
                q, key, v, dout = (plane(host[n], b, h).astype(np.float64) for n in ("q", "k", "v", "dout"))
                g_attn = to_np(plane(st.attn, b, h))
                assert_close(f"{tag} ds", plane(ds_c, b, h), oracle.softmax_bwd(g_attn, oracle.av_bwd_p(dout, v, p.k)), p.dtype)
                g_ds = to_np(plane(ds_c, b, h))
                assert_close(f"{tag} grad-q", plane(dq, b, h), oracle.qk_bwd_q(g_ds, key, st.scale, p.k), p.dtype)
                assert_close(f"{tag} grad-k", plane(dk, b, h), oracle.qk_bwd_k(g_ds, q, st.scale, p.k), p.dtype)
            assert_close_rpb("na2d_bwd grad-b", d_rpb, oracle.qk_bwd_rpb(to_np(ds_c), p.k))
    if backward:
        check_fused_backward(oracle, st, host, planes, use_rpb)
    return st, host, flat


def check_fused_backward(oracle, st: Stages, host: dict, planes, use_rpb: bool):
    """na2d_fused_bwd (inputs: q, k, v, rpb, dout and the fused forward's lse).  Where it runs its two fused
    kernels, everything is computed in fp32 from the inputs, so it is compared with the all-double oracle's
    gradients: dq / dk / dv on the given planes, d_rpb (a sum over the batch) on the whole tensors.  Where it
    falls back to the unfused steps (fp32, k >= 9, maps with awkward ragged tiles) it recomputes the attention
    weights with the same kernels as the unfused forward and must reproduce na2d_bwd bit for bit."""
    p = st.p
    dq, dk, dv, d_rpb = st.backward_fused(with_rpb_grad=True)
    torch.cuda.synchronize()
    prob = na.problem(p.B, p.heads, p.H, p.W, p.D, p.k, st.tdtype)
    if na.na2d_fused_bwd_is_fused(prob):
        assert p.dtype != "f32" and p.k <= 7
        for (b, h) in planes:
            tag = f"na2d_fused_bwd plane({b},{h})"
            q, key, v, dout = (plane(host[n], b, h).astype(np.float64) for n in ("q", "k", "v", "dout"))
            rpb = host["rpb"][h:h + 1].astype(np.float64) if use_rpb else None
            o_dq, o_dk, o_dv, _ = oracle.bwd(q, key, v, rpb, st.scale, dout, p.k)
            assert_close(f"{tag} dq", plane(dq, b, h), o_dq, p.dtype)
            assert_close(f"{tag} dk", plane(dk, b, h), o_dk, p.dtype)
            assert_close(f"{tag} dv", plane(dv, b, h), o_dv, p.dtype)
        # without a bias the gradient with respect to it still exists: the oracle gets a table of zeros
        rpb_all = host["rpb"].astype(np.float64) if use_rpb else np.zeros_like(host["rpb"], dtype=np.float64)
        want = oracle.bwd(*(host[n].astype(np.float64) for n in ("q", "k", "v")), rpb_all, st.scale,
                          host["dout"].astype(np.float64), p.k)[3]
        assert_close_rpb("na2d_fused_bwd d_rpb", d_rpb, want)
    else:
        c_dq, c_dk, c_dv, c_d_rpb, _ = st.backward_composed()
        torch.cuda.synchronize()
        for a, b_, n in ((dq, c_dq, "dq"), (dk, c_dk, "dk"), (dv, c_dv, "dv"), (d_rpb, c_d_rpb, "d_rpb")):
            assert torch.equal(a, b_), f"na2d_fused_bwd (unfused steps) {n} differs from na2d_bwd"
    # without the bias gradient the other three results are the same bits; a second run reproduces all four
    dq2, dk2, dv2, _ = st.backward_fused(with_rpb_grad=False)
    dq3, dk3, dv3, d_rpb3 = st.backward_fused(with_rpb_grad=True)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)
    assert torch.equal(dq, dq3) and torch.equal(dk, dk3) and torch.equal(dv, dv3) and torch.equal(d_rpb, d_rpb3)


# ---- small shapes, every element (several tiles, ragged tails, every k and dtype) -----------

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("k", KS)
def test_small_ragged_all_elements(oracle, k, dtype):
    p = synth.Problem(2, 2, 19, 37, 32, k, dtype)
    run_all(oracle, p, seed=100 + k)


def test_config1_tiny_fp32(oracle):
    run_all(oracle, synth.CONFIGS["tiny"], seed=1001)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("H,W,k", [(7, 7, 7), (3, 3, 3), (13, 13, 13), (14, 14, 7), (13, 40, 13), (33, 9, 9), (28, 28, 7), (23, 45, 9)])
def test_degenerate_and_border_heavy_maps(oracle, H, W, k, dtype):
    # k = H = W is the self-attention limit (every window is the whole map); short axes make
    # keys sit near both borders at once
    run_all(oracle, synth.Problem(3, 2, H, W, 32, k, dtype), seed=7 * H + W + k)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,W,k", [(40, 50, 11), (45, 70, 13), (34, 33, 9)])
def test_large_windows_many_tiles_odd_batch(oracle, H, W, k, dtype):
    # several tile rows and columns, ragged on both axes, a batch that does not divide by the workgroups'
    # split of it, no bias on the 13-wide window
    run_all(oracle, synth.Problem(5, 3, H, W, 32, k, dtype), seed=40 * H + W + k, use_rpb=(k != 13),
            planes=[(0, 0), (2, 1), (4, 2)])


@pytest.mark.parametrize("B,heads,H,W,k,dtype", [(40, 3, 20, 20, 7, "f16"), (37, 5, 9, 17, 5, "bf16"), (70, 1, 8, 16, 7, "f16")])
def test_batch_ranges_cover_every_plane(oracle, B, heads, H, W, k, dtype):
    # more batch items than ranges, ranges of unequal length, rotated per head by an amount that does not
    # divide their number: every plane is checked, so a plane that no workgroup takes (or two take) shows
    run_all(oracle, synth.Problem(B, heads, H, W, 32, k, dtype), seed=B + heads + H + W + k)


def test_no_bias_and_custom_scale(oracle):
    p = synth.Problem(1, 2, 20, 18, 32, 5, "f16")
    run_all(oracle, p, seed=5, use_rpb=False, scale=0.11)


def test_large_bias_values(oracle):
    # a bias that matters: N(0, 1) instead of N(0, 0.02^2)
    p = synth.Problem(1, 2, 17, 21, 32, 7, "f32")
    host = synth.make_inputs(p, 9, rpb_std=1.0)
    st = Stages(p, host)
    st.forward_unfused(); st.forward_fused(); st.backward_unfused()
    torch.cuda.synchronize()
    check_planes(oracle, st, host, [(0, 0), (0, 1)], backward=True)
    assert_close_rpb("grad-b", st.d_rpb, oracle.qk_bwd_rpb(to_np(st.ds), p.k))


def test_softmax_in_place_and_ds_in_place(oracle):
    p = synth.Problem(2, 1, 15, 16, 32, 7, "f16")
    host = synth.make_inputs(p, 3)
    st = Stages(p, host)
    st.forward_unfused(); st.backward_unfused()
    logits2 = st.logits.clone()
    na.na2d_softmax(logits2, p.k, st.q, logits2)
    dp2 = st.dp.clone()
    na.na2d_softmax_bwd(st.attn, dp2, p.k, st.q, dp2)
    torch.cuda.synchronize()
    assert torch.equal(logits2, st.attn) and torch.equal(dp2, st.ds)


# ---- neighbourhood indices: bit-exact ------------------------------------------------------

@pytest.mark.parametrize("H,W,k", [(14, 14, 3), (56, 56, 7), (28, 28, 7), (7, 7, 7), (200, 334, 7), (128, 128, 7),
                                   (56, 56, 13), (13, 29, 13), (9, 5, 5)])
def test_indices_bit_exact(oracle, H, W, k):
    ki = torch.empty((H, W, k * k), dtype=torch.int32, device="cuda")
    ri = torch.empty_like(ki)
    na.na2d_debug_indices(H, W, k, ki, ri)
    torch.cuda.synchronize()
    want_k, want_r = oracle.indices(H, W, k)
    assert np.array_equal(ki.cpu().numpy(), want_k)
    assert np.array_equal(ri.cpu().numpy(), want_r)


# ---- full-size configs in the launch configuration bench.py times: sampled planes ----------

FULL = [
    ("nat_tiny_stage1", True),      # config 2 / config 5 at k = 7: forward and backward
    ("nat_tiny_l1_bf16", False),
    ("nat_tiny_l2_bf16", True),     # 28 x 28: key tiles next to the far border (larger query rectangles)
    ("nat_tiny_l3_bf16", True),     # 14 x 14: axes so short that a key is near both borders
    ("nat_tiny_l4_bf16", False),    # 7x7, k = 7: full self attention
    ("detection_like", True),       # 200 x 334: ragged tiles on both axes, many tiles per column
    ("segmentation_like", True),
    ("stage1_head_dim_64", True),   # head dims other than 32 run the plain-ALU kernels
    ("stage1_head_dim_16", True),
]


@pytest.mark.parametrize("name,backward", FULL)
def test_full_size_config_sampled_planes(oracle, name, backward):
    p = synth.CONFIGS[name]
    g = np.random.default_rng(17)
    planes = {(0, 0), (p.B - 1, p.heads - 1)}
    while len(planes) < 3 and p.B * p.heads > 2:
        planes.add((int(g.integers(p.B)), int(g.integers(p.heads))))
    st, host, flat = run_all(oracle, p, seed=1000 + len(name), planes=sorted(planes), backward=backward)
    # properties that hold at any size, on the whole tensors
    rows = st.attn.float().sum(-1)
    assert float((rows - 1).abs().max()) < (2e-5 if p.dtype == "f32" else 2e-2)
    # fused and unfused agree to a few storage ulps (the unfused chain rounds logits and weights)
    diff = ((st.out.float() - st.out_fused.float()).abs() / st.out_fused.float().abs().clamp(min=1.0)).max()
    assert float(diff) < 3e-2
    print(f"{name}: elements outside a flat 2e-3 on sampled planes: {flat}")


@pytest.mark.parametrize("k", [3, 5, 9, 11, 13])
def test_config5_kernel_size_sweep_fwd_bwd(oracle, k):
    p = synth.Problem(64, 2, 56, 56, 32, k, "f16")
    run_all(oracle, p, seed=5000 + k, planes=[(0, 0), (63, 1)], backward=True)


# ---- head dims other than 32: every (dtype, D, k) class the library accepts, and the ones it refuses ------------

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D,k", [(16, 3), (16, 7), (16, 13), (64, 5), (64, 9), (64, 13), (128, 3), (128, 9)])
def test_generic_head_dims(oracle, dtype, D, k):
    p = synth.Problem(2, 2, 19, 22, D, k, dtype)
    prob = na.problem(p.B, p.heads, p.H, p.W, D, k, synth.TORCH_DTYPES[dtype])
    if na.na2d_validate_problem(prob) != 0:
        # the fp32 tiles of the largest head dims do not fit the LDS for larger windows: refused, never a wrong result
        assert dtype == "f32" and (D, k) in ((64, 13), (128, 9))
        q = torch.zeros((p.B, p.heads, p.H, p.W, D), dtype=torch.float32, device="cuda")
        with pytest.raises(na.Na2dError) as e:
            na.na2d_fused_fwd(q, q.clone(), q.clone(), None, 1.0, k, torch.empty_like(q))
        assert e.value.status == -5
        return
    run_all(oracle, p, seed=9000 + D + k)


def test_gather_gradients_are_bitwise_reproducible():
    p = synth.Problem(8, 2, 56, 56, 32, 7, "f16")
    host = synth.make_inputs(p, 77)
    st = Stages(p, host)
    st.forward_unfused(); st.backward_unfused()
    first = [t.clone() for t in (st.dq, st.dk, st.dv, st.d_rpb)]
    for _ in range(3):
        st.backward_unfused()
        torch.cuda.synchronize()
        for a, b in zip(first, (st.dq, st.dk, st.dv, st.d_rpb)):
            assert torch.equal(a, b)
