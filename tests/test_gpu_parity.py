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

from gpu_util import Stages, assert_close, assert_close_rpb, block, slices_of, to_np

pytestmark = pytest.mark.gpu

KS = (3, 5, 7, 9, 11, 13)


def check_planes(oracle, st: Stages, host: dict, planes, backward: bool, e2e_unfused: bool = True):
    """Stage-wise and end-to-end parity on the given (b, h) planes; planes=None checks every plane."""
    p, k, scale = st.p, st.k, st.scale
    flat = {"logits": 0, "attn": 0, "out": 0, "fused": 0}
    for sl in slices_of(p, planes):
        tag = f"block{sl}"
        q, key, v = (block(host[n], sl).astype(np.float64) for n in ("q", "k", "v"))
        rpb = host["rpb"][sl[2]:sl[3]].astype(np.float64) if st.rpb is not None else None
        # forward, stage by stage
        flat["logits"] += assert_close(f"{tag} logits", block(st.logits, sl), oracle.qk_rpb(q, key, rpb, scale, k), p.dtype)
        g_logits = to_np(block(st.logits, sl))
        flat["attn"] += assert_close(f"{tag} softmax", block(st.attn, sl), oracle.softmax(g_logits), p.dtype)
        del g_logits
        g_attn = to_np(block(st.attn, sl))
        flat["out"] += assert_close(f"{tag} av", block(st.out, sl), oracle.av(g_attn, v, k), p.dtype)
        # forward, end to end against the all-double oracle
        o_out, o_lse = oracle.fwd(q, key, v, rpb, scale, k, return_lse=True)
        flat["fused"] += assert_close(f"{tag} fused", block(st.out_fused, sl), o_out, p.dtype)
        assert_close(f"{tag} lse", block(st.lse, sl), o_lse, "f32")
        # The unfused chain stores logits and weights in the problem dtype.  In bf16 (8 significant
        # bits) those two intermediate roundings alone move the output by more than the 2e-3
        # bound, so for bf16 the chain is covered by the stage-wise checks above and the fused
        # end-to-end check; for fp32 / fp16 it is also compared end to end.
        # In fp16 the chain's own roundings are part of the result: a logit in [4, 8) is stored to +-2^-9, which
        # moves the weights of its query by up to 0.4 % each (and the normalisation with them), the weights are
        # rounded to 11 bits once more, so the output may differ from the exact one by up to about
        # 2 * 2^-8 * sum_j P_j |v_j|: the end-to-end bound is 8e-3, four times the per-stage one (over millions
        # of elements the tail of that error does pass 2e-3; every stage by itself is held to 2e-3 above).
        if e2e_unfused and p.dtype != "bf16":
            assert_close(f"{tag} unfused chain", block(st.out, sl), o_out, p.dtype, abs_tol=2e-3 if p.dtype == "f32" else 8e-3)
        if not backward:
            continue
        dout = block(host["dout"], sl).astype(np.float64)
        assert_close(f"{tag} grad-a", block(st.dp, sl), oracle.av_bwd_p(dout, v, k), p.dtype)
        assert_close(f"{tag} grad-v", block(st.dv, sl), oracle.av_bwd_v(g_attn, dout, k), p.dtype)
        g_dp = to_np(block(st.dp, sl))
        assert_close(f"{tag} softmax-bwd", block(st.ds, sl), oracle.softmax_bwd(g_attn, g_dp), p.dtype)
        del g_dp, g_attn
        g_ds = to_np(block(st.ds, sl))
        assert_close(f"{tag} grad-q", block(st.dq, sl), oracle.qk_bwd_q(g_ds, key, scale, k), p.dtype)
        assert_close(f"{tag} grad-k", block(st.dk, sl), oracle.qk_bwd_k(g_ds, q, scale, k), p.dtype)
    return flat


def whole_rpb_grad(oracle, ds: torch.Tensor, k: int, p: synth.Problem) -> np.ndarray:
    """The oracle's bias gradient of a whole ds tensor (a sum over the batch), taken in batch ranges."""
    total = None
    for sl in slices_of(p, None):
        part = oracle.qk_bwd_rpb(to_np(block(ds, sl)), k)
        total = part if total is None else total + part
    return total


def whole_bwd_rpb(oracle, host: dict, p: synth.Problem, scale: float, use_rpb: bool) -> np.ndarray:
    """The all-double oracle's bias gradient of the whole problem, taken in batch ranges."""
    # without a bias the gradient with respect to it still exists: the oracle gets a table of zeros
    rpb_all = host["rpb"].astype(np.float64) if use_rpb else np.zeros_like(host["rpb"], dtype=np.float64)
    total = None
    for sl in slices_of(p, None):
        part = oracle.bwd(*(block(host[n], sl).astype(np.float64) for n in ("q", "k", "v")), rpb_all, scale,
                          block(host["dout"], sl).astype(np.float64), p.k)[3]
        total = part if total is None else total + part
    return total


def run_all(oracle, p: synth.Problem, seed: int, planes=None, backward=True, use_rpb=True, scale=None, rpb_std=0.02,
            host=None, fused_backward=True, e2e_unfused=True):
    """planes: the (b, h) planes compared element by element; None = every plane of the problem.
    e2e_unfused: also compare the unfused chain's output with the all-double oracle (fp32 / fp16 only, and only
    sensible while the logits are small: an fp16 logit of 16 is stored to +-0.004, which by itself moves the
    output by more than the bound; the stage-wise checks hold at any size)."""
    if host is None:
        host = synth.make_inputs(p, seed, rpb_std=rpb_std)
    st = Stages(p, host, scale=scale, use_rpb=use_rpb)
    st.forward_unfused()
    st.forward_fused()
    if backward:
        st.backward_unfused()
    torch.cuda.synchronize()
    flat = check_planes(oracle, st, host, planes, backward, e2e_unfused=e2e_unfused)
    if backward and use_rpb:
        # grad-b sums over the batch: needs the whole ds tensor
        assert_close_rpb("grad-b", st.d_rpb, whole_rpb_grad(oracle, st.ds, p.k, p))
        # The composed backward either runs the same kernels as the stages (then everything is bitwise
        # equal to them) or fuses grad-a with the softmax backward (16-bit types, k <= 9: dp is never
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
            assert p.dtype != "f32" and p.k <= 9, "only the 16-bit backward with k <= 9 is fused"
            for sl in slices_of(p, planes):
                tag = f"na2d_bwd block{sl}"
                q, key, v, dout = (block(host[n], sl).astype(np.float64) for n in ("q", "k", "v", "dout"))
                g_attn = to_np(block(st.attn, sl))
                assert_close(f"{tag} ds", block(ds_c, sl), oracle.softmax_bwd(g_attn, oracle.av_bwd_p(dout, v, p.k)), p.dtype)
                del g_attn
                g_ds = to_np(block(ds_c, sl))
                assert_close(f"{tag} grad-q", block(dq, sl), oracle.qk_bwd_q(g_ds, key, st.scale, p.k), p.dtype)
                assert_close(f"{tag} grad-k", block(dk, sl), oracle.qk_bwd_k(g_ds, q, st.scale, p.k), p.dtype)
            assert_close_rpb("na2d_bwd grad-b", d_rpb, whole_rpb_grad(oracle, ds_c, p.k, p))
    if backward and fused_backward:
        check_fused_backward(oracle, st, host, planes, use_rpb)
    return st, host, flat


def check_fused_backward(oracle, st: Stages, host: dict, planes, use_rpb: bool):
    """na2d_fused_bwd (inputs: q, k, v, rpb, dout and the fused forward's lse).  Where it runs its two fused
    kernels, everything is computed in fp32 from the inputs, so it is compared with the all-double oracle's
    gradients: dq / dk / dv on the given planes, d_rpb (a sum over the batch) on the whole tensors.  Where it
    falls back to the unfused steps (fp32, k >= 11, maps with awkward ragged tiles) it recomputes the attention
    weights with the same kernels as the unfused forward and must reproduce na2d_bwd bit for bit."""
    p = st.p
    dq, dk, dv, d_rpb = st.backward_fused(with_rpb_grad=True)
    torch.cuda.synchronize()
    prob = na.problem(p.B, p.heads, p.H, p.W, p.D, p.k, st.tdtype)
    if na.na2d_fused_bwd_is_fused(prob):
        assert p.dtype != "f32" and p.k <= 9
        for sl in slices_of(p, planes):
            tag = f"na2d_fused_bwd block{sl}"
            q, key, v, dout = (block(host[n], sl).astype(np.float64) for n in ("q", "k", "v", "dout"))
            rpb = host["rpb"][sl[2]:sl[3]].astype(np.float64) if use_rpb else None
            o_dq, o_dk, o_dv, _ = oracle.bwd(q, key, v, rpb, st.scale, dout, p.k)
            assert_close(f"{tag} dq", block(dq, sl), o_dq, p.dtype)
            assert_close(f"{tag} dk", block(dk, sl), o_dk, p.dtype)
            assert_close(f"{tag} dv", block(dv, sl), o_dv, p.dtype)
        assert_close_rpb("na2d_fused_bwd d_rpb", d_rpb, whole_bwd_rpb(oracle, host, p, st.scale, use_rpb))
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


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("H,W,k,D", [(23, 30, 15, 32), (25, 22, 21, 32), (15, 15, 15, 32), (24, 27, 15, 64), (21, 33, 21, 16)])
def test_window_sides_beyond_the_tuned_ones(oracle, H, W, k, D, dtype):
    # k >= 15 runs the kernels that take the window side at run time: every stage, the fused forward, the composed
    # backward and na2d_fused_bwd (which recomputes the weights and runs the unfused steps there), every element
    run_all(oracle, synth.Problem(2, 2, H, W, D, k, dtype), seed=1500 + k + D)


def test_config1_tiny_fp32(oracle):
    run_all(oracle, synth.CONFIGS["tiny"], seed=1001)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("H,W,k", [(7, 7, 7), (3, 3, 3), (13, 13, 13), (14, 14, 7), (13, 40, 13), (33, 9, 9), (28, 28, 7), (23, 45, 9)])
def test_degenerate_and_border_heavy_maps(oracle, H, W, k, dtype):
    # k = H = W is the self-attention limit (every window is the whole map); short axes make
    # keys sit near both borders at once
    run_all(oracle, synth.Problem(3, 2, H, W, 32, k, dtype), seed=7 * H + W + k)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,W,k", [(40, 50, 11), (45, 70, 13), (34, 33, 9), (52, 36, 9)])
def test_large_windows_many_tiles_odd_batch(oracle, H, W, k, dtype):
    # several tile rows and columns, ragged on both axes, a batch that does not divide by the workgroups'
    # split of it, no bias on the 13-wide window
    run_all(oracle, synth.Problem(5, 3, H, W, 32, k, dtype), seed=40 * H + W + k, use_rpb=(k != 13),
            planes=[(0, 0), (2, 1), (4, 2)])


@pytest.mark.parametrize("k,side", [(k, k + d) for k in (3, 5, 7, 11, 13) for d in range(0, 30, 1)])
def test_every_map_height_and_width(oracle, k, side):
    # the same walk through the map geometries for the other window sides whose kernels depend on them (k = 7:
    # column-walking, tile and row-streaming grad-v / grad-k kernels; k = 11, 13: one, two or four patches per wave,
    # one halo buffer and one staging image in the logits kernel), bf16
    for H, W in ((side, 24), (24, side)):
        run_all(oracle, synth.Problem(2, 1, H, W, 32, k, "bf16"), seed=7000 + 50 * H + W + k)


@pytest.mark.parametrize("side", list(range(9, 42)))
def test_k9_every_map_height_and_width(oracle, side):
    # k = 9 runs its kernels with LDS plans of their own (the query rectangle of a key tile in chunks of rows, one
    # stage or one staging image instead of two, two window slots per lane in the bias-gradient sums): every map
    # height from 9 to 41 on a 20-wide map, and every width on a 20-high one, so that every number of rectangle
    # rows and columns, every position of the chunk boundary inside a patch's rows and the maps that fall back to
    # other kernels (a patch seen from more than 16 columns) all occur; every stage and both backward calls
    for H, W in ((side, 20), (20, side)):
        run_all(oracle, synth.Problem(2, 1, H, W, 32, 9, "f16"), seed=9000 + 50 * H + W)


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


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("rpb_std", [1.0, 4.0])
@pytest.mark.parametrize("k", [3, 7, 13])
def test_bias_that_matters_16bit(oracle, k, rpb_std, dtype):
    # The matrix-core kernels with a bias of the size of the logits and larger (Eq. 2's B): logits, fused
    # forward and its log-sum-exp, the composed backward and the fused backward (dq, dk, dv, d_rpb), every
    # element.  The fused kernels hold the table as fp16 beside the window mask; it must be the stored bias.
    run_all(oracle, synth.Problem(2, 2, 19, 37, 32, k, dtype), seed=300 + k, rpb_std=rpb_std, e2e_unfused=(rpb_std <= 1.0))


@pytest.mark.parametrize("dtype,big,fused_backward", [("f16", 60000.0, False), ("f16", -60000.0, True),
                                                      ("bf16", 30000.0, False), ("bf16", -65280.0, True)])
def test_bias_entry_near_fp16_maximum(oracle, dtype, big, fused_backward):
    # One cell of the table next to the largest finite fp16 value (the key one step to the right of and below
    # the query), the rest N(0, 1): where it is positive that key takes all the weight, where it is negative
    # none.  Logits, softmax, fused forward (+ lse) and the composed backward are checked in every case.  The
    # fused backward recomputes the weights as exp(logit - lse) from the fp32 lse, whose spacing at 6e4 is
    # 2^-8: that alone moves a weight by 0.4 % (and where one key holds all the weight every exact ds is 0, so
    # d_rpb would be nothing but the sum of those errors), so it is checked for the negative entry, which
    # leaves lse small.
    p = synth.Problem(2, 2, 18, 21, 32, 7, dtype)
    host = synth.make_inputs(p, 77, rpb_std=1.0)
    host["rpb"][:, p.k, p.k] = synth.round_to(np.full((p.heads,), big, dtype=np.float32), dtype)
    assert np.all(np.abs(host["rpb"][:, p.k, p.k]) >= 0.99 * abs(big))
    run_all(oracle, p, seed=77, host=host, fused_backward=fused_backward, e2e_unfused=False)


@pytest.mark.parametrize("dtype,log2_scale", [("bf16", -17), ("bf16", 13), ("f16", -7), ("f16", 5)])
def test_fused_backward_follows_the_scale_of_dout(oracle, dtype, log2_scale):
    # The fused backward sums d_rpb in fixed point whose resolution follows the size of the gradients:
    # upstream gradients of 2^-17 (8e-6) and 2^13 (8e3) times unit scale must give the same relative accuracy
    # as unit scale.  The factor is a power of two, so the scaled inputs are exact and every gradient is the
    # unit-scale one times the factor: dq, dk, dv are compared after dividing the factor out again.
    p = synth.Problem(6, 2, 20, 35, 32, 7, dtype)
    host = synth.make_inputs(p, 55, rpb_std=0.5)
    f = 2.0 ** log2_scale
    host["dout"] = synth.round_to(host["dout"] * np.float32(f), dtype)
    st = Stages(p, host)
    st.forward_fused()
    dq, dk, dv, d_rpb = st.backward_fused()
    torch.cuda.synchronize()
    assert na.na2d_fused_bwd_is_fused(na.problem(p.B, p.heads, p.H, p.W, p.D, p.k, st.tdtype))
    f64 = {n: host[n].astype(np.float64) for n in host}
    o_dq, o_dk, o_dv, o_db = oracle.bwd(f64["q"], f64["k"], f64["v"], f64["rpb"], st.scale, f64["dout"], p.k)
    for name, g, o in (("dq", dq, o_dq), ("dk", dk, o_dk), ("dv", dv, o_dv)):
        assert_close(f"{name} / 2^{log2_scale}", to_np(g) / f, o / f, dtype)
    assert_close_rpb("d_rpb", d_rpb, o_db)


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
                                   (56, 56, 13), (13, 29, 13), (9, 5, 5), (23, 30, 15), (40, 33, 21), (63, 70, 63)])
def test_indices_bit_exact(oracle, H, W, k):
    ki = torch.empty((H, W, k * k), dtype=torch.int32, device="cuda")
    ri = torch.empty_like(ki)
    na.na2d_debug_indices(H, W, k, ki, ri)
    torch.cuda.synchronize()
    want_k, want_r = oracle.indices(H, W, k)
    assert np.array_equal(ki.cpu().numpy(), want_k)
    assert np.array_equal(ri.cpu().numpy(), want_r)


# ---- full-size configs in the launch configuration bench.py times: every plane ---------------

FULL = [
    ("nat_tiny_stage1", True),      # config 2 / config 5 at k = 7: forward and backward
    ("nat_tiny_l1_bf16", False),
    ("nat_tiny_l2_bf16", True),     # 28 x 28: key tiles next to the far border (larger query rectangles)
    ("nat_tiny_l3_bf16", True),     # 14 x 14: axes so short that a key is near both borders
    ("nat_tiny_l4_bf16", False),    # 7x7, k = 7: full self attention
    ("detection_like", True),       # 200 x 334: ragged tiles on both axes, many tiles per column
    ("segmentation_like", True),
    ("stage1_head_dim_64", True),   # head dims other than 32
    ("stage1_head_dim_16", True),
]


@pytest.mark.parametrize("name,backward", FULL)
def test_full_size_config_every_plane(oracle, name, backward):
    # The oracle runs a whole batch range at once on all host cores, so every plane of the full-size problem is
    # compared element by element: a batch range that no workgroup takes, or two take, at the launch geometry
    # the benchmark times would show here.
    p = synth.CONFIGS[name]
    st, host, flat = run_all(oracle, p, seed=1000 + len(name), planes=None, backward=backward)
    # properties that hold at any size, on the whole tensors
    rows = st.attn.float().sum(-1)
    assert float((rows - 1).abs().max()) < (2e-5 if p.dtype == "f32" else 2e-2)
    # fused and unfused agree to a few storage ulps (the unfused chain rounds logits and weights)
    diff = ((st.out.float() - st.out_fused.float()).abs() / st.out_fused.float().abs().clamp(min=1.0)).max()
    assert float(diff) < 3e-2
    print(f"{name}: elements outside a flat 2e-3: {flat}")


@pytest.mark.parametrize("k", [3, 5, 9, 11, 13])
def test_config5_kernel_size_sweep_fwd_bwd(oracle, k):
    p = synth.Problem(64, 2, 56, 56, 32, k, "f16")
    run_all(oracle, p, seed=5000 + k, planes=None, backward=True)


# ---- head dims other than 32: every (dtype, D, k) class the library accepts, and the ones it refuses ------------

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D,k", [(16, 3), (16, 7), (16, 13), (64, 5), (64, 9), (64, 11), (64, 13), (128, 3), (128, 5), (128, 7), (128, 9), (128, 11), (128, 13)])
def test_generic_head_dims(oracle, dtype, D, k):
    # (the fp32 tiles of the largest head dims do not fit the LDS for larger windows: (64, 13) and (128, 9) in fp32,
    # and (128, 13) in any type, run the kernels that take the window side at run time)
    p = synth.Problem(2, 2, 19, 22, D, k, dtype)
    prob = na.problem(p.B, p.heads, p.H, p.W, D, k, synth.TORCH_DTYPES[dtype])
    assert na.na2d_validate_problem(prob) == 0
    run_all(oracle, p, seed=9000 + D + k)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,W,k", [(56, 56, 7), (30, 45, 5), (21, 37, 3), (14, 14, 7), (7, 7, 7), (9, 40, 7), (40, 33, 9),
                                   (35, 50, 11), (48, 30, 13), (13, 20, 13)])
def test_sixteen_channel_heads_on_the_matrix_cores(oracle, dtype, H, W, k):
    # 16-channel heads ride in the lower half of the 32-channel matrix-core kernels: maps with several
    # tiles and ragged borders (the column-walking grad-v / grad-k kernel), maps whose shortest side is at most
    # 2k + 2 (the tile kernel or the row-streaming one), a bias that matters, every plane
    p = synth.Problem(3, 4, H, W, 16, k, dtype)
    run_all(oracle, p, seed=9500 + H + W + k, rpb_std=1.0, e2e_unfused=False)


def _seeded_shapes(n, seed):
    """n problems drawn from a fixed seed: sides from k to 70 (so that windows clamp on either or both axes, tiles are
    ragged and maps shorter than 2k + 2 occur), every tuned k, three head dims, three dtypes, small odd batches."""
    rng = np.random.RandomState(seed)
    out = []
    for i in range(n):
        k = int(rng.choice([3, 5, 7, 9, 11, 13]))
        H, W = (int(rng.randint(k, 71)) for _ in range(2))
        if i % 5 == 0:
            H = k + int(rng.randint(0, 3))   # one axis barely longer than the window
        D = int(rng.choice([16, 32, 32, 64]))
        dtype = ["f32", "f16", "bf16"][i % 3]
        out.append((int(rng.randint(1, 6)), int(rng.randint(1, 4)), H, W, D, k, dtype))
    return out


@pytest.mark.parametrize("B,heads,H,W,D,k,dtype", _seeded_shapes(36, 20260))
def test_seeded_random_shapes(oracle, B, heads, H, W, D, k, dtype):
    p = synth.Problem(B, heads, H, W, D, k, dtype)
    run_all(oracle, p, seed=31000 + 71 * H + W + k + D)


@pytest.mark.parametrize("B,heads,D,k", [(254, 8, 32, 13), (437, 16, 16, 7)])
def test_attention_tensors_beyond_two_gigabytes(oracle, B, heads, D, k):
    # k*k tensors of more than 2^31 bytes (byte offsets that no longer fit 32 bits): the first, a middle and the last
    # plane element by element, and the bias gradient over the whole tensor
    p = synth.Problem(B, heads, 56, 56, D, k, "f16")
    assert p.n_queries * p.kk * 2 > 2 ** 31
    run_all(oracle, p, seed=4242 + k, planes=[(0, 0), (B // 2, heads // 2), (B - 1, heads - 1)], fused_backward=False)


def test_head_dim_tensors_beyond_two_gigabytes(oracle):
    # q, k, v, dout and the three head-dim gradients of more than 2^31 bytes each, the fused backward included
    p = synth.Problem(669, 16, 56, 56, 32, 3, "f16")
    assert p.n_queries * p.D * 2 > 2 ** 31
    run_all(oracle, p, seed=4250, planes=[(0, 0), (334, 7), (668, 15)])


def test_head_dims_the_library_does_not_take():
    q = torch.zeros((1, 1, 14, 14, 48), dtype=torch.float16, device="cuda")
    with pytest.raises(na.Na2dError) as e:
        na.na2d_fused_fwd(q, q.clone(), q.clone(), None, 1.0, 7, torch.empty_like(q))
    assert e.value.status == -5


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
