"""The entry point that allocates nothing: na2d_qk_bwd_rpb_noalloc keeps its partial sums in a device array
that is part of the library, so it must give the bits of na2d_qk_bwd_rpb (same kernels, same order of
additions), on every call, whatever an earlier call left in the array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2204_07143_amd import binding as na
from paper_2204_07143_amd import synth

from gpu_util import assert_close_rpb, to_np


def _ds(p: synth.Problem, seed: int) -> torch.Tensor:
    g = np.random.default_rng(seed)
    x = synth.round_to(g.standard_normal((p.B, p.heads, p.H, p.W, p.kk), dtype=np.float32), p.dtype)
    return synth.to_device(x, p.dtype)


def _both(p: synth.Problem, ds: torch.Tensor):
    like = torch.empty((p.B, p.heads, p.H, p.W, p.D), dtype=ds.dtype, device="cuda")
    nb = 2 * p.k - 1
    prob = na.problem(p.B, p.heads, p.H, p.W, p.D, p.k, ds.dtype)
    ws = torch.empty(na.na2d_workspace_bytes(prob, na.WS_QK_BWD_RPB), dtype=torch.uint8, device="cuda")
    want = na.na2d_qk_bwd_rpb(ds, p.k, like, torch.empty((p.heads, nb, nb), dtype=torch.float32, device="cuda"), ws)
    got = na.na2d_qk_bwd_rpb_noalloc(ds, p.k, like, torch.full((p.heads, nb, nb), float("nan"), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    return got, want


@pytest.mark.gpu
def test_two_calls_in_a_row_second_one_smaller(oracle):
    # a large problem first (it fills most of what the array ever holds), then a smaller one with another window
    # and dtype: the second result must not see anything the first left behind
    big = synth.Problem(24, 3, 40, 52, 32, 9, "f16")
    small = synth.Problem(3, 2, 17, 21, 32, 5, "bf16")
    for p, seed in ((big, 1), (small, 2)):
        ds = _ds(p, seed)
        got, want = _both(p, ds)
        assert torch.equal(got, want), f"{p}: differs from na2d_qk_bwd_rpb"
        assert_close_rpb(f"{p} d_rpb", got, oracle.qk_bwd_rpb(to_np(ds), p.k))
    # and the large one again, after the small one
    ds = _ds(big, 3)
    got, want = _both(big, ds)
    assert torch.equal(got, want)
    assert_close_rpb("big again d_rpb", got, oracle.qk_bwd_rpb(to_np(ds), big.k))


@pytest.mark.gpu
def test_fp32_and_the_bench_shape(oracle):
    for p, seed in ((synth.Problem(2, 2, 19, 37, 32, 7, "f32"), 4), (synth.CONFIGS["nat_tiny_stage1"], 5)):
        ds = _ds(p, seed)
        got, want = _both(p, ds)
        assert torch.equal(got, want)
    total = None
    for b0 in range(0, p.B, 16):
        part = oracle.qk_bwd_rpb(to_np(ds[b0:b0 + 16]), p.k)
        total = part if total is None else total + part
    assert_close_rpb("bench shape d_rpb", got, total)


def test_problem_beyond_the_array_is_refused_on_the_host():
    # 8192 planes at k = 13: one 625-cell partial per plane, 20 MB; refused before any HIP call (no GPU needed)
    lib = na.load()
    prob = na.problem(512, 16, 13, 13, 32, 13, torch.float16)
    assert na.na2d_validate_problem(prob) == 0
    assert na.na2d_workspace_bytes(prob, na.WS_QK_BWD_RPB) > na.NOALLOC_SCRATCH_BYTES
    fake = ctypes.c_void_p(4096)
    assert lib.na2d_qk_bwd_rpb_noalloc(ctypes.byref(prob), fake, fake, None) == -8
    # argument errors come first, as for every entry point
    assert lib.na2d_qk_bwd_rpb_noalloc(ctypes.byref(prob), None, fake, None) == -1
    assert lib.na2d_qk_bwd_rpb_noalloc(ctypes.byref(prob), ctypes.c_void_p(4100), fake, None) == -7
