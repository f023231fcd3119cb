"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, rejects bad arguments before touching HIP, and its index functions (the same
__host__ __device__ code the kernels use) agree with brute force."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_2204_07143_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="na2d.h", prefix="na2d_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_symbols()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert binding.na2d_version() >= 100
    names_1d = declared_symbols("na1d.h", "na1d_")
    assert len(names_1d) == 14
    for n in names_1d:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS_1D) == names_1d


def P(B=1, heads=1, H=14, W=14, D=32, k=3, dtype=0):
    return binding.Na2dProblem(B, heads, H, W, D, k, dtype)


@pytest.mark.parametrize("prob,code", [
    (P(), 0),
    (P(k=7, H=7, W=7), 0),
    (P(dtype=3), -2),
    (P(k=4), -3), (P(k=1), -3), (P(k=65, H=80, W=80), -3), (P(k=16, H=20, W=20), -3),
    # window sides beyond the tuned ones take the run-time-k kernels: every dtype, every head dim
    (P(k=15, H=20, W=20), 0), (P(k=63, H=63, W=70, D=128, dtype=0), 0), (P(k=21, H=20, W=30), -4), (P(k=21, H=30, W=30, D=48), -5),
    (P(k=7, H=6), -4), (P(k=7, W=5), -4),
    (P(D=64), 0), (P(D=16, k=13, H=20, W=20), 0), (P(D=128, k=9, H=20, W=20, dtype=1), 0),
    (P(D=48), -5), (P(D=8), -5), (P(D=128, k=5, H=20, W=20, dtype=0), 0), (P(D=64, k=11, H=20, W=20, dtype=0), 0),
    (P(B=0), -6), (P(H=-1), -6),
    (P(B=4096, heads=16, H=512, W=512, k=3), -6),
    # one (batch, head) plane of the attention tensor: below / beyond 2^31 bytes (offsets inside a plane are 32-bit)
    (P(B=1, heads=1, H=4096, W=4096, k=7, dtype=1), 0), (P(B=1, heads=1, H=6000, W=6000, k=7, dtype=1), -6),
    (P(B=1, heads=1, H=3000, W=3000, k=7, dtype=0), 0), (P(B=1, heads=1, H=4096, W=4096, k=7, dtype=0), -6),
])
def test_problem_validation(prob, code):
    assert binding.na2d_validate_problem(prob) == code
    assert isinstance(binding.strerror(code), str) and binding.strerror(code)


def test_entry_points_reject_bad_arguments_before_any_hip_call():
    lib = binding.load()
    good = P(k=3)
    buf = ctypes.create_string_buffer(64)
    a16 = (ctypes.addressof(buf) + 15) & ~15
    ok, off = ctypes.c_void_p(a16), ctypes.c_void_p(a16 + 4)
    # null problem / null pointers / misaligned pointers / aliasing / workspace: all host-side
    assert lib.na2d_qk_rpb(None, ok, ok, None, 1.0, ok, None) == -1
    assert lib.na2d_qk_rpb(ctypes.byref(good), None, ok, None, 1.0, ok, None) == -1
    assert lib.na2d_qk_rpb(ctypes.byref(good), ok, off, None, 1.0, ctypes.c_void_p(a16 + 16), None) == -7
    assert lib.na2d_qk_rpb(ctypes.byref(good), ok, ctypes.c_void_p(a16 + 16), None, 1.0, ok, None) == -10
    assert lib.na2d_av(ctypes.byref(P(k=4)), ok, ok, ok, None) == -3
    assert lib.na2d_softmax(ctypes.byref(P(D=24)), ok, ok, None) == -5
    assert lib.na2d_fused_fwd(ctypes.byref(P(k=7, H=5)), ok, ok, ok, None, 1.0, ok, None, None) == -4
    assert lib.na2d_qk_bwd_rpb(ctypes.byref(good), ok, ctypes.c_void_p(a16 + 16), None, 0, None) == -8
    assert lib.na2d_qk_bwd_rpb(ctypes.byref(good), ok, ctypes.c_void_p(a16 + 16), ctypes.c_void_p(a16 + 32), 8, None) == -8
    assert lib.na2d_debug_indices(ctypes.byref(good), None, None, None) == -1
    assert binding.strerror(-12345) == "unknown status"
    # fused backward: q, k, v, rpb, scale, lse, dout, dq, dk, dv, d_rpb, workspace, bytes, stream
    ptr = lambda i: ctypes.c_void_p(a16 + 16 * i)
    fb = lambda *a: lib.na2d_fused_bwd(ctypes.byref(good), *a)
    assert fb(ptr(0), ptr(0), ptr(0), None, 1.0, None, ptr(0), ptr(1), ptr(2), ptr(3), None, ptr(0), 1 << 20, None) == -1      # no lse
    assert fb(ptr(0), ptr(0), ptr(0), None, 1.0, off, ptr(0), ptr(1), ptr(2), ptr(3), None, ptr(0), 1 << 20, None) == -7       # misaligned lse
    assert fb(ptr(0), ptr(0), ptr(0), None, 1.0, ptr(0), ptr(0), ptr(0), ptr(2), ptr(3), None, ptr(0), 1 << 20, None) == -10   # dq aliases q
    assert fb(ptr(0), ptr(0), ptr(0), None, 1.0, ptr(0), ptr(0), ptr(1), ptr(1), ptr(3), None, ptr(0), 1 << 20, None) == -10   # dk aliases dq
    assert fb(ptr(0), ptr(0), ptr(0), None, 1.0, ptr(0), ptr(0), ptr(1), ptr(2), ptr(3), None, None, 1 << 20, None) == -8      # no workspace
    assert fb(ptr(0), ptr(0), ptr(0), None, 1.0, ptr(0), ptr(0), ptr(1), ptr(2), ptr(3), None, ptr(0), 16, None) == -8         # too small
    assert lib.na2d_fused_bwd(ctypes.byref(P(k=4)), ptr(0), ptr(0), ptr(0), None, 1.0, ptr(0), ptr(0), ptr(1), ptr(2), ptr(3),
                              None, ptr(0), 1 << 20, None) == -3
    assert lib.na2d_fused_bwd_is_fused(None) == -1


def test_workspace_sizes():
    p = P(B=64, heads=2, H=56, W=56, k=7, dtype=1)
    rpb = binding.na2d_workspace_bytes(p, binding.WS_QK_BWD_RPB)
    full = binding.na2d_workspace_bytes(p, binding.WS_BWD)
    assert rpb > 0 and rpb % 256 == 0
    assert full >= rpb + 64 * 2 * 56 * 56 * 49 * 2
    assert binding.na2d_workspace_bytes(P(k=4), binding.WS_BWD) == 0
    # fused backward: the two-kernel path needs delta (one fp32 per query) and the partial bias gradients,
    # far less than one attention tensor; the other path holds the attention weights and the unfused workspace
    fused = binding.na2d_workspace_bytes(p, binding.WS_FUSED_BWD)
    assert binding.na2d_fused_bwd_is_fused(p) == 1
    assert 64 * 2 * 56 * 56 * 4 <= fused < 64 * 2 * 56 * 56 * 49 * 2 and fused % 256 == 0
    for other in (P(B=2, heads=2, H=56, W=56, k=7, dtype=0), P(B=2, heads=2, H=56, W=56, k=11, dtype=1)):   # fp32; k > 9
        assert binding.na2d_fused_bwd_is_fused(other) == 0
        assert binding.na2d_workspace_bytes(other, binding.WS_FUSED_BWD) >= binding.na2d_workspace_bytes(other, binding.WS_BWD)
    for H, W, k in ((28, 28, 7), (20, 16, 5), (19, 37, 5), (7, 7, 7), (14, 14, 7), (3, 3, 3)):   # ragged / far-border tiles included
        assert binding.na2d_fused_bwd_is_fused(P(B=2, heads=2, H=H, W=W, k=k, dtype=2)) == 1
    assert binding.na2d_fused_bwd_is_fused(P(k=4)) == -3


def nearest_window(i, L, k):
    order = sorted(range(L), key=lambda j: abs(j - i))
    return sorted(order[:k])


@pytest.mark.parametrize("k", [3, 5, 7, 9, 11, 13])
def test_axis_tables_match_brute_force(k):
    for L in list(range(k, 30)) + [56, 57, 200, 334]:
        start, qs, qe = binding.na2d_host_axis_tables(L, k)
        windows = [nearest_window(i, L, k) for i in range(L)]
        assert start.tolist() == [w[0] for w in windows]
        for j in range(L):
            seen_by = [i for i in range(L) if j in windows[i]]
            # the inverse neighbourhood is contiguous and equals [qs, qe]
            assert seen_by == list(range(qs[j], qe[j] + 1)), (L, k, j)
            # k wide in the interior, k + (k-1)/2 next to one border, at most 2k-1 when the axis
            # is so short that a key is near both borders
            assert len(seen_by) <= (k + k // 2 if L >= 3 * k else 2 * k - 1)


def test_axis_table_errors():
    lib = binding.load()
    assert lib.na2d_host_axis_tables(5, 7, None, None, None) == -4
    assert lib.na2d_host_axis_tables(8, 4, None, None, None) == -3
    assert lib.na2d_host_axis_tables(0, 3, None, None, None) == -6


def test_binding_rejects_cpu_tensors():
    x = torch.zeros(1, 1, 14, 14, 32)
    with pytest.raises(ValueError):
        binding.na2d_softmax(torch.zeros(1, 1, 14, 14, 9), 3, x, torch.zeros(1, 1, 14, 14, 9))


def P1(B=1, heads=1, L=20, D=32, k=3, dtype=0):
    return binding.Na1dProblem(B, heads, L, D, k, dtype)


@pytest.mark.parametrize("prob,code", [
    (P1(), 0), (P1(k=7, L=7), 0), (P1(k=63, L=63), 0),
    (P1(dtype=5), -2),
    (P1(k=4), -3), (P1(k=1), -3), (P1(k=65, L=100), -3),
    (P1(k=7, L=6), -4),
    (P1(D=16), -5),
    (P1(B=0), -6), (P1(L=-3), -6), (P1(B=1 << 16, heads=64, L=1 << 12), -6),
])
def test_1d_problem_validation(prob, code):
    assert binding.na1d_validate_problem(prob) == code


def test_1d_entry_points_reject_bad_arguments_before_any_hip_call():
    lib = binding.load()
    good = P1(k=5)
    buf = ctypes.create_string_buffer(64)
    a16 = (ctypes.addressof(buf) + 15) & ~15
    ok, off = ctypes.c_void_p(a16), ctypes.c_void_p(a16 + 4)
    r = ctypes.byref(good)
    assert lib.na1d_qk_rpb(None, ok, ok, None, 1.0, ok, None) == -1
    assert lib.na1d_qk_rpb(r, None, ok, None, 1.0, ok, None) == -1
    assert lib.na1d_qk_rpb(r, ok, ok, off, 1.0, ctypes.c_void_p(a16 + 16), None) == -7
    assert lib.na1d_qk_rpb(r, ok, ctypes.c_void_p(a16 + 16), None, 1.0, ok, None) == -10
    assert lib.na1d_av(r, ok, ctypes.c_void_p(a16 + 16), ok, None) == -10
    assert lib.na1d_fused_fwd(r, ok, ok, ok, None, 1.0, ok, None, None) == -10
    assert lib.na1d_av_bwd_v(r, ok, off, ctypes.c_void_p(a16 + 16), None) == -7
    assert lib.na1d_softmax_bwd(r, ok, ctypes.c_void_p(a16 + 16), ok, None) == -10
    assert lib.na1d_qk_bwd_rpb(r, ok, ctypes.c_void_p(a16 + 16), None, 0, None) == -8
    assert lib.na1d_qk_bwd_rpb(r, ok, ctypes.c_void_p(a16 + 16), ctypes.c_void_p(a16 + 32), 8, None) == -8
    assert lib.na1d_qk_bwd_rpb(ctypes.byref(P1(k=6)), ok, ok, ok, 1 << 20, None) == -3
    # workspace: one (2k-1)-cell table of 64-bit integers per (plane, tile of 256 positions; 128 for k > 31)
    assert binding.na1d_workspace_bytes(P1(B=3, heads=2, L=1000, k=7)) == 3 * 2 * 4 * 13 * 8
    assert binding.na1d_workspace_bytes(P1(B=1, heads=1, L=1000, k=33)) == 8 * 65 * 8
    assert binding.na1d_workspace_bytes(P1(k=4)) == 0
    # fused backward: delta [B, heads, L] fp32 (rounded up to 256 bytes), then the bias-gradient tables
    assert binding.na1d_fused_bwd_workspace_bytes(P1(B=3, heads=2, L=1000, k=7)) == (3 * 2 * 1000 * 4 + 255) // 256 * 256 + 3 * 2 * 4 * 13 * 8
    assert lib.na1d_fused_bwd(r, ok, ok, ok, None, 1.0, ok, ok, ok, ctypes.c_void_p(a16 + 16), ctypes.c_void_p(a16 + 32), None,
                              ok, 1 << 20, None) == -10
    assert lib.na1d_fused_bwd(r, ok, ok, ok, None, 1.0, None, ok, ok, ok, ok, None, ok, 1 << 20, None) == -1
    assert lib.na1d_fused_bwd(r, ok, ok, ok, None, 1.0, ok, ok, ctypes.c_void_p(a16 + 16), ctypes.c_void_p(a16 + 32),
                              ctypes.c_void_p(a16 + 48), None, ok, 8, None) == -8
