"""Seeded synthetic inputs for 2D Neighborhood Attention.

This module holds no arithmetic of the method: it only draws Gaussian tensors of the
shapes the paper's NAT models induce (Section 3.2, Table "NAT variants": head dim 32,
heads 2/4/8/16 on 56/28/14/7-wide maps at 224x224 input; kernel 7x7 by default) and
rounds them once to the storage dtype.  Both the GPU tests/benchmark and the CPU oracle
are fed from here, so the two sides always see bit-identical inputs.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

TORCH_DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Problem:
    B: int
    heads: int
    H: int
    W: int
    D: int
    k: int
    dtype: str  # "f32" | "f16" | "bf16"

    @property
    def n_queries(self) -> int:
        return self.B * self.heads * self.H * self.W

    @property
    def kk(self) -> int:
        return self.k * self.k

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def default_scale(self) -> float:
        return float(self.D) ** -0.5


# The benchmark workloads: the map sizes and head counts of the NAT variants (Section 3.2) and of detection- and segmentation-sized inputs (shapes only; values are i.i.d. Gaussians).
CONFIGS = {
    "tiny": Problem(1, 1, 14, 14, 32, 3, "f32"),
    "nat_tiny_stage1": Problem(64, 2, 56, 56, 32, 7, "f16"),
    "nat_tiny_l1_bf16": Problem(128, 2, 56, 56, 32, 7, "bf16"),
    "nat_tiny_l2_bf16": Problem(128, 4, 28, 28, 32, 7, "bf16"),
    "nat_tiny_l3_bf16": Problem(128, 8, 14, 14, 32, 7, "bf16"),
    "nat_tiny_l4_bf16": Problem(128, 16, 7, 7, 32, 7, "bf16"),
    "detection_like": Problem(2, 2, 200, 334, 32, 7, "f16"),
    "segmentation_like": Problem(8, 2, 128, 128, 32, 7, "f16"),
    # other head dims (NAT itself always uses 32): the first-stage map with the same 64 channels as one head of
    # 64, and as four heads of 16
    "stage1_head_dim_64": Problem(64, 1, 56, 56, 64, 7, "f16"),
    "stage1_head_dim_16": Problem(64, 4, 56, 56, 16, 7, "f16"),
    # ... and half the batch with 128 channels as one head (the same tensor sizes)
    "stage1_head_dim_128": Problem(32, 1, 56, 56, 128, 7, "f16"),
    # the first-stage map in fp32 (the plain-ALU kernels)
    "nat_tiny_stage1_f32": Problem(64, 2, 56, 56, 32, 7, "f32"),
}


@dataclass(frozen=True)
class Problem1D:
    B: int
    heads: int
    L: int
    D: int
    k: int
    dtype: str

    @property
    def n_queries(self) -> int:
        return self.B * self.heads * self.L

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def default_scale(self) -> float:
        return float(self.D) ** -0.5


# 1D workloads.  The paper ships a 1D module but measures nothing on it, so the shapes are the 2D ones read
# as sequences: the tokens of NAT-Tiny's first stage (56 x 56 = 3136 per image) with the same batch, heads,
# head dim and window.
CONFIGS_1D = {
    "seq_3136_k7": Problem1D(64, 2, 3136, 32, 7, "f16"),
    "seq_3136_k31_bf16": Problem1D(64, 2, 3136, 32, 31, "bf16"),
}


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to the storage dtype (nearest-even) and return it as fp32."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(TORCH_DTYPES[dtype]).to(torch.float32).numpy()


def make_inputs(p: Problem, seed: int, rpb_std: float = 0.02, with_dout: bool = True) -> dict:
    """q, k, v ~ N(0,1), rpb ~ N(0, rpb_std^2), dout ~ N(0,1); drawn in that fixed order,
    each already rounded to ``p.dtype`` and returned as a C-contiguous fp32 numpy array."""
    g = np.random.default_rng(seed)
    shape = (p.B, p.heads, p.H, p.W, p.D)
    out = {}
    for name in ("q", "k", "v"):
        out[name] = round_to(g.standard_normal(shape, dtype=np.float32), p.dtype)
    nb = 2 * p.k - 1
    out["rpb"] = round_to((rpb_std * g.standard_normal((p.heads, nb, nb), dtype=np.float32)), p.dtype)
    if with_dout:
        out["dout"] = round_to(g.standard_normal(shape, dtype=np.float32), p.dtype)
    return out


def make_inputs_1d(p: Problem1D, seed: int, rpb_std: float = 0.02) -> dict:
    """The 1D counterpart of make_inputs: q, k, v, rpb [heads, 2k-1], dout, in that order."""
    g = np.random.default_rng(seed)
    shape = (p.B, p.heads, p.L, p.D)
    out = {}
    for name in ("q", "k", "v"):
        out[name] = round_to(g.standard_normal(shape, dtype=np.float32), p.dtype)
    out["rpb"] = round_to(rpb_std * g.standard_normal((p.heads, 2 * p.k - 1), dtype=np.float32), p.dtype)
    out["dout"] = round_to(g.standard_normal(shape, dtype=np.float32), p.dtype)
    return out


def to_device(x: np.ndarray, dtype: str, device: str = "cuda") -> torch.Tensor:
    """Host fp32 array (already representable in ``dtype``) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(TORCH_DTYPES[dtype]).to(device).contiguous()
