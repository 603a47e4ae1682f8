"""Seeded synthetic inputs for one SLiM-compressed linear layer.

Holds none of the method's arithmetic: only random tensors with the shapes of
LLaMA-2 layers (the models of the paper's layer-wise speed-up experiment,
Sec. 4 "Speedup") and the value distributions fixed for this build.  Both the
GPU path and the CPU oracle are fed from here.

Generation is on the CPU with one torch.Generator per tensor, so the same
seed gives the same bytes on any machine:
  W  fp32  N(0, 0.02)  [n][k]   seed 0
  L  fp16  N(0, 0.01)  [n][r]   seed 1
  R  fp16  N(0, 0.01)  [r][k]   seed 2
  X  fp16  N(0, 1)     [m][k]   seed 3; with outliers, ceil(0.01 k) input
     channels (chosen without replacement, seed 4) are multiplied by 20
     before the cast to fp16 (activation outlier channels of LLMs).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class LayerShape:
    name: str
    n: int          # d_out
    k: int          # d_in
    r: int          # adapter rank
    outliers: bool = True


# The configured workloads.  Rank is 10 % of the hidden size (paper, App.
# "Settings and Hyperparameters"), rounded as each configuration states.
TINY = LayerShape("tiny_512x512", 512, 512, 51, outliers=False)
L7B_ATTN = LayerShape("llama2_7b_attn_4096x4096", 4096, 4096, 410)
L7B_UP = LayerShape("llama2_7b_up_11008x4096", 11008, 4096, 410)
L7B_DOWN = LayerShape("llama2_7b_down_4096x11008", 4096, 11008, 410)
L13B_ATTN = LayerShape("llama2_13b_attn_5120x5120", 5120, 5120, 512)
L13B_UP = LayerShape("llama2_13b_up_13824x5120", 13824, 5120, 512)
L70B_ATTN = LayerShape("llama2_70b_attn_8192x8192", 8192, 8192, 820)
L70B_UP = LayerShape("llama2_70b_up_28672x8192", 28672, 8192, 820)

ALL_SHAPES = [TINY, L7B_ATTN, L7B_UP, L7B_DOWN, L13B_ATTN, L13B_UP, L70B_ATTN, L70B_UP]


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def make_weight(n: int, k: int, seed: int = 0) -> torch.Tensor:
    return torch.randn(n, k, generator=_gen(seed), dtype=torch.float32) * 0.02


def make_adapters(n: int, k: int, r: int, seed_l: int = 1, seed_r: int = 2):
    L = (torch.randn(n, r, generator=_gen(seed_l), dtype=torch.float32) * 0.01).to(torch.float16)
    R = (torch.randn(r, k, generator=_gen(seed_r), dtype=torch.float32) * 0.01).to(torch.float16)
    return L, R


def make_activations(m: int, k: int, outliers: bool = True, seed: int = 3,
                     seed_channels: int = 4) -> torch.Tensor:
    X = torch.randn(m, k, generator=_gen(seed), dtype=torch.float32)
    if outliers:
        cnt = math.ceil(0.01 * k)
        ch = torch.randperm(k, generator=_gen(seed_channels))[:cnt]
        X[:, ch] *= 20.0
    return X.to(torch.float16)


def make_layer(shape: LayerShape, m: int, seed: int = 0):
    """(W fp32, L fp16, R fp16, X fp16) on the CPU for one configured layer.
    `seed` offsets all five generator seeds together."""
    W = make_weight(shape.n, shape.k, seed + 0)
    L, R = make_adapters(shape.n, shape.k, shape.r, seed + 1, seed + 2)
    X = make_activations(m, shape.k, shape.outliers, seed + 3, seed + 4)
    return W, L, R, X
