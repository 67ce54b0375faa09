"""Seeded synthetic inputs for the DFSS attention forward pass.

This module draws random tensors and nothing else: no part of the method's
arithmetic lives here, so the HIP path and the CPU oracle can both be fed from
it without sharing any computation.

The workloads stand in for the paper's evaluation inputs, which are not
available offline: they take the sequence lengths of its tasks (384 for
question answering, 512 for masked language modelling, 1024/2048/4096 for the
long-range tasks, Sec. 5.1), the head size of its latency study (d = 64,
Sec. 5.2) and its own modelling assumption that scaled scores are i.i.d.
Gaussian (Prop. 4.2): with Q, K ~ N(0, sigma^2) the scaled scores are close to
N(0, sigma^4 * d * scale^2).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    L: int
    d: int
    N: int
    M: int
    sigma: float
    seed: int
    integer: bool = False  # Q, K integer-valued in [-4, 4] (scores exact in fp32)
    float32: bool = False  # the paper's 4-byte mode: float32 tensors, not rounded to bfloat16

    @property
    def BH(self) -> int:
        return self.B * self.H

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny_2to4", 1, 1, 256, 64, 2, 4, 1.0, 1001),
        Workload("tiny_2to4_int", 1, 1, 256, 64, 2, 4, 1.0, 1002, integer=True),
        Workload("bert_base_L384_2to4", 8, 12, 384, 64, 2, 4, 1.0, 2001),
        Workload("bert_base_L512_1to2", 16, 12, 512, 64, 1, 2, 1.0, 3001),
        Workload("long_L1024_2to4", 2, 12, 1024, 64, 2, 4, 1.0, 4001),
        Workload("long_L2048_2to4", 2, 12, 2048, 64, 2, 4, 1.0, 4002),
        Workload("long_L4096_2to4", 2, 12, 4096, 64, 2, 4, 1.0, 4003),
        Workload("large_head_L2048_d128_2to4", 4, 16, 2048, 128, 2, 4, 0.5, 5001),
        Workload("large_head_L2048_d128_1to2", 4, 16, 2048, 128, 1, 2, 0.5, 5001),
        # the paper's second precision (float data, 1:2) on the same shapes
        Workload("tiny_1to2_f32", 1, 1, 256, 64, 1, 2, 1.0, 6001, float32=True),
        Workload("tiny_1to2_f32_int", 1, 1, 256, 64, 1, 2, 1.0, 6002, integer=True, float32=True),
        Workload("bert_base_L512_1to2_f32", 16, 12, 512, 64, 1, 2, 1.0, 6003, float32=True),
        Workload("long_L4096_1to2_f32", 2, 12, 4096, 64, 1, 2, 1.0, 6004, float32=True),
        Workload("large_head_L2048_d128_1to2_f32", 4, 16, 2048, 128, 1, 2, 0.5, 6005, float32=True),
    ]
    # the paper's latency study (Sec. 5.2): 4 heads, d = 64, L = 256 .. 4096, batch large enough to keep the GPU
    # busy (here B * L = 32768 tokens at every length), in its two precisions
    + [Workload(f"curve_L{L}_2to4", 32768 // L, 4, L, 64, 2, 4, 1.0, 7000 + L) for L in (256, 512, 1024, 2048, 4096)]
    + [Workload(f"curve_L{L}_1to2_f32", 32768 // L, 4, L, 64, 1, 2, 1.0, 7500 + L, float32=True)
       for L in (256, 512, 1024, 2048, 4096)]
}


def gaussian_qkv(BH: int, Lq: int, Lk: int, d: int, sigma: float, seed: int, dtype=torch.bfloat16):
    """Q [BH,Lq,d], K,V [BH,Lk,d] ~ N(0, sigma^2), rounded to `dtype` (CPU tensors)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q = (torch.randn(BH, Lq, d, generator=g) * sigma).to(dtype)
    K = (torch.randn(BH, Lk, d, generator=g) * sigma).to(dtype)
    V = (torch.randn(BH, Lk, d, generator=g) * sigma).to(dtype)
    return Q, K, V


def integer_qkv(BH: int, Lq: int, Lk: int, d: int, seed: int, lo: int = -4, hi: int = 4, dtype=torch.bfloat16):
    """Q, K integers uniform in [lo, hi] (exact in bfloat16), V ~ N(0,1) rounded to `dtype`."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q = torch.randint(lo, hi + 1, (BH, Lq, d), generator=g).to(dtype)
    K = torch.randint(lo, hi + 1, (BH, Lk, d), generator=g).to(dtype)
    V = torch.randn(BH, Lk, d, generator=g).to(dtype)
    return Q, K, V


def make(workload: Workload | str):
    """Inputs of a named workload: (Q, K, V) CPU tensors shaped [B*H, L, d], bfloat16 (float32 for
    the workloads of the 4-byte mode)."""
    w = WORKLOADS[workload] if isinstance(workload, str) else workload
    dtype = torch.float32 if w.float32 else torch.bfloat16
    if w.integer:
        return integer_qkv(w.BH, w.L, w.L, w.d, w.seed, dtype=dtype)
    return gaussian_qkv(w.BH, w.L, w.L, w.d, w.sigma, w.seed, dtype=dtype)


def padding_lengths(B: int, Lk: int, seed: int, min_frac: float = 0.5):
    """Valid key counts of a padded batch: one integer per batch element, uniform in
    [min_frac * Lk, Lk] and not aligned to anything (a stand-in for the length mix of a padded
    question-answering batch).  Element 0 always has full length."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    lo = max(1, int(min_frac * Lk))
    lengths = torch.randint(lo, Lk + 1, (B,), generator=g)
    lengths[0] = Lk
    return lengths


def key_padding_bias(lengths: torch.Tensor, Lk: int):
    """float32 [B, Lk]: 0 for the first lengths[b] keys of batch element b, -inf for the padding."""
    j = torch.arange(Lk).view(1, Lk)
    bias = torch.zeros((lengths.numel(), Lk), dtype=torch.float32)
    bias[j >= lengths.view(-1, 1)] = float("-inf")
    return bias


def relative_position_mask(Lq: int, Lk: int, seed: int, slope: float = 0.01):
    """float32 [Lq, Lk]: a relative-position term -slope * |i + (Lk - Lq) - j| plus a seeded term per distance
    (one value for every diagonal, Gaussian, sigma 0.1): finite everywhere, different in every entry of a row."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    per_distance = 0.1 * torch.randn(Lq + Lk, generator=g)
    i = torch.arange(Lq).view(Lq, 1) + (Lk - Lq)
    j = torch.arange(Lk).view(1, Lk)
    return (-slope * (i - j).abs().float() + per_distance[i - j + Lq]).contiguous()


def block_pattern(nq: int, nk: int, seed: int, window: int = 1, n_global: int = 1, n_random: int = 2):
    """uint8 [nq, nk] block pattern in the style of the block-sparse long-sequence models the paper
    combines with (sliding window of +-`window` blocks around the diagonal, `n_global` leading key
    blocks seen by every row block and `n_global` leading row blocks that see everything, plus
    `n_random` random key blocks per row block).  Every row keeps at least its diagonal block."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    m = torch.zeros((nq, nk), dtype=torch.uint8)
    for i in range(nq):
        c = min(nk - 1, i * nk // nq)                       # diagonal block of this row block
        m[i, max(0, c - window):min(nk, c + window + 1)] = 1
        m[i, :min(n_global, nk)] = 1
        if n_random > 0:
            m[i, torch.randint(0, nk, (n_random,), generator=g)] = 1
    m[:min(n_global, nq), :] = 1
    return m


def to_numpy_f32(t: torch.Tensor):
    """Widen a (bfloat16) tensor to a float32 numpy array holding the same values."""
    return t.to(torch.float32).contiguous().numpy()
