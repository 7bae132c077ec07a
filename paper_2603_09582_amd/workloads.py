"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it holds none of the method's arithmetic
and is the one piece shared by the HIP path's tests/bench and the CPU oracle's
tests.  The five workloads stand in for the models the paper evaluates
(Sec. 5.1 efficiency study, Sec. 5.2 classification, Sec. 5.5 generation): DeiT at 224x224 has
196 patches + 1 class token with head dim 64; DiT-XL/2 has hidden size 1152
over 16 heads (head dim 72) on 16x16 or 32x32 latent patches; a ViT with patch
size 8 at 1024x1024 sees 128x128 = 16384 tokens.  The paper's datasets and
trained weights are not used.

Recipe (fixed order, one generator per workload):
  1. Q, K, V ~ N(0, 1) as fp32 [B, H, N, d], drawn in that order;
  2. workload extras (below), still in fp32;
  3. bias ~ N(0, std 0.02) as fp32 [H, N, N] (shared over the batch),
     drawn one head at a time;
  4. everything rounded to bf16 (round-to-nearest-even); scale = 1/sqrt(d).
Extras:
  deit_base : K += o[h, c], o ~ N(0, std 0.5) per head and channel, the same
              for every batch entry and token (skews the sign balance of K).
  vit_hires : a Bernoulli(0.01) mask over (b, token), shared by heads and by
              Q, K and V, marks outlier tokens whose rows are scaled by 8.
The generator lives on `device`; a given (workload, device type) pair is
reproducible, CPU and GPU streams differ.  Whoever compares two
implementations draws once and hands the same bytes to both.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    seed: int
    extra: str  # "", "k_channel_offset", "token_outliers"
    note: str

    @property
    def pairs(self) -> int:
        return self.B * self.H * self.N * self.N

    @property
    def equiv_ops(self) -> int:
        """4*B*H*N^2*d: the two contractions of attention, 2 ops per MAC."""
        return 4 * self.pairs * self.d


WORKLOADS = {
    "deit_tiny": Workload("deit_tiny", 1, 3, 197, 64, 0, "",
                          "DeiT-Tiny-shaped single layer"),
    "deit_base": Workload("deit_base", 64, 12, 197, 64, 1, "k_channel_offset",
                          "DeiT-Base-shaped batch"),
    "dit_xl2_256": Workload("dit_xl2_256", 32, 16, 256, 72, 2, "",
                            "DiT-XL/2 at 256px (16x16 latent patches)"),
    "dit_xl2_512": Workload("dit_xl2_512", 8, 16, 1024, 72, 3, "",
                            "DiT-XL/2 at 512px (32x32 latent patches)"),
    "vit_hires": Workload("vit_hires", 2, 16, 16384, 64, 4, "token_outliers",
                          "high-resolution ViT, 128x128 patch grid"),
}
# Kernel-speed setting of Sec. 5.1's speed figure: head dimension 128 over a range of sequence
# lengths.  The paper states neither batch nor head count; 16 heads and a batch that keeps
# B * N = 16384 tokens are used here (the usual convention of attention kernel benchmarks).
SWEEP_HD128 = [f"hd128_n{n}" for n in (1024, 2048, 4096, 8192, 16384, 32768)]
for _i, _name in enumerate(SWEEP_HD128):
    _n = int(_name.split("_n")[1])
    WORKLOADS[_name] = Workload(_name, max(1, 16384 // _n), 16, _n, 128, 100 + _i, "",
                                "head dim 128 sequence-length sweep")
# The five benchmark configurations, smallest first.
WORKLOAD_ORDER = ["deit_tiny", "deit_base", "dit_xl2_256", "dit_xl2_512", "vit_hires"]


@dataclass
class Inputs:
    q: torch.Tensor      # bf16 [B, H, N, d]
    k: torch.Tensor      # bf16 [B, H, N, d]
    v: torch.Tensor      # bf16 [B, H, N, d]
    bias: Optional[torch.Tensor]  # bf16 [H, N, N] or None
    scale: float
    workload: Workload


def custom_workload(B: int, H: int, N: int, d: int, seed: int, extra: str = "",
                    name: str = "custom") -> Workload:
    return Workload(name, B, H, N, d, seed, extra, "custom shape")


def make_inputs(w: Workload, device: str = "cpu", with_bias: bool = True,
                bias_dtype: torch.dtype = torch.bfloat16) -> Inputs:
    """Draw the tensors of workload `w` on `device` following the module recipe."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.d)

    def normal(*s):
        return torch.randn(*s, generator=g, device=dev, dtype=torch.float32)

    q = normal(*shape)
    k = normal(*shape)
    v = normal(*shape)
    if w.extra == "k_channel_offset":
        off = normal(w.H, w.d) * 0.5
        k = k + off[None, :, None, :]
    elif w.extra == "token_outliers":
        mask = torch.rand(w.B, w.N, generator=g, device=dev) < 0.01
        f = torch.where(mask, 8.0, 1.0).to(torch.float32)[:, None, :, None]
        q, k, v = q * f, k * f, v * f
    elif w.extra != "":
        raise ValueError(f"unknown extra {w.extra!r}")
    q, k, v = (t.to(torch.bfloat16).contiguous() for t in (q, k, v))

    bias = None
    if with_bias:
        bias = torch.empty(w.H, w.N, w.N, device=dev, dtype=bias_dtype)
        for h in range(w.H):  # one head at a time keeps the fp32 temporary small
            bias[h] = (normal(w.N, w.N) * 0.02).to(bias_dtype)
    return Inputs(q, k, v, bias, 1.0 / math.sqrt(w.d), w)
