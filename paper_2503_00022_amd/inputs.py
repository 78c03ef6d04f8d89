"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the compression method itself: only shapes, budgets and
random tensors.  The shapes stand in for the prompts the paper ran through
Llama-2/3 and Mistral (Table 1, Table 3 header: 2k-18k-token contexts, budget
2048, 25 % of it for the representatives); those datasets and weights are not
reproduced here.

Everything is generated with a CPU `torch.Generator`, so the bits do not depend
on the GPU.  bf16 workloads are rounded to bf16 once; the CPU checker and the
GPU library read the very same bf16 values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    S: int
    D: int
    dtype: str            # "bf16" | "f16" | "f32"
    budget: int
    rep_fraction: float   # share of the budget given to the representatives
    anchor: str           # "random" | "mean" | "alternating"
    reduce_groups: bool   # sum each KV group's query heads into one score row
    layers: int = 1
    sink_bias: bool = False
    paged: bool = False
    block_size: int = 16

    @property
    def n_rep(self) -> int:  # round half up
        return int(math.floor(self.budget * self.rep_fraction + 0.5))

    @property
    def n_important(self) -> int:
        return self.budget - self.n_rep

    @property
    def Hs(self) -> int:
        return self.Hkv if self.reduce_groups else self.Hq

    @property
    def torch_dtype(self):
        return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[self.dtype]

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five graded configurations.  Where a configuration does not name the
# split or the anchor, the paper's default split (25 % representatives, Table 1)
# and the alternating anchor are used.
CONFIGS = {
    1: Workload("cfg1_mha8_s512_d64_f32", 1, 8, 8, 512, 64, "f32", 128, 0.5, "alternating", False),
    2: Workload("cfg2_llama2_7b_s4096", 1, 32, 32, 4096, 128, "bf16", 1024, 0.5, "random", False,
                sink_bias=True),
    3: Workload("cfg3_llama3_8b_gqa_s16384", 1, 32, 8, 16384, 128, "bf16", 4096, 0.25, "mean", True,
                layers=32),
    4: Workload("cfg4_mistral_7b_b8_s8192", 8, 32, 8, 8192, 128, "bf16", 2048, 0.25, "alternating",
                True, sink_bias=True),
    5: Workload("cfg5_long_s32768_paged", 1, 32, 8, 32768, 128, "bf16", 1024, 0.25, "alternating",
                True, layers=32, paged=True),
}

BASE_SEED = 20250300


def layer_seed(cfg_id: int, layer: int, base_seed: int = BASE_SEED) -> int:
    return base_seed + 1000 * cfg_id + layer


def anchor_seed(layer: int, base_seed: int = BASE_SEED) -> int:
    return base_seed + layer


def make_qkv(w: Workload, seed: int, device="cpu", want_v: bool = True):
    """Q [B,Hq,S,D], K, V [B,Hkv,S,D] ~ N(0,1), rounded once to the workload dtype.

    With `sink_bias`, the keys of tokens 0-3 of every KV head are shifted by
    3 sigma along that group's mean-query direction before rounding, which gives
    the first tokens the extra attention real prompts show.
    `device` other than "cpu" generates with that device's generator instead
    (faster for the multi-layer benchmark; such tensors are copied back to the
    host whenever the CPU checker needs them, so both sides still see the same
    bits)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    G = w.Hq // w.Hkv
    q = torch.randn(w.B, w.Hq, w.S, w.D, generator=g, device=dev, dtype=torch.float32)
    k = torch.randn(w.B, w.Hkv, w.S, w.D, generator=g, device=dev, dtype=torch.float32)
    v = torch.randn(w.B, w.Hkv, w.S, w.D, generator=g, device=dev, dtype=torch.float32) if want_v else None
    if w.sink_bias:
        u = q.view(w.B, w.Hkv, G * w.S, w.D).mean(dim=2)            # [B,Hkv,D]
        u = u / u.norm(dim=-1, keepdim=True).clamp_min(1e-20)
        k[:, :, : min(4, w.S), :] += 3.0 * u[:, :, None, :]
    dt = w.torch_dtype
    q, k = q.to(dt), k.to(dt)
    v = v.to(dt) if want_v else None
    return q, k, v


def make_block_table(w: Workload, seed: int):
    """Random placement of each sequence's logical blocks in a shared pool:
    int32 [B, S/block_size], a permutation of the B*S/block_size pool blocks."""
    g = torch.Generator()
    g.manual_seed(seed ^ 0x5EED)
    nb = w.S // w.block_size
    perm = torch.randperm(w.B * nb, generator=g).to(torch.int32)
    return perm.view(w.B, nb)


def to_paged(x: torch.Tensor, block_table: torch.Tensor, block_size: int) -> torch.Tensor:
    """Scatter a dense [B,Hkv,S,D] tensor into a pool [n_blocks, block_size, Hkv, D]
    according to block_table (pure data movement)."""
    B, Hkv, S, D = x.shape
    nb = S // block_size
    pool = torch.empty(B * nb, block_size, Hkv, D, dtype=x.dtype, device=x.device)
    src = x.view(B, Hkv, nb, block_size, D).permute(0, 2, 3, 1, 4).reshape(B * nb, block_size, Hkv, D)
    pool[block_table.to(x.device).view(-1).long()] = src
    return pool


def make_scores(B: int, Hs: int, S: int, seed: int, ties: bool = False):
    """Score-like positive rows for selection tests without running stage 1:
    a decaying profile times log-normal noise; with `ties`, values are quantised
    so that many exact duplicates straddle every threshold."""
    g = torch.Generator()
    g.manual_seed(seed)
    t = torch.arange(1, S + 1, dtype=torch.float32)
    base = (math.log(S + 1.0) - torch.log(t)) + 0.05
    sc = base[None, None, :] * torch.exp(0.7 * torch.randn(B, Hs, S, generator=g))
    if ties:
        sc = torch.round(sc * 4.0) / 4.0
    return sc.to(torch.float32).contiguous()
