"""Seeded synthetic workloads shaped like the paper's LLaMA-3.1-8B / Qwen-2.5-7B KV caches.

This module only builds inputs (q, k, v, true lengths).  It holds none of the
method's arithmetic and is the one piece shared by the GPU tests, the benchmark
and the CPU-oracle tests, so that both sides see identical bits.  Everything is
generated on the CPU with a seeded torch.Generator, rounded to the storage dtype
once, and then handed out; callers move tensors to the GPU themselves.

Stand-in note: the paper measured on RULER / LongBench / PG19 prompts run through
the real models (Section 5, Appendix C).  Those caches are not available here;
these tensors take only their shapes (heads, head_dim, GQA group, context length,
window and budget regimes) plus three structural features of real caches the
scores are sensitive to: a few large-magnitude key channels, attention-sink
tokens at the start, and a handful of tokens that one query attends to almost
exclusively ("needles").
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional

import torch

VARIANTS = ("value", "key", "joint")


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    N: int                      # padded cache length (max over the batch)
    W: int                      # observation window = number of trailing query rows
    dtype: str                  # "fp32" | "bf16"
    budget: int
    variants: tuple = VARIANTS
    seed: int = 0
    layers: int = 1
    outlier_channels: int = 0   # per KV head, key channels scaled by outlier_gain
    outlier_gain: float = 8.0
    sinks: int = 0              # first `sinks` tokens get key = sink_gain * mean window query of the group
    sink_gain: float = 3.0
    needles: int = 0            # tokens whose key is needle_gain * (one window query of the group)
    needle_gain: float = 2.0
    ragged: Optional[tuple] = None   # (lo, hi): true lengths drawn uniformly from [lo, hi]
    shared_query: float = 0.0   # stress knob: adds this multiple of a common unit direction to every query
    pad_nan: bool = False       # fill rows p >= len with NaN instead of noise (masking test)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def paper_configs() -> List[Workload]:
    """The five benchmark configurations (1-based names c1..c5)."""
    llama = dict(Hq=32, Hkv=8, d=128, W=32, dtype="bf16")
    return [
        Workload("c1_single_head_fp32", B=1, Hq=1, Hkv=1, d=64, N=512, W=16, dtype="fp32", budget=128,
                 seed=0, sinks=1, sink_gain=3.0),
        Workload("c2_llama8b_8k", B=1, N=8192, budget=1024, seed=2000, outlier_channels=4, sinks=4, **llama),
        Workload("c3_llama8b_b4_32k", B=4, N=32768, budget=2048, seed=3000, outlier_channels=4, sinks=4,
                 variants=("joint",), **llama),
        Workload("c4_qwen7b_128k", B=1, Hq=28, Hkv=4, d=128, N=131072, W=64, dtype="bf16", budget=4096,
                 seed=4000, outlier_channels=4, sinks=4, needles=64),
        Workload("c5_llama8b_ragged_sweep", B=2, N=65536, budget=2048, seed=5000, sinks=1, layers=32,
                 ragged=(16384, 65536), variants=("joint",), **llama),
    ]


def config(name: str) -> Workload:
    for w in paper_configs():
        if w.name == name or w.name.split("_")[0] == name:
            return w
    raise KeyError(name)


def seq_lens_of(wl: Workload) -> Optional[List[int]]:
    """True lengths per sequence; fixed across layers (drawn from the base seed)."""
    if wl.ragged is None:
        return None
    g = torch.Generator().manual_seed(wl.seed + 777)
    lo, hi = wl.ragged
    lens = torch.randint(lo, hi + 1, (wl.B,), generator=g).tolist()
    return [min(int(x), wl.N) for x in lens]


def make_inputs(wl: Workload, layer: int = 0):
    """Returns dict(q [B,Hq,W,d], k, v [B,Hkv,N,d], seq_lens list|None) on the CPU in wl's dtype."""
    g = torch.Generator().manual_seed(wl.seed + layer)
    B, Hq, Hkv, d, N, W, G = wl.B, wl.Hq, wl.Hkv, wl.d, wl.N, wl.W, wl.G
    lens = seq_lens_of(wl)
    q = torch.randn(B, Hq, W, d, generator=g)
    k = torch.randn(B, Hkv, N, d, generator=g)
    v = torch.randn(B, Hkv, N, d, generator=g)
    if wl.shared_query:
        u = torch.randn(d, generator=g)
        q += wl.shared_query * u / u.norm() * (d ** 0.5)
    if wl.outlier_channels:
        for b in range(B):
            for h in range(Hkv):
                ch = torch.randperm(d, generator=g)[: wl.outlier_channels]
                k[b, h, :, ch] *= wl.outlier_gain
    qbar = q.view(B, Hkv, G * W, d).mean(dim=2)                     # mean window query per KV head
    for t in range(wl.sinks):
        k[:, :, t, :] = wl.sink_gain * qbar
    if wl.needles:
        min_len = min(lens) if lens else N
        pos = (torch.randperm(min_len - W - wl.sinks, generator=g)[: wl.needles] + wl.sinks).tolist()
        for b in range(B):
            for h in range(Hkv):
                rows = torch.randint(0, G * W, (wl.needles,), generator=g).tolist()
                qg = q[b].view(Hkv, G * W, d)[h]
                for p, r in zip(pos, rows):
                    k[b, h, p, :] = wl.needle_gain * qg[r]
    dt = wl.torch_dtype()
    q, k, v = q.to(dt), k.to(dt), v.to(dt)
    if lens is not None and wl.pad_nan:
        for b, L in enumerate(lens):
            k[b, :, L:, :] = float("nan")
            v[b, :, L:, :] = float("nan")
    return {"q": q.contiguous(), "k": k.contiguous(), "v": v.contiguous(), "seq_lens": lens}


def small_cases() -> List[Workload]:
    """Oracle-sized cases for element-by-element parity: several tiles and ragged tails."""
    return [
        Workload("s_fp32_mha", B=2, Hq=2, Hkv=2, d=64, N=333, W=7, dtype="fp32", budget=40, seed=11, sinks=1),
        Workload("s_fp32_gqa_ragged", B=3, Hq=4, Hkv=2, d=128, N=700, W=16, dtype="fp32", budget=64, seed=12,
                 sinks=2, ragged=(300, 700), outlier_channels=2),
        Workload("s_bf16_llama", B=2, Hq=8, Hkv=2, d=128, N=1500, W=32, dtype="bf16", budget=200, seed=13,
                 sinks=4, outlier_channels=4),
        Workload("s_bf16_ragged", B=3, Hq=8, Hkv=2, d=128, N=2100, W=32, dtype="bf16", budget=128, seed=14,
                 sinks=4, outlier_channels=4, ragged=(700, 2100), pad_nan=True),
        Workload("s_bf16_qwen", B=1, Hq=14, Hkv=2, d=128, N=3000, W=64, dtype="bf16", budget=300, seed=15,
                 sinks=4, outlier_channels=4, needles=8),
        Workload("s_bf16_w1", B=2, Hq=8, Hkv=4, d=128, N=1000, W=1, dtype="bf16", budget=100, seed=16, sinks=1),
        Workload("s_bf16_strong_sink", B=1, Hq=8, Hkv=2, d=128, N=1200, W=32, dtype="bf16", budget=150, seed=17,
                 sinks=4, shared_query=1.0),
        Workload("s_bf16_tiny", B=1, Hq=4, Hkv=1, d=128, N=40, W=32, dtype="bf16", budget=33, seed=18, sinks=1),
        # degenerate shapes: one query head per KV head with fewer window rows than a wave owns; a cache that
        # is nothing but the window; many short ragged sequences; head_dim 64 in bf16; budget == length
        Workload("s_bf16_mha_rows16", B=1, Hq=3, Hkv=3, d=128, N=777, W=16, dtype="bf16", budget=77, seed=19,
                 sinks=1, outlier_channels=2),
        Workload("s_bf16_window_only", B=2, Hq=8, Hkv=2, d=128, N=32, W=32, dtype="bf16", budget=32, seed=20),
        Workload("s_bf16_many_short", B=37, Hq=4, Hkv=2, d=128, N=300, W=8, dtype="bf16", budget=8, seed=21,
                 sinks=1, ragged=(8, 300), pad_nan=True),
        Workload("s_bf16_d64", B=2, Hq=4, Hkv=2, d=64, N=500, W=16, dtype="bf16", budget=50, seed=22, sinks=2),
        Workload("s_fp32_d128_w64", B=1, Hq=2, Hkv=1, d=128, N=260, W=64, dtype="fp32", budget=65, seed=23, sinks=1),
        # the largest shapes the library accepts: 512 window rows per KV head (G=8, W=64), 128 ragged sequences
        Workload("s_bf16_max_rows", B=1, Hq=8, Hkv=1, d=128, N=500, W=64, dtype="bf16", budget=100, seed=24,
                 sinks=2, outlier_channels=4),
        Workload("s_bf16_max_batch", B=128, Hq=2, Hkv=1, d=128, N=96, W=4, dtype="bf16", budget=4, seed=25,
                 ragged=(4, 96), pad_nan=True),
    ]
