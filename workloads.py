"""Seeded synthetic decode-attention workloads.

Shared by the tests, the smoke check and the benchmark.  It holds no part of
the method's arithmetic: only shapes, seeds and random draws.  Both the HIP
path and the CPU oracle consume the 16-bit values produced here, bit for bit.

The paper measures attention micro-benchmarks parameterised by heads, batch,
context length and head dimension on random FP16 data (Sections 5 and 6); no
dataset is involved.  The five named workloads below take those shapes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np
import torch

KV_PADDED, KV_PACKED = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    dtype: str                      # "f16" | "bf16"
    seqlens: tuple                  # per-sequence context lengths
    kv_layout: int = KV_PADDED
    seed: int = 0
    outlier_frac: float = 0.0       # fraction of key rows scaled by outlier_gain
    outlier_gain: float = 8.0
    note: str = ""
    N_q: int = 1                    # query rows per sequence (the last N_q cached tokens)
    causal: bool = False            # query row i sees the first N_b - N_q + i + 1 cached tokens
    q_lens: Optional[tuple] = None  # per-sequence query lengths (N_q is then the longest); q is packed

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))

    @property
    def n_stride(self) -> int:
        return int(max(self.seqlens)) if self.seqlens else 0

    @property
    def kv_bytes(self) -> int:
        """Algorithmic KV-cache traffic: every cached K and V element read once."""
        return 2 * self.Hkv * self.total_tokens * self.D * 2

    @property
    def torch_dtype(self):
        return torch.float16 if self.dtype == "f16" else torch.bfloat16


def _ragged_lengths(seed: int, B: int, lo: int, hi: int) -> tuple:
    rng = np.random.default_rng(seed)
    return tuple(int(x) for x in rng.integers(lo, hi + 1, size=B))


def named(idx: int) -> Workload:
    """The five benchmark configurations (index 1..5) and three widened shapes (6..8)."""
    if idx == 1:
        return Workload("cfg1_mha_b1_h8_d64_n4096_f16", 1, 8, 8, 64, "f16", (4096,), KV_PADDED, seed=1)
    if idx == 2:
        return Workload("cfg2_mha_b1_h32_d128_n65536_bf16", 1, 32, 32, 128, "bf16", (65536,), KV_PADDED,
                        seed=2)
    if idx == 3:
        return Workload("cfg3_gqa_b1_h64_kv8_d128_n262144_bf16", 1, 64, 8, 128, "bf16", (262144,),
                        KV_PADDED, seed=3)
    if idx == 4:
        return Workload("cfg4_mha_b16_h32_d128_ragged_bf16", 16, 32, 32, 128, "bf16",
                        _ragged_lengths(4, 16, 1024, 131072), KV_PACKED, seed=4)
    if idx == 5:
        return Workload("cfg5_gqa_b4_h56_kv8_d128_outliers_bf16", 4, 56, 8, 128, "bf16",
                        (3000, 17000, 100003, 250001), KV_PACKED, seed=5, outlier_frac=0.01)
    # Widened rows of the same path (not among the five headline configurations): head dim 256,
    # a causal query tile of 4 tokens per sequence (speculative decoding), 32 query heads per KV head.
    if idx == 6:
        return Workload("cfg6_gqa_b4_h32_kv4_d256_n65536_bf16", 4, 32, 4, 256, "bf16", (65536,) * 4, KV_PADDED,
                        seed=6)
    if idx == 7:
        return Workload("cfg7_gqa_b4_h32_kv8_d128_n65536_q4_causal_bf16", 4, 32, 8, 128, "bf16", (65536,) * 4,
                        KV_PADDED, seed=7, N_q=4, causal=True)
    if idx == 8:
        return Workload("cfg8_mqa_b4_h64_kv2_d128_n262144_bf16", 4, 64, 2, 128, "bf16", (262144,) * 4, KV_PADDED,
                        seed=8)
    raise ValueError("workload index must be 1..8")


def scaled_down(w: Workload, factor: int, min_len: int = 1) -> Workload:
    """Same structure with every context length divided by ``factor`` (ragged tails kept odd)."""
    lens = tuple(max(min_len, n // factor + (1 if n % 2 else 0)) for n in w.seqlens)
    return replace(w, name=f"{w.name}_div{factor}", seqlens=lens)


@dataclass
class Inputs:
    w: Workload
    q: torch.Tensor                 # [B, Hq, D]; [B, N_q, Hq, D] when N_q > 1; [sum(q_lens), Hq, D] when ragged
    k: torch.Tensor                 # PADDED [B, Hkv, n_stride, D] | PACKED [Hkv, total, D]
    v: torch.Tensor
    seqlens: List[int] = field(default_factory=list)


def generate(w: Workload, device="cpu", slab_rows: int = 1 << 16) -> Inputs:
    """Draw Q, K, V ~ N(0,1) rounded to the workload's 16-bit type.

    K rows flagged by a seeded Bernoulli(outlier_frac) draw are multiplied by
    ``outlier_gain`` (a power of two: exact in 16 bits).  Generation runs on
    ``device`` in slabs so that a multi-GB cache never needs an fp32 copy.
    Padded rows beyond a sequence's length are left as drawn (finite values
    that a correct kernel must never let reach the result).
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1000 + w.seed)
    dt = w.torch_dtype
    if w.q_lens is not None:
        assert len(w.q_lens) == w.B and max(w.q_lens) == w.N_q
        q = torch.randn(int(sum(w.q_lens)), w.Hq, w.D, generator=gen, device=dev, dtype=torch.float32).to(dt)
    else:
        q = torch.randn(w.B, w.N_q, w.Hq, w.D, generator=gen, device=dev, dtype=torch.float32).to(dt)
        if w.N_q == 1:
            q = q.view(w.B, w.Hq, w.D)
    if w.kv_layout == KV_PADDED:
        shape = (w.B * w.Hkv * w.n_stride, w.D)
        final = (w.B, w.Hkv, w.n_stride, w.D)
    else:
        shape = (w.Hkv * w.total_tokens, w.D)
        final = (w.Hkv, w.total_tokens, w.D)
    k = torch.empty(shape, device=dev, dtype=dt)
    v = torch.empty(shape, device=dev, dtype=dt)
    rows = shape[0]
    for r0 in range(0, rows, slab_rows):
        r1 = min(rows, r0 + slab_rows)
        kb = torch.randn(r1 - r0, w.D, generator=gen, device=dev, dtype=torch.float32)
        if w.outlier_frac > 0.0:
            flag = torch.rand(r1 - r0, 1, generator=gen, device=dev) < w.outlier_frac
            kb = torch.where(flag, kb * w.outlier_gain, kb)
        k[r0:r1] = kb.to(dt)
        v[r0:r1] = torch.randn(r1 - r0, w.D, generator=gen, device=dev, dtype=torch.float32).to(dt)
    return Inputs(w, q, k.view(final), v.view(final), list(w.seqlens))


def head_slice(inp: Inputs, b: int, h_kv: int):
    """K and V rows of one (sequence, KV head): two [N_b, D] tensors (views)."""
    w = inp.w
    n = inp.seqlens[b]
    if w.kv_layout == KV_PADDED:
        return inp.k[b, h_kv, :n], inp.v[b, h_kv, :n]
    start = int(sum(inp.seqlens[:b]))
    return inp.k[h_kv, start:start + n], inp.v[h_kv, start:start + n]
