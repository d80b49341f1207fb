"""Seeded synthetic packed-microbatch workloads.

This module holds NO attention arithmetic.  It only draws document lengths and
bf16-representable input values, so that the HIP path and the CPU oracle are fed the very
same bits.  The paper's training corpus (an open-source code dataset with a long-tailed
length distribution, Section 2 "sequence length variability") is not available; packed
documents of lengths {l_1..l_k} with sum N (Section 5.2, "Micro-Batch Time Prediction")
are drawn from log-normal / mixture length models instead.

Conventions
-----------
* ``cu_seqlens``: int32 [B+1], cu[0] = 0, cu[B] = N, document b owns rows cu[b]..cu[b+1]-1.
* values: float32 arrays that are exactly representable in bf16 (round-to-nearest-even),
  plus their raw uint16 bit patterns; shapes [N, H, d].
"""
from __future__ import annotations

import dataclasses
import math
from typing import Callable, List, Optional

import numpy as np


# --------------------------------------------------------------------------------------
# bf16 helpers (bit manipulation only)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 -> bf16 (round-to-nearest-even), return uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# length generators
# --------------------------------------------------------------------------------------
def lognormal_draw(median: float, sigma: float) -> Callable[[np.random.Generator], int]:
    mu = math.log(median)

    def draw(rng: np.random.Generator) -> int:
        return int(round(math.exp(mu + sigma * float(rng.standard_normal()))))

    return draw


def mixture_draw(p_short: float, median: float, sigma: float, lo_long: int, hi_long: int):
    mu = math.log(median)

    def draw(rng: np.random.Generator) -> int:
        u = float(rng.random())
        if u < p_short:
            return int(round(math.exp(mu + sigma * float(rng.standard_normal()))))
        return int(rng.integers(lo_long, hi_long + 1))

    return draw


def pack(rng: np.random.Generator, n_tokens: int, draw, lo: int) -> List[int]:
    """Draw documents until the token budget is filled.

    Each draw is clipped to [lo, n_tokens]; a draw that overshoots the budget is truncated
    to the remainder; a final piece shorter than ``lo`` is merged into the previous
    document so that every document has at least ``lo`` tokens.
    """
    lengths: List[int] = []
    filled = 0
    while filled < n_tokens:
        l = min(max(draw(rng), lo), n_tokens)
        if filled + l > n_tokens:
            l = n_tokens - filled
        lengths.append(l)
        filled += l
    if len(lengths) > 1 and lengths[-1] < lo:
        last = lengths.pop()
        lengths[-1] += last
    return lengths


def uniform_cuts(rng: np.random.Generator, n_tokens: int, n_docs: int, lo: int) -> List[int]:
    """n_docs-1 sorted uniform cut points, redrawn until every piece has >= lo tokens."""
    while True:
        c = np.sort(rng.integers(1, n_tokens, size=n_docs - 1))
        edges = np.concatenate([[0], c, [n_tokens]])
        lengths = np.diff(edges)
        if (lengths >= lo).all():
            return [int(x) for x in lengths]


def lengths_to_cu(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int64)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    assert cu[-1] < 2**31
    return cu.astype(np.int32)


# --------------------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    name: str
    n_tokens: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    lengths: List[int]
    std: float
    seed: int

    @property
    def cu_seqlens(self) -> np.ndarray:
        return lengths_to_cu(self.lengths)

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def pairs(self) -> int:
        """Number of (query, key) pairs inside the document-causal mask."""
        return sum(l * (l + 1) // 2 for l in self.lengths)

    @property
    def flops_fwd_bwd(self) -> int:
        """14 * d * Hq * pairs: 2 contractions forward, 5 backward, 2*d flop per pair each."""
        return 14 * self.head_dim * self.n_q_heads * self.pairs

    @property
    def flops_fwd(self) -> int:
        return 4 * self.head_dim * self.n_q_heads * self.pairs

    @property
    def algorithmic_bytes(self) -> int:
        """fwd reads Q,K,V writes O,LSE; bwd reads Q,K,V,O,dO,LSE,D writes dQ,dK,dV,D."""
        n, d = self.n_tokens, self.head_dim
        return 2 * d * n * (7 * self.n_q_heads + 6 * self.n_kv_heads) + 12 * n * self.n_q_heads

    def values(self, names=("q", "k", "v", "do")):
        """bf16-representable float32 arrays in the fixed order Q, K, V, dO."""
        rng = np.random.default_rng(self.seed + 500000)
        out = {}
        for nm, h in (("q", self.n_q_heads), ("k", self.n_kv_heads), ("v", self.n_kv_heads),
                      ("do", self.n_q_heads)):
            x = rng.standard_normal((self.n_tokens, h, self.head_dim), dtype=np.float32)
            if self.std != 1.0:
                x = x * np.float32(self.std)
            bits = f32_to_bf16_bits(x)
            if nm in names:
                out[nm] = bits
        return out


def custom(name, lengths, n_q_heads, n_kv_heads, head_dim, std=1.0, seed=0) -> Workload:
    return Workload(name, int(sum(lengths)), n_q_heads, n_kv_heads, head_dim,
                    [int(l) for l in lengths], std, seed)


def config(k: int, seed_offset: int = 0, microbatch: Optional[int] = None) -> Workload:
    """The five benchmark configurations (k = 1..5).  k = 5 needs ``microbatch`` in 0..63."""
    if k == 1:
        seed = 1001 + seed_offset
        rng = np.random.default_rng(seed)
        lengths = uniform_cuts(rng, 2048, 4, 64)
        return Workload("cfg1_tiny", 2048, 2, 2, 64, lengths, 1.0, seed)
    if k == 2:
        seed = 1002 + seed_offset
        rng = np.random.default_rng(seed)
        lengths = pack(rng, 8192, lognormal_draw(512, 1.2), 16)
        return Workload("cfg2_7b_tp8_8k", 8192, 4, 4, 128, lengths, 1.0, seed)
    if k == 3:
        seed = 1003 + seed_offset
        rng = np.random.default_rng(seed)
        lengths = pack(rng, 32768, mixture_draw(0.9, 300, 1.0, 4096, 32768), 16)
        return Workload("cfg3_longtail_32k", 32768, 4, 4, 128, lengths, 1.0, seed)
    if k == 4:
        seed = 1004 + seed_offset
        rng = np.random.default_rng(seed)
        lengths = pack(rng, 16384, lognormal_draw(1024, 1.3), 32)
        return Workload("cfg4_70b_gqa_16k", 16384, 8, 1, 128, lengths, 0.5, seed)
    if k == 5:
        assert microbatch is not None and 0 <= microbatch < 64
        seed = 5000 + microbatch + seed_offset
        if microbatch == 0:
            lengths = [4096]
        else:
            rng = np.random.default_rng(seed)
            lengths = pack(rng, 4096, lognormal_draw(32 * 2 ** (microbatch % 8), 0.8), 16)
        return Workload(f"cfg5_sweep_mb{microbatch:02d}", 4096, 4, 4, 128, lengths, 1.0, seed)
    raise ValueError(f"unknown config {k}")
