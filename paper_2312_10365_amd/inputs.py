"""Seeded synthetic inputs for the routed FFN (host side, numpy only).

This module holds no arithmetic of the method itself: it draws random tensors of
the shapes the routed FFN consumes, rounds the bf16 ones to bf16 with
round-to-nearest-even, and hands back both the 16-bit patterns (what the GPU
reads) and their exact float32 widening (what a CPU checker reads).  The paper's
block-level measurements use randomly generated token sequences (evaluation
section, "Random" workload), so random tokens are the natural stand-in.

Presets follow the five benchmark shapes: `T` tokens, model width `d`, `N`
hidden-unit blocks of `Bs` units each (the paper's G groups of D/G rows), `k`
activated blocks per token (the paper's G').
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class Shape:
    name: str
    T: int
    d: int
    N: int
    Bs: int
    k: int
    seed: int
    act: int = 0           # 0 = GELU (erf form), 1 = ReLU
    flags: int = 0         # bit0: route on |logit|
    zipf_bias: bool = False
    w_std: float = 0.02
    wr_std: float = 0.02

    @property
    def D(self) -> int:
        return self.N * self.Bs

    @property
    def P(self) -> int:
        return self.T * self.k

    def gemm_flop_fwd_bwd(self) -> float:
        """Algorithmic GEMM FLOP of one forward+backward pass: six GEMMs of
        2*T*k*Bs*d each (up, down, dH, dX, dW1, dW2)."""
        return 12.0 * self.T * self.d * self.k * self.Bs


PRESETS: Dict[str, Shape] = {
    "tiny": Shape("tiny", T=512, d=256, N=16, Bs=64, k=4, seed=1001),
    "bert_base": Shape("bert_base", T=2048, d=768, N=32, Bs=96, k=8, seed=1002),
    "bert_large": Shape("bert_large", T=16384, d=1024, N=64, Bs=64, k=16, seed=1003),
    "opt_1p3b_skewed": Shape("opt_1p3b_skewed", T=8192, d=2048, N=64, Bs=128, k=16,
                             seed=1004, zipf_bias=True),
    "ffn_7b": Shape("ffn_7b", T=8192, d=4096, N=128, Bs=128, k=32, seed=1005),
    # Shapes of the paper's own block-level experiments (Table 2; batch 16 x 512 tokens; G = 4 or 8
    # groups of D/G hidden units, the default half of them active, or three quarters), with the
    # activation of the model family each block comes from.
    "paper_opt2048_g4": Shape("paper_opt2048_g4", T=8192, d=2048, N=4, Bs=2048, k=2, seed=2001, act=1),
    "paper_opt2048_g8": Shape("paper_opt2048_g8", T=8192, d=2048, N=8, Bs=1024, k=4, seed=2002, act=1),
    "paper_opt2048_g8_b34": Shape("paper_opt2048_g8_b34", T=8192, d=2048, N=8, Bs=1024, k=6, seed=2003, act=1),
    "paper_llama4096_g4": Shape("paper_llama4096_g4", T=8192, d=4096, N=4, Bs=2752, k=2, seed=2004),
    "paper_llama4096_g8": Shape("paper_llama4096_g8", T=8192, d=4096, N=8, Bs=1376, k=4, seed=2005),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 patterns (uint16) exactly to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    shape: Shape
    X_bits: np.ndarray      # uint16 [T, d]
    W1_bits: np.ndarray     # uint16 [N, Bs, d]
    W2_bits: np.ndarray     # uint16 [N, Bs, d]
    dY_bits: np.ndarray     # uint16 [T, d]
    W_r: np.ndarray         # float32 [d, N]
    b_r: Optional[np.ndarray]  # float32 [N] or None
    _cache: dict = field(default_factory=dict, repr=False)

    def f32(self, name: str) -> np.ndarray:
        """Exact float32 widening of one of the bf16 tensors ('X','W1','W2','dY')."""
        if name not in self._cache:
            self._cache[name] = bf16_bits_to_f32(getattr(self, name + "_bits"))
        return self._cache[name]


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def zipf_block_bias(N: int, seed: int, scale: float = 2.0, s: float = 1.1) -> np.ndarray:
    """Deterministic per-block router bias: the block of popularity rank r
    (r = 1..N, a seeded shuffle decides which block gets which rank) receives
    scale * r**(-s).  Makes a few buckets several times larger than the mean."""
    rng = np.random.Generator(np.random.Philox(seed ^ 0x5A17F))
    order = rng.permutation(N)
    b = np.empty(N, dtype=np.float32)
    ranks = np.arange(1, N + 1, dtype=np.float64)
    b[order] = (scale * ranks ** (-s)).astype(np.float32)
    return b


def make_inputs(shape: Shape) -> Inputs:
    """Draw all tensors of one workload from a counter-based generator."""
    def rng(stream: int) -> np.random.Generator:
        return np.random.Generator(np.random.Philox(key=shape.seed, counter=[0, 0, 0, stream]))

    X = f32_to_bf16_bits(_normal(rng(1), (shape.T, shape.d), 1.0))
    W1 = f32_to_bf16_bits(_normal(rng(2), (shape.N, shape.Bs, shape.d), shape.w_std))
    W2 = f32_to_bf16_bits(_normal(rng(3), (shape.N, shape.Bs, shape.d), shape.w_std))
    dY = f32_to_bf16_bits(_normal(rng(4), (shape.T, shape.d), 1.0))
    W_r = _normal(rng(5), (shape.d, shape.N), shape.wr_std)
    b_r = zipf_block_bias(shape.N, shape.seed) if shape.zipf_bias else None
    return Inputs(shape, X, W1, W2, dY, W_r, b_r)


def custom_shape(T: int, d: int, N: int, Bs: int, k: int, seed: int = 7, **kw) -> Shape:
    return Shape(f"custom_T{T}_d{d}_N{N}_Bs{Bs}_k{k}", T=T, d=d, N=N, Bs=Bs, k=k, seed=seed, **kw)


def make_adapters(shape: Shape, r: int, std: float = 0.02, seed_offset: int = 7):
    """Seeded low-rank adapter factors for the section-2.2 variant, as bf16 bit patterns:
    A1[d,r], C1[r,D], B2[D,r], C2[r,d] ~ N(0, std^2).  (Fine-tuning usually starts one factor of
    each pair at zero; both are drawn non-zero here so that every gradient is exercised.)"""
    rng = np.random.Generator(np.random.Philox(key=shape.seed + seed_offset))
    mk = lambda *dims: f32_to_bf16_bits((rng.standard_normal(dims, dtype=np.float32) * np.float32(std)))
    return mk(shape.d, r), mk(r, shape.D), mk(shape.D, r), mk(r, shape.d)
