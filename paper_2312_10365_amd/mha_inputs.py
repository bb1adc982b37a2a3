"""Seeded synthetic inputs of the sparse multi-head attention workloads (generation only: none of
the method's arithmetic lives here; the CPU oracle and the GPU path both read these arrays).

Recipe: keys and values are standard normal.  A query is an even mix of one randomly chosen key
of its own sequence and fresh noise, so that, as in a trained model, a query has a few keys it
genuinely prefers and product quantisation has something to find.  The codebooks of a head are E
sub-vectors sampled from that head's keys (the initialisation a k-means run would start from);
queries and keys share them.  Everything is rounded to bf16 (codebooks stay fp32)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np

from .inputs import bf16_bits_to_f32, f32_to_bf16_bits


@dataclass(frozen=True)
class MhaShape:
    name: str
    batch: int
    H: int
    n: int
    dh: int
    L: int
    E: int = 16
    seed: int = 11
    scale: float = 0.0     # 0: 1 / sqrt(dh)

    @property
    def S(self) -> int:
        return self.batch * self.H

    @property
    def M(self) -> int:
        return self.dh // 8

    @property
    def softmax_scale(self) -> float:
        return self.scale if self.scale else float(self.dh) ** -0.5


PRESETS: Dict[str, MhaShape] = {
    "mha_tiny": MhaShape("mha_tiny", batch=2, H=3, n=100, dh=64, L=13, seed=3001),
    # Batch 16, sequence 512, L = n / 8 (the paper's default sparsity), 32 heads: head size 64 for
    # the model width 2048 blocks, 128 for the width 4096 blocks.
    "mha_opt2048": MhaShape("mha_opt2048", batch=16, H=32, n=512, dh=64, L=64, seed=3002),
    "mha_llama4096": MhaShape("mha_llama4096", batch=16, H=32, n=512, dh=128, L=64, seed=3003),
    "mha_l4": MhaShape("mha_l4", batch=16, H=32, n=512, dh=64, L=128, seed=3004),
}


@dataclass
class MhaInputs:
    shape: MhaShape
    Q_bits: np.ndarray    # uint16 [S, n, dh]
    K_bits: np.ndarray
    V_bits: np.ndarray
    dY_bits: np.ndarray
    C: np.ndarray         # float32 [H, M, E, 8]

    def f32(self, name: str) -> np.ndarray:
        return bf16_bits_to_f32(getattr(self, name + "_bits"))


def make_mha_inputs(shape: MhaShape) -> MhaInputs:
    def rng(stream: int) -> np.random.Generator:
        return np.random.Generator(np.random.Philox(key=shape.seed, counter=[0, 0, 0, stream]))

    S, n, dh, M, E = shape.S, shape.n, shape.dh, shape.M, shape.E
    K = rng(1).standard_normal(size=(S, n, dh), dtype=np.float32)
    V = rng(2).standard_normal(size=(S, n, dh), dtype=np.float32)
    dY = rng(3).standard_normal(size=(S, n, dh), dtype=np.float32)
    noise = rng(4).standard_normal(size=(S, n, dh), dtype=np.float32)
    pick = rng(5).integers(0, n, size=(S, n))
    Q = np.float32(0.7071) * (np.take_along_axis(K, pick[:, :, None], axis=1) + noise)
    K_bits = f32_to_bf16_bits(K)
    Kq = bf16_bits_to_f32(K_bits)
    rows = rng(6).integers(0, n, size=(shape.H, M, E))
    C = np.empty((shape.H, M, E, 8), dtype=np.float32)
    for h in range(shape.H):
        for m in range(M):
            C[h, m] = Kq[h, rows[h, m], m * 8:(m + 1) * 8]   # sequence h is batch 0, head h
    return MhaInputs(shape, f32_to_bf16_bits(Q), K_bits, f32_to_bf16_bits(V), f32_to_bf16_bits(dY), C)


def custom_mha_shape(batch, H, n, dh, L, E=16, seed=5, scale=0.0) -> MhaShape:
    return MhaShape(f"mha_b{batch}_H{H}_n{n}_dh{dh}_L{L}_E{E}", batch, H, n, dh, L, E, seed, scale)
