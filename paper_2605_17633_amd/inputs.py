"""Seeded synthetic inputs shaped like SAM's ViT encoders.

This module holds none of the method's arithmetic: it only draws random arrays
(numpy ``default_rng``), rounds them to bf16-representable fp32 values and names
the model shapes.  It is the one module both the CPU oracle's tests and the HIP
path's tests/benchmark use, so that both sides see identical arrays.

The paper evaluates on MS-COCO / HQ-44K images through trained SAM checkpoints
(Sec. 5.1); neither is available here and, because the sparsity pattern is
static, run time does not depend on content.  These generators stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    D: int            # model width
    depth: int        # number of blocks
    heads: int
    Dm: int           # MLP hidden width
    global_blocks: tuple
    ws: int = 14      # window side of the local blocks

    @property
    def d(self) -> int:
        return self.D // self.heads


VIT_B = ModelShape("vit_b", 768, 12, 12, 3072, (2, 5, 8, 11))
VIT_L = ModelShape("vit_l", 1024, 24, 16, 4096, (5, 11, 17, 23))
VIT_H = ModelShape("vit_h", 1280, 32, 16, 5120, (7, 15, 23, 31))
SHAPES = {s.name: s for s in (VIT_B, VIT_L, VIT_H)}


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def block_weights(rng: np.random.Generator, D: int, heads: int, Dm: int, w: int) -> dict:
    """Weights of one encoder block as fp32 arrays holding bf16-representable
    values (LayerNorm parameters and biases are kept in full fp32).
    ``w`` is the side of the attention group the rel-pos tables serve (window
    side for local blocks, grid side for global blocks)."""
    d = D // heads
    n = lambda *s: rng.normal(0.0, 0.02, size=s).astype(np.float32)
    return {
        "ln1_g": (1.0 + n(D)).astype(np.float32), "ln1_b": n(D),
        "wqkv": bf16_round(n(3 * D, D)), "bqkv": n(3 * D),
        "rel_h": bf16_round(n(2 * w - 1, d)), "rel_w": bf16_round(n(2 * w - 1, d)),
        "wproj": bf16_round(n(D, D)), "bproj": n(D),
        "ln2_g": (1.0 + n(D)).astype(np.float32), "ln2_b": n(D),
        "w1": bf16_round(n(Dm, D)), "b1": n(Dm),
        "w2": bf16_round(n(D, Dm)), "b2": n(D),
    }


def token_field(rng: np.random.Generator, B: int, g: int, D: int, noise: float = 0.3) -> np.ndarray:
    """[B,g,g,D] tokens: per image 8 random low-frequency 2-D sinusoids mixed into
    the channels with non-zero-mean gains, plus Gaussian noise, so that the
    channel sum keeps spatial structure and token scores vary over the grid."""
    ii, jj = np.meshgrid(np.arange(g), np.arange(g), indexing="ij")
    A = (rng.normal(0.5, 1.0, size=(8, D)) / np.sqrt(8.0)).astype(np.float32)
    x = np.empty((B, g, g, D), np.float32)
    for b in range(B):
        u = rng.uniform(-3, 3, 8)
        v = rng.uniform(-3, 3, 8)
        ph = rng.uniform(0, 2 * np.pi, 8)
        f = np.sin(2 * np.pi * (u[:, None, None] * ii / g + v[:, None, None] * jj / g)
                   + ph[:, None, None]).astype(np.float32)          # [8,g,g]
        x[b] = np.einsum("mij,mc->ijc", f, A) + noise * rng.normal(size=(g, g, D)).astype(np.float32)
    return bf16_round(x)


def lognormal_scores(rng: np.random.Generator, B: int, n: int) -> np.ndarray:
    """Heavy-tailed token scores exp(N(0,1)), fp32 [B,n]."""
    return np.exp(rng.normal(size=(B, n))).astype(np.float32)


def qkv_tensors(rng: np.random.Generator, groups: int, S: int, heads: int, d: int,
                scale: float = 0.7) -> np.ndarray:
    """Packed qkv activations [groups,S,3,heads,d] ~ N(0,scale^2), bf16-rounded."""
    return bf16_round(rng.normal(0.0, scale, size=(groups, S, 3, heads, d)).astype(np.float32))


def encoder_weights(seed: int, shape: ModelShape, g: int, depth: int | None = None) -> list:
    """One dict per block; global blocks get rel-pos tables for the g x g grid."""
    rng = np.random.default_rng(seed)
    depth = shape.depth if depth is None else depth
    out = []
    for i in range(depth):
        w = g if i in shape.global_blocks else shape.ws
        out.append(block_weights(rng, shape.D, shape.heads, shape.Dm, w))
    return out
