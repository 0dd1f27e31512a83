"""Seeded synthetic inputs for the PureKV hot path.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds no arithmetic of the method itself: it only draws random
tensors with the shapes and structure of video-LLM attention inputs (frame x
patch video tokens followed by text tokens) and rounds them to bf16 bit
patterns, so that both sides consume exactly the same bits.

Recipe (one numpy Generator per call, draw order fixed):
  1. Q[Hq, N, d]                     ~ N(0, 1)
  2. K video: frame 0 ~ N(0, 1); frame t = frame t-1 + sigma * N(0, 1)
  3. K text [Hkv, T, d]              ~ N(0, 1)
  4. V video, V text: same recipe as 2-3 with fresh draws
  5. salient set: floor(0.05 * Nv) distinct video token indices, shared by all
     KV heads; K rows at those indices are multiplied by 3 after step 2
     (the scaling does not propagate along the frame chain)
  6. decode-step tensors (q_new, k_new, v_new) ~ N(0, 1), drawn last
All values are computed in float32 and rounded once to bf16 (nearest even).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

PATTERN_DENSE = 0
PATTERN_SPATIAL = 1
PATTERN_TEMPORAL = 2
PATTERN_ST = 3


@dataclass(frozen=True)
class Workload:
    name: str
    n_frames: int
    patch_h: int
    patch_w: int
    n_text: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    sigma: float = 0.1
    ratios: Tuple[float, ...] = (0.2,)
    n_layers: int = 1
    n_dense_layers: int = 0
    decode_steps: int = 0
    seed: int = 0

    @property
    def patches(self) -> int:
        return self.patch_h * self.patch_w

    @property
    def n_video(self) -> int:
        return self.n_frames * self.patches

    @property
    def n_tokens(self) -> int:
        return self.n_video + self.n_text

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def window(self) -> int:
        """Recent window w: the trailing text tokens."""
        return self.n_text


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("tiny_4f", 4, 8, 8, 32, 2, 1, 64, decode_steps=1),
        Workload("videollama2_8f", 8, 24, 24, 128, 32, 8, 128),
        Workload("qwen25vl_32f", 32, 16, 16, 256, 28, 4, 128, decode_steps=1),
        Workload("qwen25vl_64f", 64, 16, 16, 256, 28, 4, 128, sigma=0.05,
                 ratios=(0.1, 0.2, 0.33), decode_steps=32),
        Workload("qwen25vl_128f_stack", 128, 16, 16, 512, 28, 4, 128,
                 n_layers=28, n_dense_layers=2),
    ]
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def _frame_chain(rng: np.random.Generator, heads: int, frames: int, patches: int,
                 dim: int, sigma: float) -> np.ndarray:
    x = rng.standard_normal((heads, frames, patches, dim), dtype=np.float32)
    if frames > 1:
        x[:, 1:] *= np.float32(sigma)
        np.cumsum(x, axis=1, out=x)
    return x.reshape(heads, frames * patches, dim)


@dataclass
class Inputs:
    q: np.ndarray            # uint16 [Hq, N, d]  bf16 bits
    k: np.ndarray            # uint16 [Hkv, N, d]
    v: np.ndarray            # uint16 [Hkv, N, d]
    salient: np.ndarray      # int64 [floor(0.05*Nv)] video-token indices with K scaled x3
    q_new: np.ndarray        # uint16 [steps, Hq, d]
    k_new: np.ndarray        # uint16 [steps, Hkv, d]
    v_new: np.ndarray        # uint16 [steps, Hkv, d]
    extra: dict = field(default_factory=dict)


def generate(wl: Workload, seed: int | None = None, decode_steps: int | None = None) -> Inputs:
    """Draw one layer's Q/K/V (and decode-step tensors) for a workload."""
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    hq, hkv, d = wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    n, nv, t = wl.n_tokens, wl.n_video, wl.n_text
    steps = wl.decode_steps if decode_steps is None else decode_steps

    q = rng.standard_normal((hq, n, d), dtype=np.float32)
    k = np.empty((hkv, n, d), dtype=np.float32)
    v = np.empty((hkv, n, d), dtype=np.float32)
    k[:, :nv] = _frame_chain(rng, hkv, wl.n_frames, wl.patches, d, wl.sigma)
    k[:, nv:] = rng.standard_normal((hkv, t, d), dtype=np.float32)
    v[:, :nv] = _frame_chain(rng, hkv, wl.n_frames, wl.patches, d, wl.sigma)
    v[:, nv:] = rng.standard_normal((hkv, t, d), dtype=np.float32)
    n_sal = int(np.floor(0.05 * nv))
    salient = np.sort(rng.choice(nv, size=n_sal, replace=False))
    k[:, salient] *= np.float32(3.0)
    q_new = rng.standard_normal((steps, hq, d), dtype=np.float32)
    k_new = rng.standard_normal((steps, hkv, d), dtype=np.float32)
    v_new = rng.standard_normal((steps, hkv, d), dtype=np.float32)
    return Inputs(
        q=f32_to_bf16_bits(q), k=f32_to_bf16_bits(k), v=f32_to_bf16_bits(v),
        salient=salient,
        q_new=f32_to_bf16_bits(q_new), k_new=f32_to_bf16_bits(k_new),
        v_new=f32_to_bf16_bits(v_new),
    )


def small_variant(name: str, **kw) -> Workload:
    """A custom-shaped workload for edge-case tests (ragged tails, odd patch counts)."""
    base = dict(name=name, n_frames=3, patch_h=5, patch_w=7, n_text=19,
                n_q_heads=4, n_kv_heads=2, head_dim=64)
    base.update(kw)
    return Workload(**base)
