"""Seeded synthetic inputs for the denoising hot path (shapes, weights, latents).

This module holds data recipes only: network shapes, the order and shapes of the
weight list, Gaussian draws, and the storage rounding to bf16.  None of the
method's arithmetic (no predictor, scheduler, attention or metric) lives here, so
both the CPU oracle's tests and the HIP path's tests may draw their inputs from it.

The paper drives trained models with dataset prompts; a denoising run itself only
consumes x_T ~ N(0, I) (Algorithm 1, initialisation), a conditioning tensor and the
predictor's weights.  Here the conditioning tensor is N(0,1) text-token embeddings
and the weights are Gaussian, so every input is synthetic and reproducible.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class DiTConfig:
    """Shape of the DiT noise predictor and of the latent it denoises."""

    layers: int
    hidden: int
    heads: int
    head_dim: int
    mlp_ratio: int
    in_channels: int
    patch: int
    frames: int
    height: int          # latent height (pixels of the latent, not patches)
    width: int
    text_tokens: int
    time_embed_dim: int
    dtype: str           # "f32" or "bf16": storage/operand type of matrices
    ln_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def grid(self) -> Tuple[int, int, int]:
        return (self.frames, self.height // self.patch, self.width // self.patch)

    @property
    def video_tokens(self) -> int:
        f, hp, wp = self.grid
        return f * hp * wp

    @property
    def tokens(self) -> int:
        return self.text_tokens + self.video_tokens

    @property
    def patch_dim(self) -> int:
        return self.in_channels * self.patch * self.patch

    @property
    def latent_shape(self) -> Tuple[int, int, int, int]:
        return (self.in_channels, self.frames, self.height, self.width)

    @property
    def latent_elems(self) -> int:
        c, f, h, w = self.latent_shape
        return c * f * h * w

    def with_(self, **kw) -> "DiTConfig":
        return replace(self, **kw)


def _cogvideox(frames: int, height: int, width: int, layers: int = 30) -> DiTConfig:
    return DiTConfig(layers=layers, hidden=1920, heads=30, head_dim=64, mlp_ratio=4,
                     in_channels=16, patch=2, frames=frames, height=height, width=width,
                     text_tokens=226, time_embed_dim=512, dtype="bf16")


# Named workloads.  "tiny" is the fp32 case the oracle finishes in seconds; "block"
# is one layer at CogVideoX-2b width on 4290 video + 226 text tokens; "full" is the
# 30-layer network on the 13x60x90 latent (17550 + 226 tokens); "long" is the
# 25-frame latent (33750 + 226 tokens); "reduced" keeps the 30 layers and the width
# but few tokens so the oracle can run the whole model.
CONFIGS: Dict[str, DiTConfig] = {
    "tiny": DiTConfig(layers=2, hidden=64, heads=4, head_dim=16, mlp_ratio=4,
                      in_channels=4, patch=2, frames=2, height=16, width=16,
                      text_tokens=0, time_embed_dim=64, dtype="f32"),
    "tiny_text": DiTConfig(layers=2, hidden=64, heads=4, head_dim=16, mlp_ratio=4,
                           in_channels=4, patch=2, frames=2, height=16, width=16,
                           text_tokens=6, time_embed_dim=64, dtype="f32"),
    "block": _cogvideox(13, 30, 44, layers=1),
    "full": _cogvideox(13, 60, 90),
    "long": _cogvideox(25, 60, 90),
    "reduced": _cogvideox(2, 12, 16).with_(text_tokens=16),
}

# Per-workload seeds: weights 1000 + index, x_T 42, text embeddings 7,
# stand-alone attention q/k/v 11/12/13.
WEIGHT_SEED = {"tiny": 1001, "tiny_text": 1001, "block": 1002, "full": 1003,
               "long": 1004, "reduced": 1003}
SEED_XT = 42
SEED_CTX = 7
SEED_QKV = (11, 12, 13)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even).

    Returned array is still float32; every element fits bf16 exactly, so a later
    cast to a bf16 device tensor loses nothing and both sides see the same numbers.
    """
    a = np.array(a, dtype=np.float32, order="C", copy=True)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    lsb += np.uint32(0x7FFF)
    u += lsb                      # finite inputs cannot wrap: the exponent absorbs the carry
    u &= np.uint32(0xFFFF0000)
    return a


def weight_shapes(cfg: DiTConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the weight list, in the order the library expects.

    All matrices are row-major [out_features, in_features].
    """
    D, Dt, P = cfg.hidden, cfg.time_embed_dim, cfg.patch_dim
    out: List[Tuple[str, Tuple[int, ...]]] = [
        ("W_pe", (D, P)), ("b_pe", (D,)),
        ("W_t1", (Dt, D)), ("b_t1", (Dt,)),
        ("W_t2", (Dt, Dt)), ("b_t2", (Dt,)),
    ]
    for l in range(cfg.layers):
        out += [
            (f"W_mod.{l}", (12 * D, Dt)), (f"b_mod.{l}", (12 * D,)),
            (f"W_qkv.{l}", (3 * D, D)), (f"b_qkv.{l}", (3 * D,)),
            (f"W_o.{l}", (D, D)), (f"b_o.{l}", (D,)),
            (f"W_1.{l}", (cfg.mlp_ratio * D, D)), (f"b_1.{l}", (cfg.mlp_ratio * D,)),
            (f"W_2.{l}", (D, cfg.mlp_ratio * D)), (f"b_2.{l}", (D,)),
        ]
    out += [("W_fm", (2 * D, Dt)), ("b_fm", (2 * D,)),
            ("W_out", (P, D)), ("b_out", (P,))]
    return out


def make_weights(cfg: DiTConfig, seed: int, init: str = "std002") -> List[Tuple[str, np.ndarray]]:
    """Draw every weight; tensor number i of the list comes from default_rng([seed, i]).

    init="std002": matrices and biases i.i.d. N(0, 0.02^2).
    init="unit":   matrices N(0, 1/fan_in), biases N(0, 0.02^2), and +1 added to the
                   four gate chunks of every block's modulation bias, so that logits,
                   gates and activations are O(1) and every sub-layer matters.
    Matrices are rounded to bf16-representable values when cfg.dtype == "bf16";
    biases stay fp32.  Tensors are independent streams, so they are drawn in parallel
    threads (the 30-layer network has 1.7e9 parameters).
    """
    if init not in ("std002", "unit"):
        raise ValueError(init)
    D = cfg.hidden
    shapes = weight_shapes(cfg)

    def draw(i):
        name, shape = shapes[i]
        w = np.random.default_rng([seed, i]).standard_normal(shape, dtype=np.float32)
        if len(shape) == 2:
            w *= np.float32(0.02 if init == "std002" else 1.0 / np.sqrt(shape[1]))
            if cfg.dtype == "bf16":
                w = round_to_bf16(w)
        else:
            w *= np.float32(0.02)
            if init == "unit" and name.startswith("b_mod."):
                for chunk in (2, 5, 8, 11):
                    w[chunk * D:(chunk + 1) * D] += np.float32(1.0)
        return name, w

    workers = max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(draw, range(len(shapes))))


def make_latent(cfg: DiTConfig, batch: int = 1, seed: int = SEED_XT) -> np.ndarray:
    """x_T ~ N(0, I), fp32, shape [B, C, F, H, W]."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((batch,) + cfg.latent_shape).astype(np.float32)


def make_context(cfg: DiTConfig, batch: int = 1, seed: int = SEED_CTX):
    """N(0,1) text-token embeddings [B, L_txt, D] (None when the config has no text).

    Rounded to bf16-representable values for bf16 configs.
    """
    if cfg.text_tokens == 0:
        return None
    rng = np.random.default_rng(seed)
    c = rng.standard_normal((batch, cfg.text_tokens, cfg.hidden)).astype(np.float32)
    return round_to_bf16(c) if cfg.dtype == "bf16" else c


def make_qkv(batch: int, seq: int, heads: int, head_dim: int, dtype: str = "bf16",
             seeds=SEED_QKV, scale: float = 1.0):
    """N(0, scale^2) q, k, v of shape [B, N, H, d] for the stand-alone attention call."""
    out = []
    for s in seeds:
        rng = np.random.default_rng(s)
        a = (rng.standard_normal((batch, seq, heads, head_dim)) * scale).astype(np.float32)
        out.append(round_to_bf16(a) if dtype == "bf16" else a)
    return tuple(out)


def make_tokens(rows: int, cols: int, seed: int, dtype: str = "bf16") -> np.ndarray:
    """N(0,1) activation matrix [rows, cols] (block-level and GEMM-level cases)."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((rows, cols)).astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a
