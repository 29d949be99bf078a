"""TEST INFRASTRUCTURE ONLY: plain fp64 reference of the rotary position embedding (RoPE).

Nothing in the product path imports this module; only tests, the smoke check and the CPU baseline
of a bench may.  It shares no code with the HIP kernels.

Paper, Evaluation, "Implementation based on DistServe": besides the attention kernels the
implementation carries a RoPE kernel, modified for the Llama-3.1 models.  The paper gives no
formula; what is computed here is the published definition (the readings are listed in the design
notes):

  * RoPE: a head vector x of `dim` entries at token position p is rotated pairwise.  Pair i
    (0 <= i < rotary_dim / 2) turns by the angle p * w_i with w_i = theta ** (-2 i / rotary_dim):
        x'_a = x_a cos(p w_i) - x_b sin(p w_i)
        x'_b = x_b cos(p w_i) + x_a sin(p w_i)
    where (a, b) = (i, i + rotary_dim / 2) in the "half" layout (Llama) and (2 i, 2 i + 1) in the
    "interleaved" layout.  Entries at and beyond rotary_dim pass through unchanged.
  * Llama-3.1 frequency scaling, applied to w_i before use.  With wavelength L_i = 2 pi / w_i,
    n0 = original_max_pos, f = factor, lo = low_freq_factor, hi = high_freq_factor:
        L_i < n0 / hi  : w_i unchanged                      (high frequencies)
        L_i > n0 / lo  : w_i / f                            (low frequencies)
        otherwise      : s = (n0 / L_i - lo) / (hi - lo),   w_i' = (1 - s) w_i / f + s w_i
    factor = 1 switches the scaling off.

Results are fp64 and NOT rounded: a comparison with a bf16 kernel allows for the output rounding.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class RopeConfig:
    theta: float = 500000.0
    factor: float = 1.0
    low_freq_factor: float = 1.0
    high_freq_factor: float = 4.0
    original_max_pos: int = 8192
    rotary_dim: int = 128
    interleaved: bool = False


LLAMA31 = RopeConfig(theta=500000.0, factor=8.0, low_freq_factor=1.0, high_freq_factor=4.0, original_max_pos=8192,
                     rotary_dim=128, interleaved=False)


def inv_freq(cfg: RopeConfig) -> np.ndarray:
    """w_i (after the Llama-3.1 scaling if cfg.factor != 1), fp64 [rotary_dim / 2]."""
    if cfg.rotary_dim <= 0 or cfg.rotary_dim % 2:
        raise ValueError("rotary_dim must be positive and even")
    out = np.empty(cfg.rotary_dim // 2, dtype=np.float64)
    for i in range(cfg.rotary_dim // 2):
        w = cfg.theta ** (-2.0 * i / cfg.rotary_dim)
        if cfg.factor != 1.0:
            wavelen = 2.0 * math.pi / w
            if wavelen < cfg.original_max_pos / cfg.high_freq_factor:
                pass
            elif wavelen > cfg.original_max_pos / cfg.low_freq_factor:
                w = w / cfg.factor
            else:
                s = (cfg.original_max_pos / wavelen - cfg.low_freq_factor) / (cfg.high_freq_factor - cfg.low_freq_factor)
                w = (1.0 - s) * w / cfg.factor + s * w
        out[i] = w
    return out


def pair_index(cfg: RopeConfig):
    """(a, b) entry indices of every rotating pair."""
    half = cfg.rotary_dim // 2
    if cfg.interleaved:
        return [(2 * i, 2 * i + 1) for i in range(half)]
    return [(i, i + half) for i in range(half)]


def apply_rope(x: np.ndarray, positions, cfg: RopeConfig) -> np.ndarray:
    """x: [T, n_heads, dim] (any float dtype), positions: [T] integers.  Returns fp64 [T, n_heads, dim]."""
    x = np.asarray(x, dtype=np.float64)
    positions = np.asarray(positions)
    if x.ndim != 3 or positions.shape != (x.shape[0],):
        raise ValueError("x must be [T, heads, dim] and positions [T]")
    if cfg.rotary_dim > x.shape[2]:
        raise ValueError("rotary_dim exceeds the head dimension")
    w = inv_freq(cfg)
    out = x.copy()
    for i, (a, b) in enumerate(pair_index(cfg)):
        ang = positions.astype(np.float64) * w[i]                  # [T]
        c, s = np.cos(ang)[:, None], np.sin(ang)[:, None]
        out[:, :, a] = x[:, :, a] * c - x[:, :, b] * s
        out[:, :, b] = x[:, :, b] * c + x[:, :, a] * s
    return out
