"""Seeded synthetic inputs for the semi-PD hot path.

This module only draws random numbers and shapes them: it holds none of the
method's arithmetic (no attention, no allocator).  Both the CPU oracle's tests
and the HIP path's tests / bench take their inputs from here, so the two sides
see identical bf16-rounded values.

The paper's workloads are ShareGPT / LongBench / MATH-500 request streams served
by Llama-3 and DeepSeek models (Evaluation, Setup).  None of those datasets is
reproduced: only layer shapes and length distributions are imitated, with
values drawn from N(0, 1).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

__all__ = [
    "LayerShape", "Workload", "CONFIGS", "get_config", "to_bf16_bits", "bf16_bits_to_f32",
    "normal_bf16", "prefill_inputs", "decode_inputs", "mla_decode_inputs", "mla_prefill_inputs",
    "mla_weights", "scramble_ops", "trace", "lognormal_lengths", "uniform_lengths", "ffn_inputs", "prefill_inputs_drifting",
]


# --------------------------------------------------------------------------- bf16 helpers
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32 holding exactly that value."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    """N(0, std^2) draws rounded once to bf16; returned as uint16 bit patterns."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_bf16_bits(x)


# --------------------------------------------------------------------------- shapes
@dataclass(frozen=True)
class LayerShape:
    kind: str            # "gqa" or "mla"
    n_q_heads: int
    n_kv_heads: int      # gqa: KV heads; mla: 1 (one latent row per token)
    dim_qk: int          # gqa: head dim; mla prefill: 192 (128 nope + 64 rope)
    dim_v: int           # gqa: head dim; mla prefill: 128
    page_tokens: int
    latent_dim: int = 0  # mla: 576 = 512 (kv_lora) + 64 (rope)
    latent_v_dim: int = 0  # mla: 512

    @property
    def page_bytes(self) -> int:
        if self.kind == "mla":
            return self.page_tokens * self.latent_dim * 2
        return self.page_tokens * self.n_kv_heads * (self.dim_qk + self.dim_v) * 2


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    layer: LayerShape
    num_pages: int
    prefill_lens: Tuple[int, ...]
    decode_ctx: Tuple[int, ...]
    cu_splits: Tuple[Tuple[int, int], ...] = ((50, 50),)   # (prefill %, decode %)
    note: str = ""


def uniform_lengths(rng, n, lo, hi):
    return tuple(int(v) for v in rng.integers(lo, hi + 1, size=n))


def lognormal_lengths(rng, n, median, sigma, cap, lo=1):
    v = np.rint(np.exp(rng.normal(np.log(median), sigma, size=n)))
    return tuple(int(t) for t in np.clip(v, lo, cap))


def _c1():
    layer = LayerShape("gqa", 8, 8, 64, 64, 16)
    return Workload("c1_tiny", 1000, layer, 256, (128, 128), (200, 256, 37, 129), ((50, 50),),
                    "tiny single layer; the oracle finishes in seconds")


def _c2():
    layer = LayerShape("gqa", 32, 8, 128, 128, 16)
    rng = np.random.default_rng(1001)
    return Workload("c2_llama3_8b", 1001, layer, 40_000_000_000 // layer.page_bytes,
                    (2048,) * 4, uniform_lengths(rng, 64, 512, 4096),
                    ((30, 70), (50, 50), (70, 30)), "Llama-3-8B attention layer shape, 40 GB pool")


def _c3():
    layer = LayerShape("gqa", 64, 8, 128, 128, 16)
    rng = np.random.default_rng(1002)
    return Workload("c3_llama3_70b", 1002, layer, 40_000_000_000 // layer.page_bytes,
                    (4096,) * 8, lognormal_lengths(rng, 128, 2000, 0.8, 8192),
                    ((50, 50),), "Llama-3-70B attention layer shape, full heads on one GPU")


def _c4():
    layer = LayerShape("mla", 16, 1, 192, 128, 64, latent_dim=576, latent_v_dim=512)
    rng = np.random.default_rng(1003)
    return Workload("c4_dsv2lite_mla", 1003, layer, 40_000_000_000 // layer.page_bytes,
                    (4096,) * 4, uniform_lengths(rng, 128, 1024, 8192),
                    ((50, 50),), "DeepSeek-V2-Lite MLA layer shape, latent KV cache")


CONFIGS = {w.name: w for w in (_c1(), _c2(), _c3(), _c4())}
_ALIASES = {"c1": "c1_tiny", "c2": "c2_llama3_8b", "c3": "c3_llama3_70b", "c4": "c4_dsv2lite_mla"}


def get_config(name: str) -> Workload:
    return CONFIGS[_ALIASES.get(name, name)]


# --------------------------------------------------------------------------- tensors
def prefill_inputs(layer: LayerShape, lens, seed: int):
    """Packed variable-length Q[T,H,dqk], K[T,Hkv,dqk], V[T,Hkv,dv] as bf16 bits + cu_seqlens."""
    rng = np.random.default_rng(seed)
    T = int(sum(lens))
    q = normal_bf16(rng, (T, layer.n_q_heads, layer.dim_qk))
    k = normal_bf16(rng, (T, layer.n_kv_heads, layer.dim_qk))
    v = normal_bf16(rng, (T, layer.n_kv_heads, layer.dim_v))
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return q, k, v, cu


def prefill_inputs_drifting(layer: LayerShape, lens, seed: int, rise: float, scale: float):
    """prefill_inputs with scores that drift along the keys: entry 0 of every query is 8 and entry 0 of the key at
    position j of a prompt of length L is (j / L) * rise / (8 * scale), so scale * q.k gains `rise` (natural-log
    units; negative: loses) from the first key to the last, on top of the random part.  For softmax paths whose
    reference maximum has to move (or must not) inside a prompt."""
    q, k, v, cu = prefill_inputs(layer, lens, seed)
    qf, kf = bf16_bits_to_f32(q), bf16_bits_to_f32(k)
    qf[:, :, 0] = 8.0
    for a, b in zip(cu[:-1], cu[1:]):
        L = int(b - a)
        kf[a:b, :, 0] = (np.arange(L, dtype=np.float32) / L * np.float32(rise / (8.0 * scale)))[:, None]
    return to_bf16_bits(qf), to_bf16_bits(kf), v, cu


def decode_inputs(layer: LayerShape, ctx_lens, seed: int):
    """Per request: cached K[n,Hkv,d], V[n,Hkv,d] (bf16 bits) and one query row Q[B,H,d]."""
    rng = np.random.default_rng(seed)
    q = normal_bf16(rng, (len(ctx_lens), layer.n_q_heads, layer.dim_qk))
    ks = [normal_bf16(rng, (n, layer.n_kv_heads, layer.dim_qk)) for n in ctx_lens]
    vs = [normal_bf16(rng, (n, layer.n_kv_heads, layer.dim_v)) for n in ctx_lens]
    return q, ks, vs


# Standard deviations of absorbed / up-projected MLA tensors when weights are N(0, 0.02^2)
# and activations N(0, 1): a sum of m independent products has std 0.02*sqrt(m).
MLA_W_STD = 0.02
MLA_QABS_NOPE_STD = MLA_W_STD * np.sqrt(128.0)   # q_nope (128) projected through W_UK
MLA_UP_STD = MLA_W_STD * np.sqrt(512.0)          # latent (512) projected through W_UK / W_UV


def mla_decode_inputs(layer: LayerShape, ctx_lens, seed: int):
    """Absorbed query Qabs[B,H,576] and per-request latent cache C[n,576] (bf16 bits).

    The first 512 query dims carry the std an N(0,1) q_nope gets through an
    N(0, 0.02^2) up-projection; the last 64 (rope) dims are N(0,1).
    """
    rng = np.random.default_rng(seed)
    B, H, dl, dv = len(ctx_lens), layer.n_q_heads, layer.latent_dim, layer.latent_v_dim
    q = np.empty((B, H, dl), dtype=np.uint16)
    q[..., :dv] = normal_bf16(rng, (B, H, dv), float(MLA_QABS_NOPE_STD))
    q[..., dv:] = normal_bf16(rng, (B, H, dl - dv))
    cs = [normal_bf16(rng, (n, dl)) for n in ctx_lens]
    return q, cs


def mla_prefill_inputs(layer: LayerShape, lens, seed: int):
    """MHA-form MLA prefill: Q[T,H,192], K[T,H,192], V[T,H,128], latent[T,576] as bf16 bits.

    K's last 64 dims (rope part) are one row per token shared by all heads, as in
    the model; nope/value parts carry the up-projected std.
    """
    rng = np.random.default_rng(seed)
    T, H = int(sum(lens)), layer.n_q_heads
    rope = layer.latent_dim - layer.latent_v_dim
    nope = layer.dim_qk - rope
    q = normal_bf16(rng, (T, H, layer.dim_qk))
    k = np.empty((T, H, layer.dim_qk), dtype=np.uint16)
    k[..., :nope] = normal_bf16(rng, (T, H, nope), float(MLA_UP_STD))
    k[..., nope:] = normal_bf16(rng, (T, 1, rope))
    v = normal_bf16(rng, (T, H, layer.dim_v), float(MLA_UP_STD))
    latent = normal_bf16(rng, (T, layer.latent_dim))
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return q, k, v, latent, cu


def mla_weights(n_heads: int, nope: int, kv_lora: int, dim_v: int, seed: int):
    """W_UK[h, nope, kv_lora], W_UV[h, kv_lora, dim_v] ~ N(0, 0.02^2), float64 (not rounded)."""
    rng = np.random.default_rng(seed)
    w_uk = rng.normal(0.0, MLA_W_STD, size=(n_heads, nope, kv_lora))
    w_uv = rng.normal(0.0, MLA_W_STD, size=(n_heads, kv_lora, dim_v))
    return w_uk, w_uv


def ffn_inputs(n_tokens: int, hidden: int, inter: int, seed: int):
    """Inputs of the gated FFN's first step: activations x [T, hidden] ~ N(0, 1) (a normalised hidden state),
    weights W_gate, W_up [inter, hidden] ~ N(0, 1 / hidden) (so that the projections are of order one, as after
    a trained layer's scaling); all rounded once to bf16, returned as uint16 bit patterns."""
    rng = np.random.default_rng(seed)
    x = normal_bf16(rng, (n_tokens, hidden))
    w_gate = normal_bf16(rng, (inter, hidden), std=hidden ** -0.5)
    w_up = normal_bf16(rng, (inter, hidden), std=hidden ** -0.5)
    return x, w_gate, w_up


# --------------------------------------------------------------------------- allocator op streams
def scramble_ops(num_pages_touched: int, page_tokens: int, seed: int, first_req_id: int = 1 << 40):
    """Op list that leaves a LIFO free list in a seeded random order.

    Reserves `num_pages_touched` one-page requests and frees them in a random
    order, so later reservations receive scattered physical pages (the state of
    a pool after long serving).  Ops are ("reserve", req_id, n_tokens) and
    ("free", req_id, 0); any allocator can execute them.
    """
    rng = np.random.default_rng(seed)
    ids = [first_req_id + i for i in range(num_pages_touched)]
    ops = [("reserve", r, page_tokens) for r in ids]
    for i in rng.permutation(num_pages_touched):
        ops.append(("free", ids[int(i)], 0))
    return ops


@dataclass
class Trace:
    arrival_s: np.ndarray   # float64 [N], non-decreasing
    input_len: np.ndarray   # int32 [N]
    output_len: np.ndarray  # int32 [N]


def trace(n_requests: int = 2000, rate_per_s: float = 8.0, seed: int = 1004,
          in_median: int = 1024, in_cap: int = 8192, out_median: int = 256, out_cap: int = 2048,
          sigma: float = 0.8) -> Trace:
    """Poisson arrivals with lognormal input / output lengths (dynamic mixed trace)."""
    rng = np.random.default_rng(seed)
    arrival = np.cumsum(rng.exponential(1.0 / rate_per_s, size=n_requests))
    ins = np.asarray(lognormal_lengths(rng, n_requests, in_median, sigma, in_cap), dtype=np.int32)
    outs = np.asarray(lognormal_lengths(rng, n_requests, out_median, sigma, out_cap), dtype=np.int32)
    return Trace(arrival, ins, outs)
