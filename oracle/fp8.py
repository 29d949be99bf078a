"""CPU oracle for the FP8 latent KV cache.  TEST INFRASTRUCTURE ONLY (see oracle/attention.py): nothing in the
product path imports this module, and it shares no code with the HIP path.

Paper, Evaluation "Model": DeepSeek-V3 is served "with FP8 precision"; the paper says no more.  The reading taken
here for the KV cache of the latent (MLA) path:

* values are OCP FP8 E4M3 ("e4m3fn": 1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities; the two
  codes S.1111.111 are NaN; largest finite value 448; subnormals m / 8 * 2^-6);
* a cached latent row c = [ckv (512) ; krope (64)] keeps its 64 rope entries in bf16 as they are and its 512 ckv
  entries as FP8 codes with one fp32 scale per block of 128 consecutive entries:
      scale_b = amax_b / 448   (amax_b = largest magnitude in the block; 1 if the block is all zero),
      code_i  = E4M3(clamp(x_i / scale_b, -448, 448)),   rounding to nearest, ties to the even code,
  both the division and the scale in fp32 (the precision the kernel works in: the codes are compared bit for bit);
* the dequantised value is decode(code_i) * scale_b.  The attention oracle runs on the dequantised rows.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0
BLOCK = 128          # entries per scale
KV_LORA = 512        # quantised entries of a latent row
ROPE = 64            # entries kept in bf16


def e4m3_decode_table() -> np.ndarray:
    """value of each of the 256 codes (float64; NaN for 0x7f and 0xff), from the format's definition"""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = (m / 8.0) * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[code] = -v if s else v
    return t


_TABLE = e4m3_decode_table()
_POS = _TABLE[:127]                      # codes 0x00 .. 0x7e: 0 .. 448, increasing


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    return _TABLE[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """nearest code, ties to the even code, magnitudes beyond 448 saturate; x finite"""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")            # first code with value >= a
    hi = np.clip(hi, 0, 126)
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = _POS[hi] - a, a - _POS[lo]
    take_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(take_lo, lo, hi).astype(np.uint8)
    return np.where(np.signbit(x) & (a > 0), code | 0x80, code).astype(np.uint8)


def quantise_latent(latent_f32: np.ndarray):
    """latent [n, 576] (values exactly representable in fp32, e.g. bf16) -> codes [n, 512] uint8, scales [n, 4] fp32,
    rope [n, 64] (unchanged)"""
    x = np.asarray(latent_f32, dtype=np.float32)
    n = x.shape[0]
    blocks = x[:, :KV_LORA].reshape(n, KV_LORA // BLOCK, BLOCK)
    amax = np.abs(blocks).max(axis=2)
    scale = np.where(amax > 0, amax / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)      # fp32 division
    y = (blocks / scale[:, :, None]).astype(np.float32)                                              # fp32 division
    y = np.clip(y, np.float32(-E4M3_MAX), np.float32(E4M3_MAX))
    codes = e4m3_encode(y.astype(np.float64)).reshape(n, KV_LORA)
    return codes, scale, x[:, KV_LORA:].copy()


def dequantise_latent(codes: np.ndarray, scale: np.ndarray, rope: np.ndarray) -> np.ndarray:
    """the rows the attention sees: [n, 576] float64"""
    n = codes.shape[0]
    v = e4m3_decode(codes).reshape(n, KV_LORA // BLOCK, BLOCK) * np.asarray(scale, dtype=np.float64)[:, :, None]
    return np.concatenate([v.reshape(n, KV_LORA), np.asarray(rope, dtype=np.float64)], axis=1)


def pack_rows(codes: np.ndarray, scale: np.ndarray, rope_bits: np.ndarray) -> np.ndarray:
    """a cached row as bytes: 512 codes, 4 fp32 scales (little endian), 64 bf16 rope entries = 656 bytes"""
    n = codes.shape[0]
    out = np.empty((n, KV_LORA + 16 + 2 * ROPE), dtype=np.uint8)
    out[:, :KV_LORA] = codes
    out[:, KV_LORA:KV_LORA + 16] = np.ascontiguousarray(scale, dtype="<f4").view(np.uint8).reshape(n, 16)
    out[:, KV_LORA + 16:] = np.ascontiguousarray(rope_bits, dtype="<u2").view(np.uint8).reshape(n, 2 * ROPE)
    return out
