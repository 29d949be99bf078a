"""Pins of the FP8 (E4M3) oracle: values the format's definition fixes, the library conversion of PyTorch on the
CPU as an independent implementation, brute force, and the error bound of the block scaling."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import fp8 as F


def test_decode_table_values_fixed_by_the_format():
    t = F.e4m3_decode_table()
    assert t[0x00] == 0.0 and t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9          # subnormals m / 8 * 2^-6
    assert t[0x08] == 2.0 ** -6                                                           # smallest normal
    assert t[0x38] == 1.0 and t[0x39] == 1.125 and t[0x40] == 2.0 and t[0xB8] == -1.0
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0                                         # largest finite
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(t).sum() == 254       # no infinities, two NaNs
    assert (np.diff(t[:127]) > 0).all()
    # the library's table, code by code
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    np.testing.assert_array_equal(np.nan_to_num(t, nan=12345.0), np.nan_to_num(lib, nan=12345.0))


def test_encode_is_the_inverse_on_codes_and_rounds_to_nearest_even():
    t = F.e4m3_decode_table()
    finite = np.array([c for c in range(256) if np.isfinite(t[c]) and c != 0x80], dtype=np.uint8)
    np.testing.assert_array_equal(F.e4m3_encode(t[finite]), finite)
    # ties go to the even code
    assert F.e4m3_encode(np.array([1.0625]))[0] == 0x38 and F.e4m3_encode(np.array([1.1875]))[0] == 0x3A
    assert F.e4m3_encode(np.array([-1.0625]))[0] == 0xB8
    assert F.e4m3_encode(np.array([2.0 ** -10]))[0] == 0x00 and F.e4m3_encode(np.array([3 * 2.0 ** -10]))[0] == 0x02
    # saturation instead of NaN
    np.testing.assert_array_equal(F.e4m3_encode(np.array([449.0, 1e9, -500.0])), [0x7E, 0x7E, 0xFE])
    # brute force: the nearest table entry by exhaustive search
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.normal(0, 1, 4000), rng.normal(0, 100, 4000), rng.uniform(-2.0 ** -5, 2.0 ** -5, 4000)])
    x = np.clip(x, -448, 448)
    got = F.e4m3_decode(F.e4m3_encode(x))
    pos = t[:127]
    best = np.abs(np.abs(x)[:, None] - pos[None, :]).min(axis=1)
    np.testing.assert_allclose(np.abs(np.abs(got) - np.abs(x)), best, rtol=0, atol=0)
    assert (np.sign(got) == np.sign(x))[got != 0].all()
    # the library conversion (round to nearest even, in range)
    lib = torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ours = F.e4m3_encode(x.astype(np.float32).astype(np.float64))
    same_value = F.e4m3_decode(lib) == F.e4m3_decode(ours)          # +0 and -0 are one value
    assert same_value.all()


def test_block_scaled_rows_reconstruct_within_half_a_step():
    rng = np.random.default_rng(2)
    lat = W.bf16_bits_to_f32(W.normal_bf16(rng, (40, 576)))
    lat[3, :128] = 0.0                                               # an all-zero block: scale 1, codes 0
    lat[5, 130] = 300.0                                              # an outlier sets its block's scale
    codes, scale, rope = F.quantise_latent(lat)
    assert codes.shape == (40, 512) and scale.shape == (40, 4) and scale.dtype == np.float32
    assert scale[3, 0] == 1.0 and (codes[3, :128] == 0).all()
    np.testing.assert_array_equal(rope, lat[:, 512:])
    amax = np.abs(lat[:, :512]).reshape(40, 4, 128).max(axis=2)
    np.testing.assert_allclose(scale[amax > 0], (amax / 448.0)[amax > 0], rtol=2.0 ** -23)
    # the largest entry of every block maps to +-448 exactly
    assert (np.abs(F.e4m3_decode(codes)).reshape(40, 4, 128).max(axis=2)[amax > 0] == 448.0).all()
    deq = F.dequantise_latent(codes, scale, rope)
    err = np.abs(deq[:, :512] - lat[:, :512]).reshape(40, 4, 128)
    # a normal E4M3 value is within 2^-4 of its own magnitude; below the smallest normal the step is 2^-9 (in units of the scale)
    bound = np.maximum(2.0 ** -4 * np.abs(lat[:, :512]).reshape(40, 4, 128), 2.0 ** -10 * scale[:, :, None]) * (1 + 1e-6)
    assert (err <= bound).all()
    assert deq[5, 130] == pytest.approx(300.0, rel=1e-6)
    # packed rows: 656 bytes, fields where the layout says
    rows = F.pack_rows(codes, scale, W.to_bf16_bits(lat[:, 512:]))
    assert rows.shape == (40, 656)
    np.testing.assert_array_equal(rows[:, :512], codes)
    np.testing.assert_array_equal(rows[:, 512:528].copy().view("<f4").reshape(40, 4), scale)
    np.testing.assert_array_equal(rows[:, 528:].copy().view("<u2").reshape(40, 64), W.to_bf16_bits(lat[:, 512:]))
