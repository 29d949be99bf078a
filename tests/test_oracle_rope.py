"""Pins of the fp64 RoPE oracle against what the definition and the mathematics fix (no GPU).

Paper, Evaluation "Implementation based on DistServe": the RoPE kernel (modified for Llama-3.1)."""
import cmath
import math
import os

import numpy as np
import pytest

from oracle import rope as R

HERE = os.path.dirname(__file__)


def _golden():
    cases = []
    for line in open(os.path.join(HERE, "golden", "rope_small.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, *kv = line.split()
        d = dict(item.split("=") for item in kv)
        cases.append((name, d))
    return cases


@pytest.mark.parametrize("name,d", _golden())
def test_hand_worked_cases(name, d):
    cfg = R.RopeConfig(theta=float(d["theta"]), rotary_dim=int(d["dim"]), interleaved=d.get("interleaved", "0") == "1")
    x = np.array([float(t) for t in d["x"].split(",")]).reshape(1, 1, -1)
    want = np.array([float(t) for t in d["want"].split(",")])
    got = R.apply_rope(x, [int(d["pos"])], cfg)[0, 0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)


def test_position_zero_is_identity_and_tail_passes_through():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 3, 16))
    cfg = R.RopeConfig(theta=10000.0, rotary_dim=8)
    np.testing.assert_array_equal(R.apply_rope(x, np.zeros(5, dtype=np.int64), cfg), x)
    y = R.apply_rope(x, np.arange(5) * 7 + 1, cfg)
    np.testing.assert_array_equal(y[:, :, 8:], x[:, :, 8:])          # beyond rotary_dim: untouched
    assert np.abs(y[:, :, :8] - x[:, :, :8]).max() > 1e-3


@pytest.mark.parametrize("interleaved", [False, True])
def test_equals_complex_multiplication(interleaved):
    # an independent formulation: each pair is a complex number multiplied by exp(i p w)
    rng = np.random.default_rng(2)
    cfg = R.RopeConfig(theta=500000.0, rotary_dim=12, interleaved=interleaved)
    x = rng.standard_normal((4, 2, 12))
    pos = [3, 11, 4095, 131071]
    y = R.apply_rope(x, pos, cfg)
    for t in range(4):
        for h in range(2):
            for i in range(6):
                a, b = (2 * i, 2 * i + 1) if interleaved else (i, i + 6)
                w = 500000.0 ** (-2.0 * i / 12)
                z = complex(x[t, h, a], x[t, h, b]) * cmath.exp(1j * pos[t] * w)
                assert abs(y[t, h, a] - z.real) < 1e-9 and abs(y[t, h, b] - z.imag) < 1e-9


def test_rotation_keeps_every_pairs_norm():
    rng = np.random.default_rng(3)
    cfg = R.LLAMA31
    x = rng.standard_normal((6, 2, 128))
    y = R.apply_rope(x, [0, 1, 17, 8191, 8192, 100000], cfg)
    for a, b in R.pair_index(cfg):
        np.testing.assert_allclose(y[:, :, a] ** 2 + y[:, :, b] ** 2, x[:, :, a] ** 2 + x[:, :, b] ** 2, rtol=1e-12)


@pytest.mark.parametrize("cfg", [R.RopeConfig(theta=10000.0, rotary_dim=64), R.LLAMA31])
def test_scores_depend_on_the_position_difference_only(cfg):
    # <rope(q, m), rope(k, n)> = <rope(q, m - n), k>: the property attention relies on
    rng = np.random.default_rng(4)
    d = cfg.rotary_dim
    q, k = rng.standard_normal((1, 1, d)), rng.standard_normal((1, 1, d))
    for m, n in [(5, 3), (1000, 1), (70000, 69000), (12, 12)]:
        lhs = float(np.sum(R.apply_rope(q, [m], cfg) * R.apply_rope(k, [n], cfg)))
        rhs = float(np.sum(R.apply_rope(q, [m - n], cfg) * k))
        assert abs(lhs - rhs) < 1e-9 * (1 + abs(rhs))


def test_layouts_differ_by_a_permutation_only():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 2, 8))
    pos = [1, 50, 999]
    half = R.apply_rope(x, pos, R.RopeConfig(theta=10000.0, rotary_dim=8, interleaved=False))
    perm = [0, 4, 1, 5, 2, 6, 3, 7]            # interleaved entry j holds half-layout entry perm[j]
    inter = R.apply_rope(x[:, :, perm], pos, R.RopeConfig(theta=10000.0, rotary_dim=8, interleaved=True))
    np.testing.assert_allclose(inter, half[:, :, perm], rtol=0, atol=1e-14)


def test_unscaled_frequencies_are_the_geometric_sequence():
    w = R.inv_freq(R.RopeConfig(theta=10000.0, rotary_dim=8))
    np.testing.assert_allclose(w, [1.0, 0.1, 0.01, 0.001], rtol=1e-14)


def test_llama31_scaling_bands():
    # theta 5e5, dim 128, n0 8192, hi 4, lo 1: wavelength 2 pi 5e5^(i/64) is below 2048 for i <= 28,
    # above 8192 for i >= 35 (closed form: i < 64 ln(2048 / 2 pi) / ln 5e5 = 28.2, i > 64 ln(8192 / 2 pi) / ln 5e5 = 34.98)
    plain = R.inv_freq(R.RopeConfig(theta=500000.0, rotary_dim=128))
    scaled = R.inv_freq(R.LLAMA31)
    ratio = scaled / plain
    np.testing.assert_array_equal(ratio[:29], np.ones(29))
    np.testing.assert_allclose(ratio[35:], np.full(29, 0.125), rtol=1e-15)
    mid = ratio[29:35]
    assert np.all(mid > 0.125) and np.all(mid < 1.0) and np.all(np.diff(mid) < 0)   # smooth, falling towards 1/8
    assert np.all(np.diff(scaled) < 0)                                                # still a falling sequence


def test_llama31_interpolation_at_a_chosen_wavelength():
    # a frequency whose wavelength is n0 / 2.5: s = (2.5 - 1) / (4 - 1) = 0.5, so w' = w (0.5 + 0.5 / 8) = 0.5625 w
    n0 = 8192
    w_target = 2.0 * math.pi / (n0 / 2.5)
    theta = w_target ** -2.0                      # dim 4: w_1 = theta^(-1/2)
    cfg = R.RopeConfig(theta=theta, factor=8.0, low_freq_factor=1.0, high_freq_factor=4.0, original_max_pos=n0, rotary_dim=4)
    w = R.inv_freq(cfg)
    assert w[0] == 1.0                            # wavelength 2 pi: far in the high band
    assert abs(w[1] / w_target - 0.5625) < 1e-12
    # and the two band edges: just inside the high band nothing changes, just inside the low band 1/8
    for frac, want in [(4.0 * 1.0001, 1.0), (1.0 / 1.0001, 0.125)]:
        wt = 2.0 * math.pi / (n0 / frac)
        c = R.RopeConfig(theta=wt ** -2.0, factor=8.0, original_max_pos=n0, rotary_dim=4)
        assert abs(R.inv_freq(c)[1] / wt - want) < 1e-12


def test_argument_checks():
    with pytest.raises(ValueError):
        R.inv_freq(R.RopeConfig(rotary_dim=3))
    with pytest.raises(ValueError):
        R.apply_rope(np.zeros((2, 1, 4)), [0], R.RopeConfig(rotary_dim=4))
    with pytest.raises(ValueError):
        R.apply_rope(np.zeros((1, 1, 4)), [0], R.RopeConfig(rotary_dim=8))
