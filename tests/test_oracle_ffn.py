"""Pins of the fp64 gated-FFN oracle against what the definition and the mathematics fix (no GPU).

Paper, Evaluation "Implementation based on DistServe": the first two GEMMs of the gated FFN fused into one."""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import ffn as F

HERE = os.path.dirname(__file__)


def _golden():
    cases = []
    for line in open(os.path.join(HERE, "golden", "ffn_small.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, *kv = line.split()
        d = dict(item.split("=") for item in kv)
        cases.append((name, d))
    return cases


def _mat(s):
    return np.array([[float(t) for t in row.split(",")] for row in s.split(";")])


@pytest.mark.parametrize("name,d", _golden())
def test_hand_worked_cases(name, d):
    x = _mat(d["x"])
    want = np.array([float(t) for t in d["want"].split(",")])
    got = F.gate_up(x, _mat(d["wg"]), _mat(d["wu"]))[0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)


def test_silu_against_the_logistic_function_and_its_symmetry():
    z = np.linspace(-30, 30, 241)
    np.testing.assert_allclose(F.silu(z), z * scipy.special.expit(z), rtol=1e-14, atol=0)
    np.testing.assert_allclose(F.silu(z) - F.silu(-z), z, rtol=1e-13, atol=1e-15)     # silu(z) - silu(-z) = z
    assert F.silu(np.array([0.0]))[0] == 0.0
    assert abs(F.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-16
    assert abs(F.silu(np.array([40.0]))[0] - 40.0) < 1e-12 and abs(F.silu(np.array([-40.0]))[0]) < 1e-15


def test_against_a_triple_loop():
    rng = np.random.default_rng(3)
    T, K, I = 3, 5, 4
    x, wg, wu = rng.standard_normal((T, K)), rng.standard_normal((I, K)), rng.standard_normal((I, K))
    got = F.gate_up(x, wg, wu)
    for t in range(T):
        for n in range(I):
            g = sum(x[t, k] * wg[n, k] for k in range(K))
            u = sum(x[t, k] * wu[n, k] for k in range(K))
            assert abs(got[t, n] - g / (1.0 + math.exp(-g)) * u) < 1e-13


def test_operands_are_not_transposed_or_swapped():
    # a gate row that selects one input, an up row that selects another: out = silu(x_a) * x_b
    x = np.array([[0.5, -2.0, 3.0]])
    wg = np.array([[0.0, 0.0, 1.0], [1.0, 0.0, 0.0]])
    wu = np.array([[0.0, 1.0, 0.0], [0.0, 0.0, 1.0]])
    want = [F.silu(np.array([3.0]))[0] * -2.0, F.silu(np.array([0.5]))[0] * 3.0]
    np.testing.assert_allclose(F.gate_up(x, wg, wu)[0], want, rtol=1e-15)
    # swapping gate and up changes the result (silu is applied to the gate only)
    assert np.abs(F.gate_up(x, wu, wg)[0] - want).max() > 0.1


def test_linear_in_up_and_zero_cases():
    rng = np.random.default_rng(4)
    x, wg, wu = rng.standard_normal((6, 8)), rng.standard_normal((32, 8)), rng.standard_normal((32, 8))
    base = F.gate_up(x, wg, wu)
    np.testing.assert_allclose(F.gate_up(x, wg, 3.0 * wu), 3.0 * base, rtol=1e-13)
    np.testing.assert_array_equal(F.gate_up(x, np.zeros_like(wg), wu), np.zeros_like(base))     # silu(0) = 0
    np.testing.assert_array_equal(F.gate_up(np.zeros_like(x), wg, wu), np.zeros_like(base))


def test_joint_rows_and_single_product_give_the_same():
    rng = np.random.default_rng(5)
    x, wg, wu = rng.standard_normal((7, 16)), rng.standard_normal((96, 16)), rng.standard_normal((96, 16))
    w = F.joint_rows(wg, wu)
    assert w.shape == (192, 16)
    # row order: 32 gate rows, the 32 up rows of the same outputs, and so on
    for b in range(3):
        np.testing.assert_array_equal(w[64 * b:64 * b + 32], wg[32 * b:32 * b + 32])
        np.testing.assert_array_equal(w[64 * b + 32:64 * b + 64], wu[32 * b:32 * b + 32])
    np.testing.assert_allclose(F.gate_up_joint(x, w), F.gate_up(x, wg, wu), rtol=1e-13, atol=1e-15)
    with pytest.raises(ValueError):
        F.joint_rows(wg[:40], wu[:40])


def test_packed_weight_reader_follows_the_header_formula():
    # the reader the GPU tests use for spd_ffn_pack_gate_up's output, on an array whose elements are their own
    # flat positions: spots worked out by hand from the formula in include/semipd.h
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from ffn_layout import unpack_gate_up
    inter, hidden = 256, 96
    packed = np.arange(2 * inter * hidden, dtype=np.int64)
    g, u = unpack_gate_up(packed, hidden)
    assert sorted(np.concatenate([g.ravel(), u.ravel()]).tolist()) == packed.tolist()           # a permutation
    n_ks = hidden // 32
    # joint row 0 = gate row 0, (r >> 2) & 3 = 0: piece s holds hidden 8 s ..
    np.testing.assert_array_equal(g[0, 0:8], np.arange(0, 8))
    # joint row 4 = gate row 4, (r >> 2) & 3 = 1: piece 0 holds hidden 8..15, piece 1 hidden 0..7
    np.testing.assert_array_equal(g[4, 8:16], 4 * 32 + np.arange(0, 8))
    np.testing.assert_array_equal(g[4, 0:8], 4 * 32 + 8 + np.arange(0, 8))
    # joint row 32 = up row 0; hidden 32..39 lie in tile (0, ks = 1), which starts at element 8192
    np.testing.assert_array_equal(u[0, 32:40], 8192 + 32 * 32 + np.arange(0, 8))
    # joint row 256 opens tile row tn = 1: gate row 128, at element (1 * n_ks + 0) * 8192
    np.testing.assert_array_equal(g[128, 0:8], n_ks * 8192 + np.arange(0, 8))
