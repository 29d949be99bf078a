"""GPU parity of the gated FFN's first step (C-ABI spd_ffn_gate_up, spd_ffn_pack_gate_up) against the fp64 oracle.

Paper, Evaluation "Implementation based on DistServe": the first two GEMMs of the gated FFN fused into one.
Bar: |got - exact| <= 2^-8 |exact| + 2^-10.  The kernel rounds silu(g) * u once to bf16 (nearest even): half an ulp
is at most 2^-8 of the exact value's magnitude.  Before that, g and u are fp32 sums of `hidden` exact bf16 products:
the expected error is about 2^-24 sqrt(hidden) times partial sums of order one (4e-6 at hidden 4096), the activation
adds a few 2^-24, and the result moves by at most 1.1 |u| dg + |g| du; the absolute term 2^-10 covers all of that with
a wide margin for the generator's scale (|g|, |u| of order one)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import ffn as F
from paper_2504_19867_amd import semipd as S
from ffn_layout import unpack_gate_up
from gpu_util import DEV, dev_bf16, f64, host_bits, host_f64

pytestmark = pytest.mark.gpu
PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE


def _assert_ffn(got: np.ndarray, want: np.ndarray, what: str):
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), what
    bar = 2.0 ** -8 * np.abs(want) + 2.0 ** -10
    err = np.abs(got - want)
    bad = err > bar
    assert not bad.any(), f"{what}: {int(bad.sum())} entries beyond the bar, worst {err[bad].max():.3e}"
    return float(err.max())


def _run(ctx, phase, xb, wgb, wub, poison_out=True):
    T, K = xb.shape
    I = wgb.shape[0]
    x, wg, wu = dev_bf16(xb), dev_bf16(wgb), dev_bf16(wub)
    w_gu = torch.empty((2 * I, K), dtype=torch.bfloat16, device=DEV)
    out = torch.full((max(T, 1), I), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx.ffn_pack_gate_up(phase, wg, wu, w_gu, K, I)
    ctx.ffn_gate_up(phase, x, w_gu, out, T, K, I)
    ctx.phase_sync(phase)
    return out[:T], w_gu


@pytest.mark.parametrize("T,K,I", [(300, 256, 256), (1, 64, 128), (64, 512, 384), (256, 32, 128), (257, 96, 128), (515, 1024, 512),
                                   (300, 32, 128), (100, 96, 256), (200, 320, 128), (130, 4096, 128)])
def test_gate_up_matches_oracle(T, K, I):
    ctx = S.Context(0)
    xb, wgb, wub = W.ffn_inputs(T, K, I, seed=100 + T)
    out, w_gu = _run(ctx, PRE, xb, wgb, wub)
    # the packed weights are a permutation of 16-byte pieces: read back through the header's index formula
    # (element by element, for the smaller shapes) they are the two matrices bit for bit
    if K * I <= 512 * 384:
        g2, u2 = unpack_gate_up(host_bits(w_gu), K)
        np.testing.assert_array_equal(g2, wgb)
        np.testing.assert_array_equal(u2, wub)
    want = F.gate_up(f64(xb), f64(wgb), f64(wub))
    _assert_ffn(host_f64(out), want, f"ffn T={T} K={K} I={I}")
    ctx.close()


@pytest.mark.parametrize("T,K,I", [(1, 256, 128), (7, 512, 384), (31, 256, 640), (32, 1024, 128), (33, 256, 128), (48, 768, 256),
                                   (63, 512, 128), (64, 256, 384), (16, 4096, 256), (64, 4096, 128)])
def test_gate_up_batches_of_up_to_64_tokens(T, K, I):
    """At most 64 tokens: the small-tile instances (which one depends on the phase's share of compute units and on
    inter), ragged token counts, 8 to 128 slices."""
    ctx = S.Context(0)
    xb, wgb, wub = W.ffn_inputs(T, K, I, seed=500 + T)
    for phase in (PRE, DEC):
        out, _ = _run(ctx, phase, xb, wgb, wub)
        _assert_ffn(host_f64(out), F.gate_up(f64(xb), f64(wgb), f64(wub)), f"ffn small batch T={T} K={K} I={I}")
    ctx.close()


@pytest.mark.parametrize("T,K", [(5, 256), (33, 512), (64, 1024)])
def test_gate_up_small_batch_on_a_small_share_takes_the_wide_tile(T, K):
    """inter = 3584 gives 28 tiles of 256 joint columns: on a 32-CU decode share that is enough for the 64 x 256
    instance (eight waves, one piece of x per wave), which the shapes above never reach on larger shares."""
    ctx = S.Context(0)
    total, _, gran = ctx.device_info()
    ctx.set_partition(total - gran, gran)
    I = 3584
    xb, wgb, wub = W.ffn_inputs(T, K, I, seed=900 + T)
    out, _ = _run(ctx, DEC, xb, wgb, wub)
    assert ctx.get_partition()[1] == gran
    _assert_ffn(host_f64(out), F.gate_up(f64(xb), f64(wgb), f64(wub)), f"ffn small batch, wide tile T={T} K={K}")
    ctx.close()


def test_both_phases_and_partitions_give_the_same_bits():
    ctx = S.Context(0)
    total = ctx.device_info()[0]
    xb, wgb, wub = W.ffn_inputs(700, 256, 640, seed=7)
    ref, _ = _run(ctx, PRE, xb, wgb, wub)
    ref = host_bits(ref)
    ctx.set_partition(total // 4, 3 * total // 4)
    for phase in (PRE, DEC):
        got, _ = _run(ctx, phase, xb, wgb, wub)
        np.testing.assert_array_equal(host_bits(got), ref)
    ctx.close()


def test_rows_past_the_batch_are_not_written_and_zero_tokens_is_a_no_op():
    ctx = S.Context(0)
    T, K, I = 130, 128, 128
    xb, wgb, wub = W.ffn_inputs(T, K, I, seed=9)
    x, wg, wu = dev_bf16(xb), dev_bf16(wgb), dev_bf16(wub)
    w_gu = torch.empty((2 * I, K), dtype=torch.bfloat16, device=DEV)
    out = torch.full((T + 40, I), 7.0, dtype=torch.bfloat16, device=DEV)
    ctx.ffn_pack_gate_up(PRE, wg, wu, w_gu, K, I)
    ctx.ffn_gate_up(PRE, x, w_gu, out, 0, K, I)
    ctx.phase_sync(PRE)
    assert (out == 7.0).all()
    ctx.ffn_gate_up(PRE, x, w_gu, out, T, K, I)
    ctx.phase_sync(PRE)
    assert (out[T:] == 7.0).all()
    _assert_ffn(host_f64(out[:T]), F.gate_up(f64(xb), f64(wgb), f64(wub)), "ffn ragged")
    ctx.close()


def test_large_gate_values_saturate_like_the_definition():
    # silu(z) -> z for large z and -> 0 for very negative z: no NaN from exp overflow
    ctx = S.Context(0)
    T, K, I = 4, 32, 128
    x = np.zeros((T, K), dtype=np.float32)
    x[:, 0] = [100.0, -100.0, 30.0, -30.0]
    wg = np.zeros((I, K), dtype=np.float32)
    wg[:, 0] = 1.0
    wu = np.zeros((I, K), dtype=np.float32)
    wu[:, 0] = 0.5
    xb, wgb, wub = W.to_bf16_bits(x), W.to_bf16_bits(wg), W.to_bf16_bits(wu)
    out, _ = _run(ctx, DEC, xb, wgb, wub)
    _assert_ffn(host_f64(out), F.gate_up(f64(xb), f64(wgb), f64(wub)), "ffn saturation")
    ctx.close()


def test_llama3_8b_shape_sampled():
    """The Llama-3-8B layer shape (hidden 4096, inter 14336) on a prefill batch of 8192 tokens, as the bench times it;
    the oracle checks a sample of token rows, all columns."""
    ctx = S.Context(0)
    T, K, I = 8192, 4096, 14336
    xb, wgb, wub = W.ffn_inputs(T, K, I, seed=2024)
    out, _ = _run(ctx, PRE, xb, wgb, wub)
    rows = np.array([0, 1, 255, 256, 4095, 4096, 5000, 8191])
    want = F.gate_up(f64(xb[rows]), f64(wgb), f64(wub))
    _assert_ffn(host_f64(out[torch.from_numpy(rows).to(DEV)]), want, "ffn llama-3-8b sampled rows")
    ctx.close()


def test_prompt_and_decode_batches_at_the_same_time_on_disjoint_partitions():
    """The paper's setting for this step: a prompt batch on the prefill partition while the decode partition runs
    decode batches; every launch gives the bits it gives alone."""
    ctx = S.Context(0)
    total = ctx.device_info()[0]
    K, I = 512, 1024
    xpb, wgb, wub = W.ffn_inputs(1500, K, I, seed=31)
    xdb, _, _ = W.ffn_inputs(48, K, I, seed=32)
    ref_p, w_gu = _run(ctx, PRE, xpb, wgb, wub)
    ref_p = host_bits(ref_p)
    xd = dev_bf16(xdb)
    od = torch.full((48, I), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx.ffn_gate_up(DEC, xd, w_gu, od, 48, K, I)
    ctx.phase_sync(DEC)
    ref_d = host_bits(od)
    _assert_ffn(host_f64(od), F.gate_up(f64(xdb), f64(wgb), f64(wub)), "ffn decode batch")
    ctx.set_partition(total // 2, total // 2)
    xp = dev_bf16(xpb)
    outs_p = [torch.full((1500, I), float("nan"), dtype=torch.bfloat16, device=DEV) for _ in range(3)]
    outs_d = [torch.full((48, I), float("nan"), dtype=torch.bfloat16, device=DEV) for _ in range(12)]
    for i in range(3):                            # both streams fill up before either drains
        ctx.ffn_gate_up(PRE, xp, w_gu, outs_p[i], 1500, K, I)
        for j in range(4):
            ctx.ffn_gate_up(DEC, xd, w_gu, outs_d[4 * i + j], 48, K, I)
    ctx.phase_sync(PRE)
    ctx.phase_sync(DEC)
    assert ctx.get_partition()[:2] == (total // 2, total // 2)
    for o in outs_p:
        np.testing.assert_array_equal(host_bits(o), ref_p)
    for o in outs_d:
        np.testing.assert_array_equal(host_bits(o), ref_d)
    ctx.close()


def test_random_shapes():
    """Seeded random (tokens, hidden, inter) within the interface's conditions: every tile instance, ragged token
    counts, hidden sizes that are not a multiple of the 64-wide register pipeline's unroll."""
    rng = np.random.default_rng(77)
    ctx = S.Context(0)
    for case in range(12):
        T = int(rng.integers(1, 700))
        K = 32 * int(rng.integers(1, 33))
        I = 128 * int(rng.integers(1, 7))
        xb, wgb, wub = W.ffn_inputs(T, K, I, seed=500 + case)
        out, _ = _run(ctx, (PRE, DEC)[case % 2], xb, wgb, wub)
        _assert_ffn(host_f64(out), F.gate_up(f64(xb), f64(wgb), f64(wub)), f"ffn random case {case}: T={T} K={K} I={I}")
    ctx.close()
