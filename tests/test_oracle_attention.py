"""Pins for the fp64 attention oracle (CPU only).

The paper prints no numeric attention value, so the oracle is pinned by what the
mathematics fixes: a loop-by-loop brute force that shares no code with it, closed
forms, a library routine (torch SDPA, fp64), and invariants chosen so that a
dropped term, a wrong sign/index, a wrong mask or a transposed operand fails.
"""
import math
import os

import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as A

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# --------------------------------------------------------------------------- brute force
def brute_causal(q, k, v, scale):
    """Definition with python loops and math.exp only (no matmul, no numpy reductions)."""
    L, H, dq = q.shape
    Hkv, dv = k.shape[1], v.shape[2]
    out = np.zeros((L, H, dv))
    for i in range(L):
        for h in range(H):
            g = h // (H // Hkv)
            scores = []
            for j in range(i + 1):
                s = 0.0
                for c in range(dq):
                    s += q[i, h, c] * k[j, g, c]
                scores.append(scale * s)
            mx = max(scores)
            w = [math.exp(s - mx) for s in scores]
            z = sum(w)
            for j in range(i + 1):
                for c in range(dv):
                    out[i, h, c] += w[j] / z * v[j, g, c]
    return out


@pytest.mark.parametrize("L,H,Hkv,dq,dv", [(1, 1, 1, 1, 1), (5, 2, 2, 3, 3), (8, 4, 2, 4, 2), (7, 6, 2, 2, 5)])
def test_causal_matches_brute_force(L, H, Hkv, dq, dv):
    rng = np.random.default_rng(L * 100 + H)
    q, k, v = _rand(rng, L, H, dq), _rand(rng, L, Hkv, dq), _rand(rng, L, Hkv, dv)
    got = A.causal_attention(q, k, v, 0.7)
    np.testing.assert_allclose(got, brute_causal(q, k, v, 0.7), rtol=1e-12, atol=1e-13)


def test_decode_matches_brute_force_last_row():
    rng = np.random.default_rng(3)
    L, H, Hkv, d = 9, 4, 2, 3
    q, k, v = _rand(rng, L, H, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    want = brute_causal(q, k, v, 0.5)[L - 1]
    np.testing.assert_allclose(A.decode_attention(q[L - 1], k, v, 0.5), want, rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- closed forms
def test_hand_worked_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "attention_closed_form.txt")) if l.strip() and l[0] != "#"]
    q = np.array([[float(r[0])] for r in rows])[:, None, :]
    k = np.array([[float(r[1])] for r in rows])[:, None, :]
    v = np.array([[float(r[2])] for r in rows])[:, None, :]
    want = np.array([float(r[3]) for r in rows])
    got = A.causal_attention(q, k, v, 1.0)[:, 0, 0]
    np.testing.assert_allclose(got, want, rtol=1e-14)


def test_single_token_returns_v0():
    rng = np.random.default_rng(0)
    q, k, v = _rand(rng, 1, 4, 8), _rand(rng, 1, 2, 8), _rand(rng, 1, 2, 8)
    out = A.causal_attention(q, k, v, 0.3)
    for h in range(4):
        np.testing.assert_array_equal(out[0, h], v[0, h // 2])


def test_equal_keys_give_running_mean():
    rng = np.random.default_rng(1)
    L = 6
    q, v = _rand(rng, L, 2, 4), _rand(rng, L, 1, 4)
    k = np.broadcast_to(_rand(rng, 1, 1, 4), (L, 1, 4)).copy()
    out = A.causal_attention(q, k, v, 1.0)
    for i in range(L):
        np.testing.assert_allclose(out[i, 0], v[: i + 1, 0].mean(axis=0), rtol=1e-13)
        np.testing.assert_allclose(out[i, 1], v[: i + 1, 0].mean(axis=0), rtol=1e-13)


def test_zero_scale_gives_running_mean_and_uniform_decode():
    rng = np.random.default_rng(2)
    q, k, v = _rand(rng, 5, 2, 3), _rand(rng, 5, 2, 3), _rand(rng, 5, 2, 3)
    out = A.causal_attention(q, k, v, 0.0)
    np.testing.assert_allclose(out[4], v.mean(axis=0), rtol=1e-13)
    np.testing.assert_allclose(A.decode_attention(q[0], k, v, 0.0), v.mean(axis=0), rtol=1e-13)


def test_dominant_score_selects_its_value():
    # one key aligned with the query and scaled up: softmax -> one-hot on that key
    d, L, jstar = 4, 6, 2
    rng = np.random.default_rng(4)
    v = _rand(rng, L, 1, d)
    k = np.zeros((L, 1, d))
    k[jstar, 0, 0] = 1.0
    q = np.zeros((L, 1, d))
    q[:, 0, 0] = 800.0
    out = A.causal_attention(q, k, v, 1.0)
    for i in range(jstar, L):
        np.testing.assert_allclose(out[i, 0], v[jstar, 0], atol=1e-300, rtol=1e-13)
    # rows before jstar cannot see it (causal mask): they average what they see
    np.testing.assert_allclose(out[1, 0], v[:2, 0].mean(axis=0), rtol=1e-13)


def test_future_tokens_do_not_matter():
    rng = np.random.default_rng(5)
    L = 7
    q, k, v = _rand(rng, L, 2, 3), _rand(rng, L, 1, 3), _rand(rng, L, 1, 3)
    base = A.causal_attention(q, k, v, 0.9)
    k2, v2 = k.copy(), v.copy()
    k2[4:] = _rand(rng, L - 4, 1, 3)
    v2[4:] = _rand(rng, L - 4, 1, 3)
    np.testing.assert_array_equal(A.causal_attention(q, k2, v2, 0.9)[:4], base[:4])
    assert not np.allclose(A.causal_attention(q, k2, v2, 0.9)[4:], base[4:])


# --------------------------------------------------------------------------- library second opinion
@pytest.mark.parametrize("L,H,Hkv,d", [(33, 4, 4, 16), (50, 8, 2, 32)])
def test_causal_matches_torch_sdpa_fp64(L, H, Hkv, d):
    rng = np.random.default_rng(6)
    q, k, v = _rand(rng, L, H, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    scale = 1.0 / math.sqrt(d)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(H // Hkv, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(H // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    np.testing.assert_allclose(A.causal_attention(q, k, v, scale), ref[0].permute(1, 0, 2).numpy(),
                               rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------- invariants
def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(7)
    L, H, Hkv, d = 12, 8, 2, 5
    q, k, v = _rand(rng, L, H, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    rep = H // Hkv
    full = A.causal_attention(q, np.repeat(k, rep, axis=1), np.repeat(v, rep, axis=1), 0.4)
    np.testing.assert_allclose(A.causal_attention(q, k, v, 0.4), full, rtol=1e-13)
    dfull = A.decode_attention(q[-1], np.repeat(k, rep, axis=1), np.repeat(v, rep, axis=1), 0.4)
    np.testing.assert_allclose(A.decode_attention(q[-1], k, v, 0.4), dfull, rtol=1e-13)


def test_key_shift_invariance_and_value_linearity():
    rng = np.random.default_rng(8)
    L, H, Hkv, d = 10, 4, 2, 6
    q, k, v, v2 = _rand(rng, L, H, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    base = A.causal_attention(q, k, v, 0.6)
    # adding one vector to every key shifts each row's scores by a constant: softmax unchanged
    np.testing.assert_allclose(A.causal_attention(q, k + _rand(rng, 1, Hkv, d), v, 0.6), base, rtol=1e-11, atol=1e-12)
    both = A.causal_attention(q, k, 2.0 * v + v2, 0.6)
    np.testing.assert_allclose(both, 2.0 * base + A.causal_attention(q, k, v2, 0.6), rtol=1e-12, atol=1e-13)
    # weights are a convex combination: a constant V comes back unchanged
    ones = np.ones_like(v)
    np.testing.assert_allclose(A.causal_attention(q, k, ones, 0.6), 1.0, rtol=1e-13)


def test_decode_is_permutation_invariant_over_cached_tokens():
    rng = np.random.default_rng(9)
    n, H, Hkv, d = 21, 4, 2, 4
    q, k, v = _rand(rng, H, d), _rand(rng, n, Hkv, d), _rand(rng, n, Hkv, d)
    perm = rng.permutation(n)
    np.testing.assert_allclose(A.decode_attention(q, k[perm], v[perm], 0.5), A.decode_attention(q, k, v, 0.5),
                               rtol=1e-12, atol=1e-14)


def test_decode_equals_last_prefill_row_at_every_length():
    rng = np.random.default_rng(10)
    L, H, Hkv, d = 19, 4, 2, 8
    q, k, v = _rand(rng, L, H, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    full = A.causal_attention(q, k, v, 0.35)
    for n in (1, 2, 15, 16, 17, 19):
        np.testing.assert_allclose(A.decode_attention(q[n - 1], k[:n], v[:n], 0.35), full[n - 1], rtol=1e-12, atol=1e-14)


def test_prefill_batch_requests_are_independent():
    layer = W.LayerShape("gqa", 4, 2, 8, 8, 4)
    q, k, v, cu = W.prefill_inputs(layer, (5, 1, 9), seed=11)
    qf, kf, vf = (W.bf16_bits_to_f32(a).astype(np.float64) for a in (q, k, v))
    out = A.prefill_attention(qf, kf, vf, cu, 0.25)
    for r in range(3):
        a, b = cu[r], cu[r + 1]
        np.testing.assert_array_equal(out[a:b], A.causal_attention(qf[a:b], kf[a:b], vf[a:b], 0.25))
    with pytest.raises(ValueError):
        A.prefill_attention(qf, kf, vf, np.array([0, 5, 5, 15]), 0.25)   # zero-length prompt


def test_empty_context_raises():
    with pytest.raises(ValueError):
        A.decode_attention(np.zeros((2, 4)), np.zeros((0, 1, 4)), np.zeros((0, 1, 4)), 1.0)


# --------------------------------------------------------------------------- paged == contiguous
@pytest.mark.parametrize("n", [1, 15, 16, 17, 37, 48, 129])
def test_paged_equals_contiguous_bit_for_bit(n):
    P, Hkv, H, d = 16, 2, 4, 8
    rng = np.random.default_rng(n)
    k, v, q = _rand(rng, n, Hkv, d), _rand(rng, n, Hkv, d), _rand(rng, H, d)
    store = A.PagedKV(64, P, Hkv, d, d)
    table = rng.permutation(64)[: -(-n // P)]
    store.write(table, 0, k, v)
    gk, gv = store.gather(table, n)
    np.testing.assert_array_equal(gk, k)
    np.testing.assert_array_equal(gv, v)
    np.testing.assert_array_equal(A.paged_decode_attention(q, store, table, n, 0.3), A.decode_attention(q, k, v, 0.3))


def test_paged_write_in_two_pieces_and_bf16_bits_roundtrip():
    layer = W.LayerShape("gqa", 4, 2, 8, 8, 16)
    _, ks, vs = W.decode_inputs(layer, (41,), seed=12)
    store = A.PagedKV(8, 16, 2, 8, 8, dtype=np.uint16)
    table = [5, 0, 7]
    store.write(table, 0, ks[0][:30], vs[0][:30])
    store.write(table, 30, ks[0][30:], vs[0][30:])        # append continues mid-page
    gk, gv = store.gather(table, 41)
    np.testing.assert_array_equal(gk, ks[0])
    np.testing.assert_array_equal(gv, vs[0])
    # untouched pages stay zero: no write strays outside the block table
    for p in (1, 2, 3, 4, 6):
        assert not store.k[p].any() and not store.v[p].any()


# --------------------------------------------------------------------------- MLA
def test_mla_absorbed_equals_unabsorbed():
    H, nope, rope, lora, dv, n = 4, 16, 8, 32, 16, 23
    rng = np.random.default_rng(13)
    w_uk, w_uv = W.mla_weights(H, nope, lora, dv, seed=14)
    w_uk, w_uv = w_uk * 20, w_uv * 20       # O(0.4) weights so that scores are not all ~0
    q_nope, q_rope, latent = _rand(rng, H, nope), _rand(rng, H, rope), _rand(rng, n, lora + rope)
    scale = 1.0 / math.sqrt(nope + rope)
    qabs = A.mla_absorb_query(q_nope, q_rope, w_uk)
    assert qabs.shape == (H, lora + rope)
    o_lat = A.mla_decode_latent(qabs, latent, scale, lora)
    got = np.einsum("hc,hcd->hd", o_lat, w_uv)
    want = A.mla_decode_unabsorbed(q_nope, q_rope, latent, w_uk, w_uv, scale, lora)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    assert np.abs(want).max() > 1e-3


def test_mla_latent_decode_matches_brute_force():
    H, lora, rope, n = 3, 4, 2, 6
    rng = np.random.default_rng(15)
    qabs, latent = _rand(rng, H, lora + rope), _rand(rng, n, lora + rope)
    want = np.zeros((H, lora))
    for h in range(H):
        s = [0.8 * sum(qabs[h, c] * latent[t, c] for c in range(lora + rope)) for t in range(n)]
        mx = max(s)
        w = [math.exp(x - mx) for x in s]
        for t in range(n):
            for c in range(lora):
                want[h, c] += w[t] / sum(w) * latent[t, c]
    np.testing.assert_allclose(A.mla_decode_latent(qabs, latent, 0.8, lora), want, rtol=1e-12)


def test_mla_expand_kv_shares_rope_row_across_heads():
    H, nope, rope, lora, dv, n = 3, 4, 2, 5, 4, 7
    rng = np.random.default_rng(16)
    w_uk, w_uv = W.mla_weights(H, nope, lora, dv, seed=17)
    latent = _rand(rng, n, lora + rope)
    k, v = A.mla_expand_kv(latent, w_uk, w_uv, lora)
    assert k.shape == (n, H, nope + rope) and v.shape == (n, H, dv)
    for h in range(H):
        np.testing.assert_array_equal(k[:, h, nope:], latent[:, lora:])
        np.testing.assert_allclose(k[:, h, :nope], latent[:, :lora] @ w_uk[h].T, rtol=1e-13)
        np.testing.assert_allclose(v[:, h], latent[:, :lora] @ w_uv[h], rtol=1e-13)


def test_paged_latent_roundtrip():
    rng = np.random.default_rng(18)
    lat = _rand(rng, 130, 12)
    store = A.PagedLatent(8, 64, 12)
    table = [6, 2, 3]
    store.write(table, 0, lat[:64])
    store.write(table, 64, lat[64:])
    np.testing.assert_array_equal(store.gather(table, 130), lat)
    np.testing.assert_array_equal(store.gather(table, 65), lat[:65])


# --------------------------------------------------------------------------- input generators
def test_bf16_rounding_is_nearest_even_and_exact():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.140625, 0.0], dtype=np.float32)
    b = W.to_bf16_bits(x)
    back = W.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to the even mantissa (1.0)
    assert back[1] == 1.0
    # 1 + 3*2^-9 is above the tie: rounds up to 1 + 2^-7
    assert back[2] == 1.0078125
    # 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even): goes up
    assert back[3] == 1.015625
    np.testing.assert_array_equal(W.to_bf16_bits(back), b)          # idempotent
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(back, t)


def test_workload_generators_are_seeded_and_shaped():
    c2 = W.get_config("c2")
    assert len(c2.decode_ctx) == 64 and min(c2.decode_ctx) >= 512 and max(c2.decode_ctx) <= 4096
    assert c2.layer.page_bytes == 65536 and c2.num_pages == 610351
    c3 = W.get_config("c3")
    assert len(c3.decode_ctx) == 128 and max(c3.decode_ctx) <= 8192
    c4 = W.get_config("c4")
    assert c4.layer.page_bytes == 73728 and min(c4.decode_ctx) >= 1024
    assert W.get_config("c2").decode_ctx == c2.decode_ctx
    a = W.prefill_inputs(W.get_config("c1").layer, (128, 128), 1000)
    b = W.prefill_inputs(W.get_config("c1").layer, (128, 128), 1000)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert a[0].shape == (256, 8, 64) and a[0].dtype == np.uint16 and list(a[3]) == [0, 128, 256]
    tr = W.trace(200)
    assert np.all(np.diff(tr.arrival_s) >= 0) and tr.input_len.max() <= 8192 and tr.output_len.min() >= 1


# ---------------------------------------------------------------- chunked prefill over a cached prefix
def test_chunk_attention_is_the_matching_rows_of_causal_attention():
    """The definition: processing a prompt piece by piece must give the rows that processing it whole gives."""
    rng = np.random.default_rng(41)
    L, H, Hkv, d = 53, 4, 2, 16
    q, k, v = rng.normal(size=(L, H, d)), rng.normal(size=(L, Hkv, d)), rng.normal(size=(L, Hkv, d))
    whole = A.causal_attention(q, k, v, 0.25)
    cuts = [0, 1, 17, 18, 40, 53]
    for a, b in zip(cuts[:-1], cuts[1:]):
        got = A.chunk_attention(q[a:b], k[:b], v[:b], 0.25)
        np.testing.assert_allclose(got, whole[a:b], rtol=1e-12, atol=1e-14)
    # no prefix: the chunk is the whole prompt
    np.testing.assert_allclose(A.chunk_attention(q, k, v, 0.25), whole, rtol=1e-12, atol=1e-14)


def test_chunk_attention_brute_force_and_single_row_is_decode():
    rng = np.random.default_rng(42)
    n, C, H, Hkv, d = 11, 4, 2, 1, 8
    q, k, v = rng.normal(size=(C, H, d)), rng.normal(size=(n, Hkv, d)), rng.normal(size=(n, Hkv, d))
    got = A.chunk_attention(q, k, v, 0.3)
    for i in range(C):
        for h in range(H):
            pos = n - C + i
            w = [math.exp(0.3 * sum(q[i, h, x] * k[j, 0, x] for x in range(d))) for j in range(pos + 1)]
            z = sum(w)
            for x in range(d):
                assert got[i, h, x] == pytest.approx(sum(w[j] * v[j, 0, x] for j in range(pos + 1)) / z, rel=1e-11, abs=1e-13)
    # a chunk of one row over its context is the decode step
    np.testing.assert_allclose(A.chunk_attention(q[-1:], k, v, 0.3)[0], A.decode_attention(q[-1], k, v, 0.3), rtol=1e-12)
    with pytest.raises(ValueError):
        A.chunk_attention(q, k[:3], v[:3], 0.3)
