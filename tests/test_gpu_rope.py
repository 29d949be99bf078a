"""GPU parity of the rotary-embedding step (C-ABI spd_rope_qk) against the fp64 oracle.

Paper, Evaluation "Implementation based on DistServe": the RoPE kernel, modified for Llama-3.1.
Bar: the kernel rounds the rotated value to bf16 (nearest even): half an ulp is at most 2^-8 of
the exact value's magnitude; on top of that the fp32 rotation and sine / cosine may err by a few
2^-24 of the operands, taken as 2^-18 (|x_a| + |x_b|) with a wide margin."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as OA
from oracle import rope as R
from paper_2504_19867_amd import semipd as S
from gpu_util import DEV, GpuPool, assert_parity, dev_bf16, f64, host_f64

pytestmark = pytest.mark.gpu
PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE


def _lib_cfg(o: R.RopeConfig, offset: int = 0):
    return S.rope_config(theta=o.theta, factor=o.factor, low_freq_factor=o.low_freq_factor, high_freq_factor=o.high_freq_factor,
                         original_max_pos=o.original_max_pos, rotary_dim=o.rotary_dim, rotary_offset=offset,
                         interleaved=o.interleaved)


def _oracle(x64: np.ndarray, positions, o: R.RopeConfig, offset: int):
    """The oracle rotates the leading rotary_dim entries: hand it the rotating slice."""
    out = x64.copy()
    out[:, :, offset:offset + o.rotary_dim] = R.apply_rope(x64[:, :, offset:offset + o.rotary_dim], positions, o)
    return out


def _pair_magnitude(x64: np.ndarray, o: R.RopeConfig, offset: int):
    """|x_a| + |x_b| for every entry (0 outside the rotating range)."""
    mag = np.zeros_like(x64)
    for a, b in R.pair_index(o):
        s = np.abs(x64[:, :, offset + a]) + np.abs(x64[:, :, offset + b])
        mag[:, :, offset + a] = s
        mag[:, :, offset + b] = s
    return mag


def _assert_rope(got: np.ndarray, want: np.ndarray, mag: np.ndarray, what: str):
    assert np.isfinite(got).all(), what
    bar = 2.0 ** -8 * np.abs(want) + 2.0 ** -18 * mag
    bad = np.abs(got - want) > bar
    assert not bad.any(), f"{what}: {int(bad.sum())} entries beyond the bar, worst {np.abs(got - want)[bad].max():.3e}"


CASES = [
    # name, oracle config, offset, dim, Hq, Hkv, positions
    ("llama31 prompt", R.LLAMA31, 0, 128, 32, 8, lambda rng: np.arange(300) + 5),
    ("llama31 far positions", R.LLAMA31, 0, 128, 8, 2, lambda rng: rng.integers(0, 131072, size=97)),
    ("plain theta 1e4 dim 64", R.RopeConfig(theta=10000.0, rotary_dim=64), 0, 64, 5, 1, lambda rng: rng.integers(0, 4096, size=33)),
    ("partial rotary", R.RopeConfig(theta=10000.0, rotary_dim=32), 0, 128, 4, 4, lambda rng: rng.integers(0, 9000, size=50)),
    ("interleaved tail (MLA rope part)", R.RopeConfig(theta=10000.0, rotary_dim=64, interleaved=True), 128, 192, 16, 16,
     lambda rng: rng.integers(0, 20000, size=40)),
    ("decode batch", R.LLAMA31, 0, 128, 32, 8, lambda rng: rng.integers(511, 131072, size=64)),
    ("one token at position 0", R.LLAMA31, 0, 128, 32, 8, lambda rng: np.array([0])),
]


@pytest.mark.parametrize("name,o,offset,dim,hq,hkv,posf", CASES, ids=[c[0] for c in CASES])
def test_rope_matches_the_oracle(name, o, offset, dim, hq, hkv, posf):
    rng = np.random.default_rng(77)
    pos = np.asarray(posf(rng), dtype=np.int64)
    T = len(pos)
    qb, kb = W.normal_bf16(rng, (T, hq, dim)), W.normal_bf16(rng, (T, hkv, dim))
    ctx = S.Context(0)
    tq, tk = dev_bf16(qb), dev_bf16(kb)
    phase = DEC if "decode" in name else PRE
    ctx.rope_qk(phase, _lib_cfg(o, offset), [int(p) for p in pos], tq, hq, tk, hkv, dim)
    ctx.phase_sync(phase)
    for bits, t, what in ((qb, tq, "q"), (kb, tk, "k")):
        x = f64(bits)
        _assert_rope(host_f64(t), _oracle(x, pos, o, offset), _pair_magnitude(x, o, offset), f"{name}: {what}")
    if offset or o.rotary_dim < dim:      # entries outside the rotating range come back bit for bit
        keep = np.ones(dim, dtype=bool)
        keep[offset:offset + o.rotary_dim] = False
        assert np.array_equal(host_f64(tq)[:, :, keep], f64(qb)[:, :, keep])


def test_rope_one_tensor_only_and_empty_batch():
    rng = np.random.default_rng(78)
    o = R.RopeConfig(theta=500000.0, rotary_dim=128)
    pos = rng.integers(0, 8192, size=19)
    xb = W.normal_bf16(rng, (19, 3, 128))
    ctx = S.Context(0)
    for which in ("q", "k"):
        t = dev_bf16(xb)
        if which == "q":
            ctx.rope_qk(PRE, _lib_cfg(o), [int(p) for p in pos], t, 3, None, 0, 128)
        else:
            ctx.rope_qk(PRE, _lib_cfg(o), [int(p) for p in pos], None, 0, t, 3, 128)
        ctx.phase_sync(PRE)
        x = f64(xb)
        _assert_rope(host_f64(t), _oracle(x, pos, o, 0), _pair_magnitude(x, o, 0), which + " only")
    t = dev_bf16(xb)
    ctx.rope_qk(PRE, _lib_cfg(o), [], t, 3, None, 0, 128)             # nothing to do, nothing touched
    ctx.phase_sync(PRE)
    assert np.array_equal(host_f64(t), f64(xb))


def test_rope_refuses_shapes_the_kernel_cannot_take():
    ctx = S.Context(0)
    t = torch.zeros((4, 2, 128), dtype=torch.bfloat16, device=DEV)
    for cfg, dim in [(S.rope_config(rotary_dim=24), 128),                 # not a multiple of 16
                     (S.rope_config(rotary_dim=64, rotary_offset=4), 128),  # offset not on a 16-byte piece
                     (S.rope_config(rotary_dim=128, rotary_offset=8), 128),  # runs past the head
                     (S.rope_config(rotary_dim=64), 68)]:                   # rows not made of 16-byte pieces
        with pytest.raises(S.SpdError):
            ctx.rope_qk(PRE, cfg, [0, 1, 2, 3], t, 2, None, 0, dim)
    with pytest.raises(S.SpdError):
        ctx.rope_qk(PRE, S.rope_config(), [0, -1, 2, 3], t, 2, None, 0, 128)   # negative position


def test_rope_then_prefill_step_end_to_end():
    """RoPE on the prefill partition, then the prefill step on the same stream: against the oracle's
    rotation (rounded to bf16, which is what the interface hands on) followed by its attention."""
    cfg = W.get_config("c1")
    L = cfg.layer
    lens = [37, 150]
    q, k, v, cu = W.prefill_inputs(L, lens, cfg.seed + 11)
    pos = np.concatenate([np.arange(n) for n in lens])
    scale = 1.0 / np.sqrt(L.dim_qk)
    gp = GpuPool(L, cfg.num_pages)
    tq, tk, tv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    out = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    o = R.RopeConfig(theta=500000.0, factor=8.0, rotary_dim=L.dim_qk)
    gp.ctx.rope_qk(PRE, _lib_cfg(o), [int(p) for p in pos], tq, L.n_q_heads, tk, L.n_kv_heads, L.dim_qk)
    gp.pool.prefill_step([1, 2], cu, tq, tk, tv, out, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale)
    gp.ctx.phase_sync(PRE)
    q_rot = f64(W.to_bf16_bits(R.apply_rope(f64(q), pos, o)))
    k_rot = f64(W.to_bf16_bits(R.apply_rope(f64(k), pos, o)))
    want = OA.prefill_attention(q_rot, k_rot, f64(v), cu, scale)
    assert_parity(host_f64(out), want, "rope + prefill step")
    # and the pages hold the rotated keys
    kg_t = torch.empty((lens[0], L.n_kv_heads, L.dim_qk), dtype=torch.bfloat16, device=DEV)
    vg_t = torch.empty((lens[0], L.n_kv_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    gp.pool.kv_gather(PRE, 1, lens[0], kg_t, vg_t)
    gp.ctx.phase_sync(PRE)
    kg = host_f64(kg_t)
    _assert_rope(kg, R.apply_rope(f64(k), pos, o)[:lens[0]], _pair_magnitude(f64(k), o, 0)[:lens[0]], "rotated keys in the pages")


# ----------------------------------------------------------------------------- inside the prefill step
FUSED_CASES = [
    # name, layer, oracle config, offset, prompt lengths, cached prefix per request (None: plain prefill)
    ("llama31 128 dims", W.LayerShape("gqa", 8, 2, 128, 128, 16), R.LLAMA31, 0, (37, 150, 16), None),
    ("64 dims, 8 KV heads", W.LayerShape("gqa", 8, 8, 64, 64, 16), R.RopeConfig(theta=10000.0, rotary_dim=64), 0, (70, 1, 33), None),
    ("interleaved part of the head", W.LayerShape("gqa", 4, 2, 128, 128, 16),
     R.RopeConfig(theta=10000.0, rotary_dim=32, interleaved=True), 64, (45, 90), None),
    ("half layout, part of the head", W.LayerShape("gqa", 4, 4, 128, 128, 16), R.RopeConfig(theta=10000.0, rotary_dim=64), 32, (100,), None),
    ("piece of a prompt over a cached prefix", W.LayerShape("gqa", 8, 2, 128, 128, 16), R.LLAMA31, 0, (40, 21), (27, 100)),
    ("one KV head: no fused form, same result", W.LayerShape("gqa", 4, 1, 128, 128, 16), R.LLAMA31, 0, (50, 19), None),
]


@pytest.mark.parametrize("name,L,o,offset,lens,prefix", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_prefill_step_with_rope_inside(name, L, o, offset, lens, prefix):
    """`rope` on the prefill batch: the step rotates q and k itself (the keys on their way into the pages).  Bit for
    bit what spd_rope_qk followed by the plain step gives (same arithmetic), and the oracle's rotation + attention."""
    rng = np.random.default_rng(len(name))
    q, k, v, cu = W.prefill_inputs(L, lens, seed=90 + len(name))
    scale = 1.0 / np.sqrt(L.dim_qk)
    cfg = _lib_cfg(o, offset)
    pre = list(prefix) if prefix else [0] * len(lens)
    pos = np.concatenate([p0 + np.arange(n) for p0, n in zip(pre, lens)])
    ids = list(range(1, len(lens) + 1))
    # cached prefixes: rotated keys already in the pages (written through the unfused path)
    cached = []
    results = []
    for fused in (True, False):
        gp = GpuPool(L, 64, poison=True)
        for r, p0 in zip(ids, pre):
            if p0:
                kc = W.normal_bf16(np.random.default_rng(1000 + r), (p0, L.n_kv_heads, L.dim_qk))
                vc = W.normal_bf16(np.random.default_rng(2000 + r), (p0, L.n_kv_heads, L.dim_v))
                tkc = dev_bf16(kc)
                gp.ctx.rope_qk(PRE, cfg, list(range(p0)), None, 0, tkc, L.n_kv_heads, L.dim_qk)
                gp.pool.kv_reserve(r, p0)
                gp.pool.kv_write(PRE, r, 0, p0, tkc, dev_bf16(vc))
                if fused:
                    cached.append((kc, vc))
        tq, tk, tv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
        out = torch.zeros((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
        if fused:
            gp.pool.prefill_step(ids, cu, tq, tk, tv, out, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale,
                                 prefix_lens=prefix, rope=cfg)
        else:
            gp.ctx.rope_qk(PRE, cfg, [int(p) for p in pos], tq, L.n_q_heads, tk, L.n_kv_heads, L.dim_qk)
            gp.pool.prefill_step(ids, cu, tq, tk, tv, out, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale, prefix_lens=prefix)
        pages = []
        for r, p0, n in zip(ids, pre, lens):
            kg = torch.zeros((p0 + n, L.n_kv_heads, L.dim_qk), dtype=torch.bfloat16, device=DEV)
            vg = torch.zeros((p0 + n, L.n_kv_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
            gp.pool.kv_gather(PRE, r, p0 + n, kg, vg)
            pages.append((kg, vg))
        gp.ctx.phase_sync(PRE)
        from gpu_util import host_bits
        results.append((host_bits(out), host_bits(tq), host_bits(tk), [(host_bits(a), host_bits(b)) for a, b in pages]))
        gp.close()
    (out_f, q_f, k_f, pages_f), (out_u, q_u, k_u, pages_u) = results
    np.testing.assert_array_equal(q_f, q_u)           # q and k rotated in place, as by spd_rope_qk
    np.testing.assert_array_equal(k_f, k_u)
    for (ka, va), (kb, vb) in zip(pages_f, pages_u):
        np.testing.assert_array_equal(ka, kb)
        np.testing.assert_array_equal(va, vb)
    np.testing.assert_array_equal(out_f, out_u)
    # against the oracle: rotation in fp64, rounded to bf16 (what the pages and the attention hold), then attention
    q_rot = f64(W.to_bf16_bits(_oracle(f64(q), pos, o, offset)))
    k_rot = f64(W.to_bf16_bits(_oracle(f64(k), pos, o, offset)))
    _assert_rope(f64(k_f), _oracle(f64(k), pos, o, offset), _pair_magnitude(f64(k), o, offset), "keys rotated by the step")
    for i, (r, p0, n) in enumerate(zip(ids, pre, lens)):
        a, b = cu[i], cu[i + 1]
        if p0:
            kc, vc = cached[i]
            kc_rot = f64(W.to_bf16_bits(_oracle(f64(kc), np.arange(p0), o, offset)))
            kk = np.concatenate([kc_rot, k_rot[a:b]])
            vv = np.concatenate([f64(vc), f64(v[a:b])])
            want = OA.chunk_attention(q_rot[a:b], kk, vv, scale)
        else:
            want = OA.causal_attention(q_rot[a:b], k_rot[a:b], f64(v[a:b]), scale)
        assert_parity(f64(out_f)[a:b], want, f"{name}: request {r}")


# ----------------------------------------------------------------------------- fused into the decode step
def _round_bf16(x64: np.ndarray) -> np.ndarray:
    return f64(W.to_bf16_bits(x64))


def test_decode_step_with_rope_rotates_query_and_appended_key_gqa():
    """rope in the decode batch: query and new key are rotated by position ctx_len - 1, the key goes to the
    page rotated, the caller's tensors stay as they were; several appends across a page border."""
    import math
    from test_gpu_parity import fill_decode_contexts, oracle_decode
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    gp = GpuPool(layer, 32, poison=True)
    o = R.RopeConfig(theta=500000.0, factor=8.0, rotary_dim=128)
    cfg = _lib_cfg(o)
    scale = 1.0 / math.sqrt(128)
    start = (14, 31)
    _, ks, vs, ids = fill_decode_contexts(gp, start, seed=141)           # cached keys: taken as already rotated
    ks, vs = [x.copy() for x in ks], [x.copy() for x in vs]
    rng = np.random.default_rng(142)
    lens = list(start)
    for step in range(4):
        lens = [n + 1 for n in lens]
        knew, vnew, qn = (W.normal_bf16(rng, (2, 2, 128)), W.normal_bf16(rng, (2, 2, 128)), W.normal_bf16(rng, (2, 8, 128)))
        tq, tk = dev_bf16(qn), dev_bf16(knew)
        out = torch.empty((2, 8, 128), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, lens, tq, out, 8, scale, k_new=tk, v_new=dev_bf16(vnew), rope=cfg)
        gp.ctx.phase_sync(DEC)
        assert np.array_equal(host_f64(tq), f64(qn)) and np.array_equal(host_f64(tk), f64(knew))    # inputs untouched
        pos = [n - 1 for n in lens]
        q_rot = _round_bf16(R.apply_rope(f64(qn), pos, o))
        k_rot = W.to_bf16_bits(R.apply_rope(f64(knew), pos, o))
        for i in range(2):
            ks[i] = np.concatenate([ks[i], k_rot[i][None]])
            vs[i] = np.concatenate([vs[i], vnew[i][None]])
        want = np.stack([OA.decode_attention(q_rot[i], f64(ks[i]), f64(vs[i]), scale) for i in range(2)])
        assert_parity(host_f64(out), want, f"rope + append step {step}")
        # the page holds the rotated key, to the rotation's own bar
        for i in range(2):
            kg = torch.empty((lens[i], 2, 128), dtype=torch.bfloat16, device=DEV)
            vg = torch.empty((lens[i], 2, 128), dtype=torch.bfloat16, device=DEV)
            gp.pool.kv_gather(DEC, ids[i], lens[i], kg, vg)
            gp.ctx.phase_sync(DEC)
            x = f64(knew)[i:i + 1]
            _assert_rope(host_f64(kg)[-1:], R.apply_rope(x, [pos[i]], o), _pair_magnitude(x, o, 0), "appended key")
            assert np.array_equal(host_f64(vg)[-1], f64(vnew)[i])
    # attend-only with rope: the query alone is rotated
    qn = W.normal_bf16(rng, (2, 8, 128))
    out = torch.empty((2, 8, 128), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step(ids, lens, dev_bf16(qn), out, 8, scale, rope=cfg)
    gp.ctx.phase_sync(DEC)
    q_rot = _round_bf16(R.apply_rope(f64(qn), [n - 1 for n in lens], o))
    want = np.stack([OA.decode_attention(q_rot[i], f64(ks[i]), f64(vs[i]), scale) for i in range(2)])
    assert_parity(host_f64(out), want, "rope, attend only")
    # a rotating range that does not fit the head is refused, nothing changes
    before = gp.pool.stats()
    with pytest.raises(S.SpdError):
        gp.pool.decode_step(ids, [n + 1 for n in lens], dev_bf16(qn), out, 8, scale, k_new=dev_bf16(knew), v_new=dev_bf16(vnew),
                            rope=S.rope_config(rotary_dim=128, rotary_offset=64))
    assert gp.pool.stats() == before
    gp.close()


def test_decode_step_with_rope_on_the_latent_tail_mla():
    """MLA: the last 64 of the 576 latent entries are the decoupled RoPE part (interleaved pairs); the
    absorbed query carries its RoPE part in the same place."""
    import math
    from test_gpu_mla import fill_latent, mla_layer
    layer = mla_layer(16)
    gp = GpuPool(layer, 16, poison=True)
    o = R.RopeConfig(theta=10000.0, rotary_dim=64, interleaved=True)
    cfg = _lib_cfg(o, offset=512)
    scale = 1.0 / math.sqrt(192)
    start = (62, 127)
    _, cs, ids = fill_latent(gp, start, seed=151)
    cs = [c.copy() for c in cs]
    rng = np.random.default_rng(152)
    lens = list(start)
    for step in range(3):
        lens = [n + 1 for n in lens]
        cnew = W.normal_bf16(rng, (2, 576))
        qn = W.normal_bf16(rng, (2, 16, 576), 0.3)
        out = torch.empty((2, 16, 512), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, lens, dev_bf16(qn), out, 16, scale, k_new=dev_bf16(cnew), rope=cfg)
        gp.ctx.phase_sync(DEC)
        pos = [n - 1 for n in lens]
        q_rot = _round_bf16(_oracle(f64(qn), pos, o, 512))
        c_rot = W.to_bf16_bits(_oracle(f64(cnew)[:, None, :], pos, o, 512)[:, 0, :])
        for i in range(2):
            cs[i] = np.concatenate([cs[i], c_rot[i][None]])
        want = np.stack([OA.mla_decode_latent(q_rot[i], f64(cs[i]), scale, 512) for i in range(2)])
        assert_parity(host_f64(out), want, f"mla rope + append step {step}")
    gp.close()
