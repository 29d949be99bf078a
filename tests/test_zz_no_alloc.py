"""The decode step that allocates nothing (spd_decode_step_noalloc), through the C ABI: its output against
spd_decode_step's on the same inputs (same kernels: bit for bit, which is inside the parity bar) and
against the fp64 oracle, on two calls in a row, the second with a smaller batch; the limits are enforced."""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as OA
from paper_2504_19867_amd import semipd as S
from gpu_util import DEV, GpuPool, assert_parity, dev_bf16, f64, host_bits, host_f64

pytestmark = pytest.mark.gpu
PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE


def _fill(gp, ctx_lens, seed, first_id):
    L = gp.layer
    q, ks, vs = W.decode_inputs(L, ctx_lens, seed)
    ids = [first_id + i for i in range(len(ctx_lens))]
    for rid, n, kb, vb in zip(ids, ctx_lens, ks, vs):
        gp.pool.kv_reserve(rid, n)
        gp.pool.kv_write(DEC, rid, 0, n, dev_bf16(kb), dev_bf16(vb))
    gp.ctx.phase_sync(DEC)
    return q, ks, vs, ids


def test_noalloc_decode_equals_decode_step_twice_second_call_smaller():
    layer = W.LayerShape("gqa", 32, 8, 128, 128, 16)
    gp = GpuPool(layer, 2048, poison=True)
    gp.ctx.set_partition(128, 128)
    scale = 1.0 / math.sqrt(layer.dim_qk)
    # first call: contexts long enough for several split-K chunks (the partials go through the scratch array);
    # second call: fewer, shorter requests, one of them a single token
    cases = [((3000, 517, 1, 2049, 4096, 16, 33, 1200), 11, 100), ((700, 1, 95), 12, 200)]
    for ctx_lens, seed, first_id in cases:
        q, ks, vs, ids = _fill(gp, ctx_lens, seed, first_id)
        tq = dev_bf16(q)
        out_a = torch.full((len(ids), layer.n_q_heads, layer.dim_v), float("nan"), dtype=torch.bfloat16, device=DEV)
        out_b = torch.full_like(out_a, float("nan"))
        batch_a = gp.pool.make_decode_batch(ids, ctx_lens, tq, out_a, layer.n_q_heads, scale)
        batch_b = gp.pool.make_decode_batch(ids, ctx_lens, tq, out_b, layer.n_q_heads, scale)
        gp.pool.decode_step_batch(batch_a)
        gp.pool.decode_step_noalloc_batch(batch_b)
        gp.ctx.phase_sync(DEC)
        assert np.array_equal(host_bits(out_a), host_bits(out_b)), "noalloc decode differs from spd_decode_step"
        want = np.stack([OA.decode_attention(f64(q[i]), f64(ks[i]), f64(vs[i]), scale) for i in range(len(ids))])
        assert_parity(host_f64(out_b), want, f"noalloc decode, contexts {ctx_lens}")
    gp.close()


def test_noalloc_decode_with_append_and_mla():
    # MLA latent pool, append variant: the new latent row goes to the page in the same call
    layer = W.get_config("c4").layer
    gp = GpuPool(layer, 256)
    gp.ctx.set_partition(128, 128)
    scale = 1.0 / math.sqrt(layer.dim_qk)
    for ctx_lens, seed, first_id in [((1500, 65, 640, 2047), 21, 300), ((64, 3), 22, 400)]:
        q, cs = W.mla_decode_inputs(layer, ctx_lens, seed)
        ids = [first_id + i for i in range(len(ctx_lens))]
        for rid, n, c in zip(ids, ctx_lens, cs):
            if n > 1:
                gp.pool.kv_reserve(rid, n - 1)
                gp.pool.kv_write(DEC, rid, 0, n - 1, dev_bf16(c[: n - 1]))
        gp.ctx.phase_sync(DEC)
        tq = dev_bf16(q)
        new_rows = dev_bf16(np.stack([c[n - 1] for n, c in zip(ctx_lens, cs)]))
        out = torch.full((len(ids), layer.n_q_heads, layer.latent_v_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
        batch = gp.pool.make_decode_batch(ids, ctx_lens, tq, out, layer.n_q_heads, scale, k_new=new_rows)
        gp.pool.decode_step_noalloc_batch(batch)
        gp.ctx.phase_sync(DEC)
        want = np.stack([OA.mla_decode_latent(f64(q[i]), f64(cs[i]), scale, layer.latent_v_dim) for i in range(len(ids))])
        assert_parity(host_f64(out), want, f"noalloc MLA decode with append, contexts {ctx_lens}")
        # the same step again through the allocating entry point, attend only: bit for bit
        out2 = torch.full_like(out, float("nan"))
        gp.pool.decode_step_batch(gp.pool.make_decode_batch(ids, ctx_lens, tq, out2, layer.n_q_heads, scale))
        gp.ctx.phase_sync(DEC)
        assert np.array_equal(host_bits(out), host_bits(out2))
    gp.close()


def test_noalloc_limits_are_enforced_and_change_nothing():
    meta, ws = S.noalloc_limits()
    assert meta == 256 * 1024 and ws == 32 * 1024 * 1024
    layer = W.LayerShape("gqa", 8, 8, 64, 64, 16)
    n_pages = 70000
    gp = GpuPool(layer, n_pages)
    # a block table beyond the metadata limit: one request of 66 000 pages (4 bytes each)
    n = 66000 * 16
    gp.pool.kv_reserve(1, n)
    q = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device=DEV)
    before = gp.pool.stats()
    with pytest.raises(S.SpdError) as e:
        gp.pool.decode_step_noalloc_batch(gp.pool.make_decode_batch([1], [n], q, out, 8, 0.125))
    assert e.value.status == S.SPD_ETOOBIG
    assert gp.pool.stats() == before
    gp.close()
