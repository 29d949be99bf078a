"""GPU parity of the MLA (latent KV cache) paths against the fp64 oracle: latent page write /
gather (bit-exact), absorbed-form decode over the latent pool, and the MHA-form prefill (qk 192,
v 128) with the latent page write."""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as OA
from oracle.allocator import BlockAllocator
from paper_2504_19867_amd import semipd as S
from gpu_util import DEV, GpuPool, assert_parity, dev_bf16, f64, host_bits, host_f64

pytestmark = pytest.mark.gpu
PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE


def mla_layer(heads=16, P=64):
    return W.LayerShape("mla", heads, 1, 192, 128, P, latent_dim=576, latent_v_dim=512)


def fill_latent(gp, ctx_lens, seed, first_id=100):
    q, cs = W.mla_decode_inputs(gp.layer, ctx_lens, seed)
    ids = [first_id + i for i in range(len(ctx_lens))]
    for rid, n, c in zip(ids, ctx_lens, cs):
        gp.pool.kv_reserve(rid, n)
        gp.pool.kv_write(DEC, rid, 0, n, dev_bf16(c))
    gp.ctx.phase_sync(DEC)
    return q, cs, ids


def oracle_mla(q, cs, scale):
    return np.stack([OA.mla_decode_latent(f64(q[i]), f64(cs[i]), scale, 512) for i in range(len(cs))])


@pytest.mark.parametrize("P", [64, 32])
def test_latent_page_write_gather_bit_exact(P):
    layer = mla_layer(P=P)
    gp = GpuPool(layer, 32, poison=True)
    ora = BlockAllocator(32, P)
    for op, r, n in W.scramble_ops(20, P, seed=3):
        (gp.pool.kv_reserve(r, n), ora.reserve(r, n)) if op == "reserve" else (gp.pool.kv_free(r), ora.free(r))
    n = 3 * P + 11
    _, cs = W.mla_decode_inputs(layer, (n,), seed=4)
    gp.pool.kv_reserve(7, n)
    ora.reserve(7, n)
    table = gp.pool.kv_block_table(7)
    assert table == ora.block_table(7)
    for a, b in ((0, 5), (5, P + 9), (P + 9, n)):
        gp.pool.kv_write(PRE, 7, a, b - a, dev_bf16(cs[0][a:b]))
    back = torch.zeros((n, 576), dtype=torch.bfloat16, device=DEV)
    gp.pool.kv_gather(PRE, 7, n, back)
    gp.ctx.phase_sync(PRE)
    store = OA.PagedLatent(32, P, 576, dtype=np.uint16)
    store.write(table, 0, cs[0])
    np.testing.assert_array_equal(host_bits(back), store.gather(table, n))
    gp.close()


@pytest.mark.parametrize("H", [16, 8, 5])
def test_mla_decode_edges_and_split_k(H):
    layer = mla_layer(H)
    ctx_lens = (1, 31, 32, 33, 63, 64, 65, 200, 1000, 2500, 4097)
    gp = GpuPool(layer, 160, poison=True)
    for op, r, n in W.scramble_ops(140, 64, seed=5):
        gp.pool.kv_reserve(r, n) if op == "reserve" else gp.pool.kv_free(r)
    scale = 1.0 / math.sqrt(192)
    q, cs, ids = fill_latent(gp, ctx_lens, seed=6 + H)
    out = torch.empty((len(ids), H, 512), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step(ids, ctx_lens, dev_bf16(q), out, H, scale)
    gp.ctx.phase_sync(DEC)
    got, want = host_f64(out), oracle_mla(q, cs, scale)
    for i, n in enumerate(ctx_lens):
        assert_parity(got[i], want[i], f"mla decode n={n}")
    # context 1: the output is exactly the token's first 512 latent dims, for every head
    np.testing.assert_array_equal(host_bits(out)[0], np.repeat(cs[0][:1, :512], H, axis=0))
    # a prefix of the cached context: the rest of the page must be ignored
    short = [max(1, n - 7) for n in ctx_lens]
    gp.pool.decode_step(ids, short, dev_bf16(q), out, H, scale)
    gp.ctx.phase_sync(DEC)
    want2 = np.stack([OA.mla_decode_latent(f64(q[i]), f64(cs[i][:m]), scale, 512) for i, m in enumerate(short)])
    assert_parity(host_f64(out), want2, "mla decode on a prefix")
    gp.close()


def test_mla_decode_append_matches_oracle_and_allocator():
    layer = mla_layer(16)
    gp = GpuPool(layer, 16, poison=True)
    ora = BlockAllocator(16, 64)
    scale = 1.0 / math.sqrt(192)
    start = (62, 127)
    _, cs, ids = fill_latent(gp, start, seed=9)
    for r, n in zip(ids, start):
        ora.reserve(r, n)
    cs = [c.copy() for c in cs]
    rng = np.random.default_rng(10)
    lens = list(start)
    for step in range(4):
        lens = [n + 1 for n in lens]
        cnew = W.normal_bf16(rng, (2, 576))
        qn = W.normal_bf16(rng, (2, 16, 576), 0.3)
        out = torch.empty((2, 16, 512), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, lens, dev_bf16(qn), out, 16, scale, k_new=dev_bf16(cnew))
        gp.ctx.phase_sync(DEC)
        for i in range(2):
            cs[i] = np.concatenate([cs[i], cnew[i][None]])
            ora.reserve(ids[i], lens[i])
            assert gp.pool.kv_block_table(ids[i]) == ora.block_table(ids[i])
        assert_parity(host_f64(out), oracle_mla(qn, cs, scale), f"mla append step {step}")
    assert gp.pool.kv_free_list() == ora.free_stack
    gp.close()


def test_mla_prefill_mha_form_and_latent_pages():
    layer = mla_layer(16)
    lens = (100, 300, 65)
    gp = GpuPool(layer, 16, poison=True)
    q, k, v, latent, cu = W.mla_prefill_inputs(layer, lens, seed=11)
    scale = 1.0 / math.sqrt(192)
    out = torch.empty((q.shape[0], 16, 128), dtype=torch.bfloat16, device=DEV)
    gp.pool.prefill_step([1, 2, 3], cu, dev_bf16(q), dev_bf16(k), dev_bf16(v), out, 16, 16, 192, 128, scale,
                         latent=dev_bf16(latent))
    gp.ctx.phase_sync(PRE)
    want = OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale)
    assert_parity(host_f64(out), want, "mla prefill (MHA form)")
    for r, (a, b) in zip((1, 2, 3), zip(cu[:-1], cu[1:])):
        back = torch.empty((int(b - a), 576), dtype=torch.bfloat16, device=DEV)
        gp.pool.kv_gather(PRE, r, int(b - a), back)
        gp.ctx.phase_sync(PRE)
        np.testing.assert_array_equal(host_bits(back), latent[a:b])
    # the decode kernel then reads what prefill wrote
    qd, _ = W.mla_decode_inputs(layer, lens, seed=12)
    od = torch.empty((3, 16, 512), dtype=torch.bfloat16, device=DEV)
    gp.ctx.phase_wait_for(DEC, PRE)
    gp.pool.decode_step([1, 2, 3], lens, dev_bf16(qd), od, 16, scale)
    gp.ctx.phase_sync(DEC)
    want_d = np.stack([OA.mla_decode_latent(f64(qd[i]), f64(latent[cu[i]:cu[i + 1]]), scale, 512) for i in range(3)])
    assert_parity(host_f64(od), want_d, "mla decode over prefilled latent pages")
    gp.close()


def test_c4_full_size_sampled_against_oracle():
    cfg = W.get_config("c4")
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    gp = GpuPool(L, 16384)                     # 1.2 GB of the 40 GB pool holds the whole batch
    total, _, _ = gp.ctx.device_info()
    gp.ctx.set_partition(total // 2, total // 2)
    for op, r, n in W.scramble_ops(12000, 64, seed=cfg.seed):
        gp.pool.kv_reserve(r, n) if op == "reserve" else gp.pool.kv_free(r)
    qd, cs, dids = fill_latent(gp, cfg.decode_ctx, cfg.seed + 1)
    q, k, v, latent, cu = W.mla_prefill_inputs(L, cfg.prefill_lens, cfg.seed)
    op_ = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    od = torch.empty((len(dids), L.n_q_heads, 512), dtype=torch.bfloat16, device=DEV)
    tq, tk, tv, tl, tqd = dev_bf16(q), dev_bf16(k), dev_bf16(v), dev_bf16(latent), dev_bf16(qd)
    gp.pool.prefill_step([1, 2, 3, 4], cu, tq, tk, tv, op_, L.n_q_heads, L.n_q_heads, L.dim_qk, L.dim_v, scale, latent=tl)
    gp.pool.decode_step(dids, cfg.decode_ctx, tqd, od, L.n_q_heads, scale)
    gp.ctx.phase_sync(PRE)
    gp.ctx.phase_sync(DEC)
    assert_parity(host_f64(od), oracle_mla(qd, cs, scale), "c4 decode (all 128 requests)")
    got = host_f64(op_)
    qf, kf, vf = f64(q), f64(k), f64(v)
    for r, h in [(0, 0), (2, 9), (3, 15)]:
        a, b = cu[r], cu[r + 1]
        want = OA.causal_attention(qf[a:b, h:h + 1], kf[a:b, h:h + 1], vf[a:b, h:h + 1], scale)
        assert_parity(got[a:b, h:h + 1], want, f"c4 prefill request {r} head {h}")
    gp.close()
