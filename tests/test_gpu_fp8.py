"""GPU parity of the FP8 latent KV cache (pool kind SPD_KV_MLA_LATENT_FP8): the bytes in the pages are the oracle's
quantisation bit for bit, the gather hands back its dequantised rows bit for bit, and the decode step attends over
exactly those rows (spec bar against the fp64 oracle on the dequantised inputs)."""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as OA
from oracle import fp8 as F8
from oracle.allocator import BlockAllocator
from paper_2504_19867_amd import semipd as S
from gpu_util import DEV, GpuPool, assert_parity, dev_bf16, f64, host_bits, host_f64

pytestmark = pytest.mark.gpu
PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE
ROW = 656


def fp8_pool(H=16, P=64, pages=64, poison=True):
    layer = W.LayerShape("mla", H, 1, 192, 128, P, latent_dim=576, latent_v_dim=512)
    return GpuPool(layer, pages, poison=poison, kind=S.SPD_KV_MLA_LATENT_FP8)


def oracle_rows(latent_bits):
    """(packed page rows [n, 656] uint8, dequantised rows [n, 576] float64, the same rounded to bf16 the way the
    kernels do it: fp32 product, one rounding)"""
    lat = W.bf16_bits_to_f32(latent_bits)
    codes, scale, rope = F8.quantise_latent(lat)
    rows = F8.pack_rows(codes, scale, latent_bits[:, 512:])
    deq = F8.dequantise_latent(codes, scale, rope)
    n = codes.shape[0]
    prod32 = (F8.e4m3_decode(codes).astype(np.float32).reshape(n, 4, 128) * scale[:, :, None]).reshape(n, 512)
    deq_bf16 = np.concatenate([W.to_bf16_bits(prod32), latent_bits[:, 512:]], axis=1)
    return rows, deq, deq_bf16


def page_rows(gp, table, n):
    """the first n cached rows of a request, as raw bytes out of the pool memory"""
    P = gp.layer.page_tokens
    mem = gp.mem.cpu().numpy()
    out = np.empty((n, ROW), dtype=np.uint8)
    for t in range(n):
        off = table[t // P] * P * ROW + (t % P) * ROW
        out[t] = mem[off:off + ROW]
    return out


def special_latent(rng, n):
    lat = W.normal_bf16(rng, (n, 576))
    f = W.bf16_bits_to_f32(lat)
    if n > 3:
        f[1, :128] = 0.0                                # an all-zero block
        f[2, 200] = 250.0                               # an outlier that sets its block's scale
        f[3, 256:384] *= 1e-3                           # a block of small values
    return W.to_bf16_bits(f)


@pytest.mark.parametrize("P", [64, 32])
def test_pages_hold_the_oracles_bytes_and_gather_its_dequantised_rows(P):
    gp = fp8_pool(P=P, pages=32)
    ora = BlockAllocator(32, P)
    for op, r, n in W.scramble_ops(20, P, seed=3):
        (gp.pool.kv_reserve(r, n), ora.reserve(r, n)) if op == "reserve" else (gp.pool.kv_free(r), ora.free(r))
    n = 3 * P + 11
    lat = special_latent(np.random.default_rng(4), n)
    gp.pool.kv_reserve(7, n)
    ora.reserve(7, n)
    table = gp.pool.kv_block_table(7)
    assert table == ora.block_table(7)
    for a, b in ((0, 5), (5, P + 9), (P + 9, n)):       # pieces whose borders fall inside tiles and pages
        gp.pool.kv_write(PRE, 7, a, b - a, dev_bf16(lat[a:b]))
    back = torch.zeros((n, 576), dtype=torch.bfloat16, device=DEV)
    gp.pool.kv_gather(PRE, 7, n, back)
    gp.ctx.phase_sync(PRE)
    rows, _, deq_bf16 = oracle_rows(lat)
    np.testing.assert_array_equal(page_rows(gp, table, n), rows)
    np.testing.assert_array_equal(host_bits(back), deq_bf16)
    # slots of the last page beyond the request were not touched
    last = page_rows(gp, table, len(table) * P)[n:]
    assert (last.view(np.uint16) == 0x7FC0).all()
    gp.close()


@pytest.mark.parametrize("H", [16, 5])
def test_fp8_decode_edges_and_split_k(H):
    ctx_lens = (1, 15, 16, 17, 33, 64, 65, 200, 1000, 2500, 4097)
    gp = fp8_pool(H=H, pages=160)
    for op, r, n in W.scramble_ops(140, 64, seed=5):
        gp.pool.kv_reserve(r, n) if op == "reserve" else gp.pool.kv_free(r)
    scale = 1.0 / math.sqrt(192)
    q, cs = W.mla_decode_inputs(gp.layer, ctx_lens, seed=16 + H)
    ids = [100 + i for i in range(len(ctx_lens))]
    deqs = []
    for rid, n, c in zip(ids, ctx_lens, cs):
        gp.pool.kv_reserve(rid, n)
        gp.pool.kv_write(DEC, rid, 0, n, dev_bf16(c))
        deqs.append(oracle_rows(c)[1])
    out = torch.empty((len(ids), H, 512), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step(ids, ctx_lens, dev_bf16(q), out, H, scale)
    gp.ctx.phase_sync(DEC)
    got = host_f64(out)
    for i, n in enumerate(ctx_lens):
        want = OA.mla_decode_latent(f64(q[i]), deqs[i], scale, 512)
        assert_parity(got[i], want, f"fp8 mla decode n={n}")
    # context 1: the output is the token's dequantised leading 512 entries, for every head
    np.testing.assert_array_equal(host_bits(out)[0], np.repeat(oracle_rows(cs[0])[2][:1, :512], H, axis=0))
    # a prefix of the cached context: the rest of the page is ignored
    short = [max(1, n - 7) for n in ctx_lens]
    gp.pool.decode_step(ids, short, dev_bf16(q), out, H, scale)
    gp.ctx.phase_sync(DEC)
    want2 = np.stack([OA.mla_decode_latent(f64(q[i]), deqs[i][:m], scale, 512) for i, m in enumerate(short)])
    assert_parity(host_f64(out), want2, "fp8 mla decode on a prefix")
    gp.close()


def test_fp8_append_and_prefill_write_the_same_pages():
    gp = fp8_pool(H=16, pages=16)
    ora = BlockAllocator(16, 64)
    scale = 1.0 / math.sqrt(192)
    # a prefill step writes the prompts' latent rows (attention in the un-absorbed form on bf16 K, V as ever)
    lens = (62, 127)
    q, k, v, latent, cu = W.mla_prefill_inputs(gp.layer, lens, seed=21)
    outp = torch.empty((q.shape[0], 16, 128), dtype=torch.bfloat16, device=DEV)
    ids = [1, 2]
    gp.pool.prefill_step(ids, cu, dev_bf16(q), dev_bf16(k), dev_bf16(v), outp, 16, 16, 192, 128, scale, latent=dev_bf16(latent))
    gp.ctx.phase_sync(PRE)
    assert_parity(host_f64(outp), OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale), "prefill on an fp8 latent pool")
    cs = []
    for r, a, b in zip(ids, cu[:-1], cu[1:]):
        ora.reserve(r, int(b - a))
        table = gp.pool.kv_block_table(r)
        assert table == ora.block_table(r)
        np.testing.assert_array_equal(page_rows(gp, table, int(b - a)), oracle_rows(latent[a:b])[0])
        cs.append(latent[a:b].copy())
    # decode steps append one latent row each; both requests cross a page border
    rng = np.random.default_rng(22)
    cur = list(lens)
    gp.ctx.phase_wait_for(DEC, PRE)
    for step in range(4):
        cur = [n + 1 for n in cur]
        cnew = W.normal_bf16(rng, (2, 576))
        qn = W.normal_bf16(rng, (2, 16, 576), 0.3)
        out = torch.empty((2, 16, 512), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, cur, dev_bf16(qn), out, 16, scale, k_new=dev_bf16(cnew))
        gp.ctx.phase_sync(DEC)
        for i, r in enumerate(ids):
            cs[i] = np.concatenate([cs[i], cnew[i][None]])
            ora.reserve(r, cur[i])
            table = gp.pool.kv_block_table(r)
            assert table == ora.block_table(r)
            np.testing.assert_array_equal(page_rows(gp, table, cur[i]), oracle_rows(cs[i])[0])
        want = np.stack([OA.mla_decode_latent(f64(qn[i]), oracle_rows(cs[i])[1], scale, 512) for i in range(2)])
        assert_parity(host_f64(out), want, f"fp8 append step {step}")
    assert gp.pool.kv_free_list() == ora.free_stack
    # RoPE inside the decode step is not offered on such a pool
    with pytest.raises(S.SpdError) as e:
        gp.pool.decode_step(ids, cur, dev_bf16(qn), out, 16, scale, rope=S.rope_config(rotary_dim=64, rotary_offset=512))
    assert e.value.status == S.SPD_EINVAL
    gp.close()
