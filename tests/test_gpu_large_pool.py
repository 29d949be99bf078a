"""GPU parity on a pool larger than 4 GiB: every page the checked requests own lies beyond byte offset 2^32 of the
pool (a filler request holds the pages below), so page addressing that dropped to 32 bits anywhere on the way
(page number x page bytes, a block table entry widened too late) reads or writes the wrong page and fails here.
One case per KV layout: prefill page write, gather, decode over the written pages, decode with append."""
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
FOUR_GIB = 1 << 32


def occupy_low_pages(gp, ora, page_bytes, seed):
    """A filler request takes every page that starts below 4 GiB; the free list above is then scrambled."""
    P = gp.layer.page_tokens
    n_low = -(-FOUR_GIB // page_bytes)
    gp.pool.kv_reserve(7_000_000, n_low * P)
    ora.reserve(7_000_000, n_low * P)
    for op, r, n in W.scramble_ops(2000, P, seed=seed):
        (gp.pool.kv_reserve(r, n), ora.reserve(r, n)) if op == "reserve" else (gp.pool.kv_free(r), ora.free(r))
    return n_low


def assert_table_above_4gib(gp, ora, rid, page_bytes, n_low):
    table = gp.pool.kv_block_table(rid)
    assert table == ora.block_table(rid)
    assert min(table) >= n_low and min(table) * page_bytes >= FOUR_GIB, (min(table), page_bytes)
    return table


def test_gqa_pages_beyond_4gib():
    L = W.LayerShape("gqa", 32, 8, 128, 128, 16)
    num_pages = 73728                                   # x 64 KiB = 4.5 GiB
    page_bytes = L.page_bytes
    assert num_pages * page_bytes > FOUR_GIB + (256 << 20)
    gp = GpuPool(L, num_pages, poison=True)
    ora = BlockAllocator(num_pages, L.page_tokens)
    n_low = occupy_low_pages(gp, ora, page_bytes, seed=61)
    scale = 1.0 / math.sqrt(128)

    # prefill step: attention + page write
    lens = (300, 77, 1)
    q, k, v, cu = W.prefill_inputs(L, lens, seed=62)
    out = torch.empty((q.shape[0], 32, 128), dtype=torch.bfloat16, device=DEV)
    ids = [1, 2, 3]
    gp.pool.prefill_step(ids, cu, dev_bf16(q), dev_bf16(k), dev_bf16(v), out, 32, 8, 128, 128, scale)
    gp.ctx.phase_sync(PRE)
    assert_parity(host_f64(out), OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale), "prefill above 4 GiB")
    for r, a, b in zip(ids, cu[:-1], cu[1:]):
        ora.reserve(r, int(b - a))
        assert_table_above_4gib(gp, ora, r, page_bytes, n_low)
        ko = torch.zeros((int(b - a), 8, 128), dtype=torch.bfloat16, device=DEV)
        vo = torch.zeros_like(ko)
        gp.pool.kv_gather(PRE, r, int(b - a), ko, vo)
        gp.ctx.phase_sync(PRE)
        np.testing.assert_array_equal(host_bits(ko), k[a:b])
        np.testing.assert_array_equal(host_bits(vo), v[a:b])

    # decode over the pages the prefill step wrote, appending one token per step (request 1 crosses a page border)
    ks = [k[a:b].copy() for a, b in zip(cu[:-1], cu[1:])]
    vs = [v[a:b].copy() for a, b in zip(cu[:-1], cu[1:])]
    cur = list(lens)
    rng = np.random.default_rng(63)
    gp.ctx.phase_wait_for(DEC, PRE)
    for step in range(5):
        cur = [n + 1 for n in cur]
        kn, vn, qn = W.normal_bf16(rng, (3, 8, 128)), W.normal_bf16(rng, (3, 8, 128)), W.normal_bf16(rng, (3, 32, 128))
        od = torch.empty((3, 32, 128), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, cur, dev_bf16(qn), od, 32, scale, k_new=dev_bf16(kn), v_new=dev_bf16(vn))
        gp.ctx.phase_sync(DEC)
        for i, r in enumerate(ids):
            ks[i] = np.concatenate([ks[i], kn[i][None]])
            vs[i] = np.concatenate([vs[i], vn[i][None]])
            ora.reserve(r, cur[i])
            assert_table_above_4gib(gp, ora, r, page_bytes, n_low)
        want = np.stack([OA.decode_attention(f64(qn[i]), f64(ks[i]), f64(vs[i]), scale) for i in range(3)])
        assert_parity(host_f64(od), want, f"decode + append above 4 GiB, step {step}")

    # longer contexts written through kv_write: split-K over pages that all lie above 4 GiB
    ctx_lens = (2049, 1000, 17)
    qd, kd, vd = W.decode_inputs(L, ctx_lens, seed=64)
    dids = [11, 12, 13]
    for r, n, kb, vb in zip(dids, ctx_lens, kd, vd):
        gp.pool.kv_reserve(r, n)
        ora.reserve(r, n)
        assert_table_above_4gib(gp, ora, r, page_bytes, n_low)
        gp.pool.kv_write(DEC, r, 0, n, dev_bf16(kb), dev_bf16(vb))
    od = torch.empty((3, 32, 128), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step(dids, ctx_lens, dev_bf16(qd), od, 32, scale)
    gp.ctx.phase_sync(DEC)
    want = np.stack([OA.decode_attention(f64(qd[i]), f64(kd[i]), f64(vd[i]), scale) for i in range(3)])
    assert_parity(host_f64(od), want, "split-K decode above 4 GiB")
    assert gp.pool.kv_free_list() == ora.free_stack and gp.pool.stats()[3] == ora.op_seq
    gp.close()


def test_mla_latent_pages_beyond_4gib_with_k_v_made_from_the_latent():
    """The MLA case also ties the two forms together: the prefill step's K and V are the cached latent rows sent
    through one set of up-projection weights (as in the model), so its last output row and the absorbed-form decode
    over the latent pages it wrote describe the same attention."""
    L = W.LayerShape("mla", 16, 1, 192, 128, 64, latent_dim=576, latent_v_dim=512)
    H, lora, rope, nope = 16, 512, 64, 128
    num_pages = 65536                                   # x 72 KiB = 4.5 GiB
    page_bytes = L.page_bytes
    assert num_pages * page_bytes > FOUR_GIB + (256 << 20)
    gp = GpuPool(L, num_pages, poison=True)
    ora = BlockAllocator(num_pages, L.page_tokens)
    n_low = occupy_low_pages(gp, ora, page_bytes, seed=71)
    scale = 1.0 / math.sqrt(192)

    lens = (130, 300, 64)
    T = sum(lens)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    rng = np.random.default_rng(72)
    latent = W.normal_bf16(rng, (T, 576))
    w_uk, w_uv = W.mla_weights(H, nope, lora, 128, seed=73)
    lat = f64(latent)
    k_full = np.concatenate([np.einsum("tc,hnc->thn", lat[:, :lora], w_uk),
                             np.broadcast_to(lat[:, None, lora:], (T, H, rope))], axis=-1)
    k = W.to_bf16_bits(k_full.astype(np.float32))
    v = W.to_bf16_bits(np.einsum("tc,hcd->thd", lat[:, :lora], w_uv).astype(np.float32))
    q = W.normal_bf16(rng, (T, H, 192))
    out = torch.empty((T, H, 128), dtype=torch.bfloat16, device=DEV)
    ids = [1, 2, 3]
    gp.pool.prefill_step(ids, cu, dev_bf16(q), dev_bf16(k), dev_bf16(v), out, H, H, 192, 128, scale, latent=dev_bf16(latent))
    gp.ctx.phase_sync(PRE)
    assert_parity(host_f64(out), OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale), "mla prefill above 4 GiB")
    for r, a, b in zip(ids, cu[:-1], cu[1:]):
        ora.reserve(r, int(b - a))
        assert_table_above_4gib(gp, ora, r, page_bytes, n_low)
        back = torch.zeros((int(b - a), 576), dtype=torch.bfloat16, device=DEV)
        gp.pool.kv_gather(PRE, r, int(b - a), back)
        gp.ctx.phase_sync(PRE)
        np.testing.assert_array_equal(host_bits(back), latent[a:b])

    # absorbed-form decode of each prompt's last token over the latent pages the prefill step wrote
    last = [int(b) - 1 for b in cu[1:]]
    qf = f64(q[last])                                                        # [3, H, 192]
    qabs = np.concatenate([np.einsum("bhn,hnc->bhc", qf[..., :nope], w_uk), qf[..., nope:]], axis=-1)
    qabs_bits = W.to_bf16_bits(qabs.astype(np.float32))
    od = torch.empty((3, H, lora), dtype=torch.bfloat16, device=DEV)
    gp.ctx.phase_wait_for(DEC, PRE)
    gp.pool.decode_step(ids, list(lens), dev_bf16(qabs_bits), od, H, scale)
    gp.ctx.phase_sync(DEC)
    want = np.stack([OA.mla_decode_latent(f64(qabs_bits[i]), lat[cu[i]:cu[i + 1]], scale, lora) for i in range(3)])
    assert_parity(host_f64(od), want, "mla decode above 4 GiB")
    # the same attention in both forms: the decode output sent through W_UV is the prefill step's last row
    # (K, V and the absorbed query were each rounded to bf16 once more on the way, hence the wider bar)
    via_latent = np.einsum("bhc,hcd->bhd", host_f64(od), w_uv)
    assert np.abs(via_latent - host_f64(out)[last]).max() <= 3e-2

    # append: one new latent row per step, request 3 crosses a page border on the first
    cs = [latent[a:b].copy() for a, b in zip(cu[:-1], cu[1:])]
    cur = list(lens)
    for step in range(3):
        cur = [n + 1 for n in cur]
        cnew = W.normal_bf16(rng, (3, 576))
        qn = W.normal_bf16(rng, (3, H, 576), 0.3)
        gp.pool.decode_step(ids, cur, dev_bf16(qn), od, H, scale, k_new=dev_bf16(cnew))
        gp.ctx.phase_sync(DEC)
        for i, r in enumerate(ids):
            cs[i] = np.concatenate([cs[i], cnew[i][None]])
            ora.reserve(r, cur[i])
            assert_table_above_4gib(gp, ora, r, page_bytes, n_low)
        want = np.stack([OA.mla_decode_latent(f64(qn[i]), f64(cs[i]), scale, lora) for i in range(3)])
        assert_parity(host_f64(od), want, f"mla decode + append above 4 GiB, step {step}")
    assert gp.pool.kv_free_list() == ora.free_stack and gp.pool.stats()[3] == ora.op_seq
    gp.close()
