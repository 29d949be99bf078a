"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Bar: max abs <= 2e-2 and mean abs <= 2e-3 on bf16 outputs; page contents,
block tables and allocator state bit-exact."""
import time
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


def run_prefill(gp, lens, seed, req_ids=None):
    L = gp.layer
    q, k, v, cu = W.prefill_inputs(L, lens, seed)
    scale = 1.0 / math.sqrt(L.dim_qk)
    out = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    ids = req_ids or list(range(1, len(lens) + 1))
    tq, tk, tv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    gp.pool.prefill_step(ids, cu, tq, tk, tv, out, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale)
    gp.ctx.phase_sync(PRE)
    return (q, k, v, cu, scale), out, ids


def fill_decode_contexts(gp, ctx_lens, seed, first_id=100):
    L = gp.layer
    q, ks, vs = W.decode_inputs(L, ctx_lens, seed)
    ids = [first_id + i for i in range(len(ctx_lens))]
    for rid, n, kb, vb in zip(ids, ctx_lens, ks, vs):
        gp.pool.kv_reserve(rid, n)
        gp.pool.kv_write(DEC, rid, 0, n, dev_bf16(kb), dev_bf16(vb))
    gp.ctx.phase_sync(DEC)
    return q, ks, vs, ids


def oracle_decode(q, ks, vs, scale):
    return np.stack([OA.decode_attention(f64(q[i]), f64(ks[i]), f64(vs[i]), scale) for i in range(len(ks))])


# ----------------------------------------------------------------------------- page write / gather
@pytest.mark.parametrize("d,hkv,P", [(64, 8, 16), (128, 2, 16), (128, 3, 32)])
def test_page_write_gather_bit_exact(d, hkv, P):
    layer = W.LayerShape("gqa", hkv, hkv, d, d, P)
    gp = GpuPool(layer, 64, poison=True)
    ora_alloc = BlockAllocator(64, P)
    for op, r, n in W.scramble_ops(40, P, seed=d + hkv):          # scattered physical pages on both sides
        (gp.pool.kv_reserve(r, n), ora_alloc.reserve(r, n)) if op == "reserve" else (gp.pool.kv_free(r), ora_alloc.free(r))
    n = 5 * P + 7
    _, ks, vs = W.decode_inputs(layer, (n,), seed=7)
    kb, vb = ks[0], vs[0]
    gp.pool.kv_reserve(9, n)
    ora_alloc.reserve(9, n)
    table = gp.pool.kv_block_table(9)
    assert table == ora_alloc.block_table(9)
    # write in three pieces whose borders fall inside tiles and pages
    cuts = [0, 3, 2 * P + 5, n]
    for a, b in zip(cuts[:-1], cuts[1:]):
        gp.pool.kv_write(PRE, 9, a, b - a, dev_bf16(kb[a:b]), dev_bf16(vb[a:b]))
    ko = torch.zeros((n, hkv, d), dtype=torch.bfloat16, device=DEV)
    vo = torch.zeros((n, hkv, d), dtype=torch.bfloat16, device=DEV)
    gp.pool.kv_gather(PRE, 9, n, ko, vo)
    gp.ctx.phase_sync(PRE)
    # the oracle's own paged store, filled through the same block table, must gather the same bits
    store = OA.PagedKV(64, P, hkv, d, d, dtype=np.uint16)
    store.write(table, 0, kb, vb)
    gk, gv = store.gather(table, n)
    np.testing.assert_array_equal(host_bits(ko), gk)
    np.testing.assert_array_equal(host_bits(vo), gv)
    # pages the request does not own were not touched
    gp.pool.kv_reserve(10, P)
    other = torch.zeros((P, hkv, d), dtype=torch.bfloat16, device=DEV)
    other_v = torch.zeros((P, hkv, d), dtype=torch.bfloat16, device=DEV)
    gp.pool.kv_gather(PRE, 10, P, other, other_v)
    gp.ctx.phase_sync(PRE)
    assert (host_bits(other) == 0x7FC0).all() and (host_bits(other_v) == 0x7FC0).all()
    gp.close()


# ----------------------------------------------------------------------------- config 1
def test_c1_prefill_and_page_contents():
    cfg = W.get_config("c1")
    gp = GpuPool(cfg.layer, cfg.num_pages, poison=True)
    (q, k, v, cu, scale), out, ids = run_prefill(gp, cfg.prefill_lens, cfg.seed)
    want = OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale)
    assert_parity(host_f64(out), want, "c1 prefill")
    ora = BlockAllocator(cfg.num_pages, cfg.layer.page_tokens)
    for r, (a, b) in zip(ids, zip(cu[:-1], cu[1:])):
        ora.reserve(r, int(b - a))
        assert gp.pool.kv_block_table(r) == ora.block_table(r)
        n = int(b - a)
        ko = torch.empty((n, cfg.layer.n_kv_heads, cfg.layer.dim_qk), dtype=torch.bfloat16, device=DEV)
        vo = torch.empty_like(ko)
        gp.pool.kv_gather(PRE, r, n, ko, vo)
        gp.ctx.phase_sync(PRE)
        np.testing.assert_array_equal(host_bits(ko), k[a:b])      # the page write is a bit-exact copy
        np.testing.assert_array_equal(host_bits(vo), v[a:b])
    assert gp.pool.kv_free_list() == ora.free_stack
    gp.close()


def test_c1_decode():
    cfg = W.get_config("c1")
    gp = GpuPool(cfg.layer, cfg.num_pages, poison=True)
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    q, ks, vs, ids = fill_decode_contexts(gp, cfg.decode_ctx, cfg.seed + 1)
    out = torch.empty((len(ids), L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step(ids, cfg.decode_ctx, dev_bf16(q), out, L.n_q_heads, scale)
    gp.ctx.phase_sync(DEC)
    assert_parity(host_f64(out), oracle_decode(q, ks, vs, scale), "c1 decode")
    gp.close()


def test_c1_concurrent_on_a_50_50_partition_equals_solo_bit_for_bit():
    cfg = W.get_config("c1")
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    gp = GpuPool(L, cfg.num_pages)
    total, xcds, gran = gp.ctx.device_info()
    qd, ks, vs, dids = fill_decode_contexts(gp, cfg.decode_ctx, cfg.seed + 1)
    q, k, v, cu = W.prefill_inputs(L, cfg.prefill_lens, cfg.seed)
    tq, tk, tv, tqd = dev_bf16(q), dev_bf16(k), dev_bf16(v), dev_bf16(qd)

    def both():
        op = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
        od = torch.empty((len(dids), L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
        gp.pool.prefill_step([1, 2], cu, tq, tk, tv, op, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale)
        gp.pool.decode_step(dids, cfg.decode_ctx, tqd, od, L.n_q_heads, scale)
        gp.ctx.phase_sync(PRE)
        gp.ctx.phase_sync(DEC)
        return host_bits(op), host_bits(od)

    solo_p, solo_d = both()                                   # initial partition: (all, all)
    assert gp.ctx.get_partition() == (total, total, total, total)
    gp.ctx.set_partition(total // 2, total // 2)
    assert gp.ctx.get_partition() == (total, total, total // 2, total // 2)      # staged, not yet adopted
    part_p, part_d = both()
    assert gp.ctx.get_partition() == (total // 2,) * 4
    np.testing.assert_array_equal(part_p, solo_p)
    np.testing.assert_array_equal(part_d, solo_d)
    assert_parity(f64(part_p), OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale), "c1 prefill 50/50")
    assert_parity(f64(part_d), oracle_decode(qd, ks, vs, scale), "c1 decode 50/50")
    # the pool and the block tables survive the resize untouched
    for r in dids:
        assert len(gp.pool.kv_block_table(r)) > 0
    gp.close()


# ----------------------------------------------------------------------------- edge cases
@pytest.mark.parametrize("H,Hkv,d", [(8, 2, 128), (16, 2, 128), (6, 6, 64), (16, 1, 128)])
def test_decode_context_edges_and_split_k(H, Hkv, d):
    layer = W.LayerShape("gqa", H, Hkv, d, d, 16)
    ctx_lens = (1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 1000, 2049)
    gp = GpuPool(layer, 400, poison=True)
    for op, r, n in W.scramble_ops(300, 16, seed=11):
        gp.pool.kv_reserve(r, n) if op == "reserve" else gp.pool.kv_free(r)
    scale = 1.0 / math.sqrt(d)
    q, ks, vs, ids = fill_decode_contexts(gp, ctx_lens, seed=H * 7 + d)
    out = torch.empty((len(ids), H, d), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step(ids, ctx_lens, dev_bf16(q), out, H, scale)
    gp.ctx.phase_sync(DEC)
    got, want = host_f64(out), oracle_decode(q, ks, vs, scale)
    for i, n in enumerate(ctx_lens):
        assert_parity(got[i], want[i], f"decode n={n}")
    # context 1: softmax over one token is exactly that token's V
    np.testing.assert_array_equal(host_bits(out)[0], np.repeat(vs[0][0], H // Hkv, axis=0))
    # attending to a prefix of a longer cached context must ignore the rest of the page
    short = [max(1, n - 5) for n in ctx_lens]
    gp.pool.decode_step(ids, short, dev_bf16(q), out, H, scale)
    gp.ctx.phase_sync(DEC)
    want2 = np.stack([OA.decode_attention(f64(q[i]), f64(ks[i][:m]), f64(vs[i][:m]), scale) for i, m in enumerate(short)])
    assert_parity(host_f64(out), want2, "decode on a prefix")
    gp.close()


@pytest.mark.parametrize("H,Hkv,d", [(4, 2, 128), (3, 3, 64)])
def test_prefill_ragged_lengths(H, Hkv, d):
    layer = W.LayerShape("gqa", H, Hkv, d, d, 16)
    lens = (1, 63, 64, 65, 127, 128, 129, 300)
    gp = GpuPool(layer, 128, poison=True)
    (q, k, v, cu, scale), out, ids = run_prefill(gp, lens, seed=21 + d)
    want = OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale)
    got = host_f64(out)
    for r in range(len(lens)):
        assert_parity(got[cu[r]:cu[r + 1]], want[cu[r]:cu[r + 1]], f"prefill len={lens[r]}")
    # first row of every request attends to itself only: output is exactly V[0]
    for r in range(len(lens)):
        np.testing.assert_array_equal(host_bits(out)[cu[r]], np.repeat(v[cu[r]], H // Hkv, axis=0))
    gp.close()


@pytest.mark.parametrize("rise", [30.0, 100.0, 400.0, -200.0])
@pytest.mark.parametrize("H,Hkv,d", [(8, 2, 128), (4, 4, 64)])
def test_prefill_scores_drifting_along_the_keys(H, Hkv, d, rise):
    """Scores that climb (or fall) steadily from the first key to the last: the softmax reference of a row has to
    follow them over many powers of two inside one prompt (the kernel moves it only when it must), or must stay
    where the first keys put it."""
    layer = W.LayerShape("gqa", H, Hkv, d, d, 16)
    lens = (700, 64, 1, 333)
    scale = 1.0 / math.sqrt(d)
    q, k, v, cu = W.prefill_inputs_drifting(layer, lens, seed=int(abs(rise)) + d, rise=rise, scale=scale)
    gp = GpuPool(layer, 128, poison=True)
    out = torch.empty((q.shape[0], H, d), dtype=torch.bfloat16, device=DEV)
    gp.pool.prefill_step([1, 2, 3, 4], cu, dev_bf16(q), dev_bf16(k), dev_bf16(v), out, H, Hkv, d, d, scale)
    gp.ctx.phase_sync(PRE)
    want = OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale)
    assert_parity(host_f64(out), want, f"prefill drifting scores rise={rise}")
    gp.close()


@pytest.mark.parametrize("H,Hkv,d", [(16, 2, 128), (8, 1, 64), (32, 2, 128), (6, 2, 128), (12, 2, 64), (5, 1, 128)])
def test_prefill_head_groupings(H, Hkv, d):
    """Every way the 8 waves of a workgroup are split over query heads and row sub-tiles: group sizes
    8 and 16 (8 heads per workgroup), 6 (2 heads), 3 and 5 (1 head: 256 rows per workgroup)."""
    layer = W.LayerShape("gqa", H, Hkv, d, d, 16)
    lens = (70, 129, 1, 300, 257, 513)
    gp = GpuPool(layer, 128, poison=True)
    (q, k, v, cu, scale), out, ids = run_prefill(gp, lens, seed=31 + H + d)
    want = OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale)
    got = host_f64(out)
    for r in range(len(lens)):
        assert_parity(got[cu[r]:cu[r + 1]], want[cu[r]:cu[r + 1]], f"prefill H={H} Hkv={Hkv} d={d} len={lens[r]}")
    gp.close()


def test_decode_equals_last_prefill_row_on_gpu():
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    gp = GpuPool(layer, 64)
    lens = (77, 200)
    (q, k, v, cu, scale), out, ids = run_prefill(gp, lens, seed=31)
    qlast = np.stack([q[cu[1] - 1], q[cu[2] - 1]])
    od = torch.empty((2, 8, 128), dtype=torch.bfloat16, device=DEV)
    gp.ctx.phase_wait_for(DEC, PRE)
    gp.pool.decode_step(ids, lens, dev_bf16(qlast), od, 8, scale)      # reads the pages the prefill step wrote
    gp.ctx.phase_sync(DEC)
    want = np.stack([OA.decode_attention(f64(qlast[i]), f64(k[cu[i]:cu[i + 1]]), f64(v[cu[i]:cu[i + 1]]), scale) for i in range(2)])
    assert_parity(host_f64(od), want, "decode over prefilled pages")
    last_rows = host_f64(out)[[cu[1] - 1, cu[2] - 1]]
    assert np.abs(last_rows - host_f64(od)).max() <= 2e-2
    gp.close()


def test_decode_append_grows_tables_like_the_oracle():
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    gp = GpuPool(layer, 32, poison=True)
    ora = BlockAllocator(32, 16)
    scale = 1.0 / math.sqrt(128)
    start = (14, 31)
    q0, ks, vs, ids = fill_decode_contexts(gp, start, seed=41)
    for r, n in zip(ids, start):
        ora.reserve(r, n)
    rng = np.random.default_rng(42)
    ks, vs = [x.copy() for x in ks], [x.copy() for x in vs]
    lens = list(start)
    for step in range(4):                       # crosses a page border for both requests
        lens = [n + 1 for n in lens]
        knew, vnew, qn = (W.normal_bf16(rng, (2, 2, 128)), W.normal_bf16(rng, (2, 2, 128)), W.normal_bf16(rng, (2, 8, 128)))
        out = torch.empty((2, 8, 128), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, lens, dev_bf16(qn), out, 8, scale, k_new=dev_bf16(knew), v_new=dev_bf16(vnew))
        gp.ctx.phase_sync(DEC)
        for i in range(2):
            ks[i] = np.concatenate([ks[i], knew[i][None]])
            vs[i] = np.concatenate([vs[i], vnew[i][None]])
            ora.reserve(ids[i], lens[i])
            assert gp.pool.kv_block_table(ids[i]) == ora.block_table(ids[i])
        assert_parity(host_f64(out), oracle_decode(qn, ks, vs, scale), f"append step {step}")
    assert gp.pool.kv_free_list() == ora.free_stack and gp.pool.stats()[3] == ora.op_seq
    gp.close()


def test_pool_exhaustion_in_steps_changes_nothing():
    layer = W.LayerShape("gqa", 2, 2, 64, 64, 16)
    gp = GpuPool(layer, 4)
    q, k, v, cu = W.prefill_inputs(layer, (40, 40), seed=51)       # needs 3 + 3 pages, pool has 4
    out = torch.empty((80, 2, 64), dtype=torch.bfloat16, device=DEV)
    before = (gp.pool.kv_free_list(), gp.pool.stats())
    with pytest.raises(S.PoolExhausted):
        gp.pool.prefill_step([1, 2], cu, dev_bf16(q), dev_bf16(k), dev_bf16(v), out, 2, 2, 64, 64, 0.125)
    assert (gp.pool.kv_free_list(), gp.pool.stats()) == before
    with pytest.raises(S.SpdError) as e:
        gp.pool.decode_step([77], [5], dev_bf16(q[:1]), out, 2, 0.125)      # unknown request, attend-only
    assert e.value.status == S.SPD_ENOENT
    gp.close()


# ----------------------------------------------------------------------------- partition
def test_masked_streams_stay_on_their_cus():
    ctx = S.Context(0)
    total, xcds, gran = ctx.device_info()
    full = set(ctx.phase_probe_cus(PRE, 8192))
    assert len(full) == total, f"unmasked launch reached {len(full)} distinct CUs, device has {total}"
    ctx.set_partition(total // 4, 3 * total // 4)
    p_ids = set(ctx.phase_probe_cus(PRE, 8192))
    d_ids = set(ctx.phase_probe_cus(DEC, 8192))
    assert ctx.get_partition() == (total // 4, 3 * total // 4, total // 4, 3 * total // 4)
    assert len(p_ids) == total // 4 and len(d_ids) == 3 * total // 4, (len(p_ids), len(d_ids))
    assert not (p_ids & d_ids), "the two phases share a compute unit"
    for ids in (p_ids, d_ids):                                  # every XCD contributes equally
        per_xcd = [sum(1 for i in ids if i >> 16 == x) for x in range(xcds)]
        assert len(set(per_xcd)) == 1, per_xcd
    ctx.set_partition(total, total)                             # oversubscribed: both may use everything
    assert len(set(ctx.phase_probe_cus(PRE, 8192))) == total
    ctx.close()


# ----------------------------------------------------------------------------- config 2 at full size
def test_partition_sizes_are_whole_rows_of_shader_arrays():
    """On the device, shares are rounded to one compute unit per shader array and XCD (32 CUs): what is beyond
    such a row adds no throughput, the dispatcher deals workgroups to the shader arrays in turn."""
    ctx = S.Context(0)
    total, xcds, gran = ctx.device_info()
    assert gran == 4 * xcds and total % gran == 0
    ctx.set_partition(80, 176)
    pa, da, pp, dp = ctx.get_partition()
    assert (pp, dp) == (96, 160) and pp % gran == 0 and dp % gran == 0
    ctx.set_partition(1, total)
    assert ctx.get_partition()[2:] == (gran, total)
    ctx.close()


def test_c2_full_size_sampled_against_oracle():
    cfg = W.get_config("c2")
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    num_pages = 40960                               # 2.5 GiB of the 40 GB pool is enough to hold the batch
    gp = GpuPool(L, num_pages)
    total, _, _ = gp.ctx.device_info()
    gp.ctx.set_partition(total // 2, total // 2)
    for op, r, n in W.scramble_ops(30000, 16, seed=cfg.seed):
        gp.pool.kv_reserve(r, n) if op == "reserve" else gp.pool.kv_free(r)
    qd, ks, vs, dids = fill_decode_contexts(gp, cfg.decode_ctx, cfg.seed + 1)
    q, k, v, cu = W.prefill_inputs(L, cfg.prefill_lens, cfg.seed)
    tq, tk, tv, tqd = dev_bf16(q), dev_bf16(k), dev_bf16(v), dev_bf16(qd)
    op = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    od = torch.empty((len(dids), L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    gp.pool.prefill_step([1, 2, 3, 4], cu, tq, tk, tv, op, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale)
    gp.pool.decode_step(dids, cfg.decode_ctx, tqd, od, L.n_q_heads, scale)
    gp.ctx.phase_sync(PRE)
    gp.ctx.phase_sync(DEC)
    assert_parity(host_f64(od), oracle_decode(qd, ks, vs, scale), "c2 decode (all 64 requests)")
    got = host_f64(op)
    rng = np.random.default_rng(5)
    qf, kf, vf = f64(q), f64(k), f64(v)
    for r, h in [(0, 0), (1, 13), (2, 31), (3, 7), (int(rng.integers(4)), int(rng.integers(32)))]:
        a, b = cu[r], cu[r + 1]
        g = h // (L.n_q_heads // L.n_kv_heads)
        want = OA.causal_attention(qf[a:b, h:h + 1], kf[a:b, g:g + 1], vf[a:b, g:g + 1], scale)
        assert_parity(got[a:b, h:h + 1], want, f"c2 prefill request {r} head {h}")
    gp.close()


def test_c3_full_size_sampled_against_oracle():
    """Llama-3-70B layer shape (64 query heads over 8 KV heads: 8 heads per prefill workgroup) at the
    bench's sizes: 8 x 4096 prefill tokens (sampled against the oracle), 128 decode requests (all checked)."""
    cfg = W.get_config("c3")
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    gp = GpuPool(L, 40960)
    total, _, _ = gp.ctx.device_info()
    gp.ctx.set_partition(total // 2, total // 2)
    for op, r, n in W.scramble_ops(30000, 16, seed=cfg.seed):
        gp.pool.kv_reserve(r, n) if op == "reserve" else gp.pool.kv_free(r)
    qd, ks, vs, dids = fill_decode_contexts(gp, cfg.decode_ctx, cfg.seed + 1)
    q, k, v, cu = W.prefill_inputs(L, cfg.prefill_lens, cfg.seed)
    tq, tk, tv, tqd = dev_bf16(q), dev_bf16(k), dev_bf16(v), dev_bf16(qd)
    op = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    od = torch.empty((len(dids), L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    gp.pool.prefill_step(list(range(1, len(cfg.prefill_lens) + 1)), cu, tq, tk, tv, op, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale)
    gp.pool.decode_step(dids, cfg.decode_ctx, tqd, od, L.n_q_heads, scale)
    gp.ctx.phase_sync(PRE)
    gp.ctx.phase_sync(DEC)
    assert_parity(host_f64(od), oracle_decode(qd, ks, vs, scale), "c3 decode (all 128 requests)")
    G = L.n_q_heads // L.n_kv_heads
    for r, h in [(0, 0), (3, 29), (7, 63)]:
        a, b = cu[r], cu[r + 1]
        g = h // G
        want = OA.causal_attention(f64(q[a:b, h:h + 1]), f64(k[a:b, g:g + 1]), f64(v[a:b, g:g + 1]), scale)
        assert_parity(host_f64(op[a:b, h:h + 1]), want, f"c3 prefill request {r} head {h}")
    gp.close()


def test_decode_worker_thread_runs_beside_prefill_steps():
    """The library's decode worker (a host thread of its own) keeps issuing decode steps while this
    thread drives prefill steps on the other partition; outputs stay the oracle's."""
    cfg = W.get_config("c1")
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    gp = GpuPool(L, cfg.num_pages)
    total, _, _ = gp.ctx.device_info()
    gp.ctx.set_partition(total // 2, total // 2)
    qd, ks, vs, dids = fill_decode_contexts(gp, cfg.decode_ctx, cfg.seed + 1)
    od = [torch.zeros((len(dids), L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV) for _ in range(2)]
    tqd = dev_bf16(qd)
    batches = [gp.pool.make_decode_batch(dids, cfg.decode_ctx, tqd, o, L.n_q_heads, scale) for o in od]
    q, k, v, cu = W.prefill_inputs(L, cfg.prefill_lens, cfg.seed)
    tq, tk, tv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    op = torch.empty((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    pids = list(range(1, len(cfg.prefill_lens) + 1))
    worker = gp.pool.decode_worker_start(batches)
    t_end = time.monotonic() + 0.2              # long enough for the worker thread to get several steps in
    n_prefill = 0
    while n_prefill < 20 or time.monotonic() < t_end:
        gp.pool.prefill_step(pids, cu, tq, tk, tv, op, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale)
        n_prefill += 1
    gp.ctx.phase_sync(PRE)
    steps = gp.pool.decode_worker_stop(worker)
    gp.ctx.phase_sync(DEC)
    assert steps >= 2
    want = oracle_decode(qd, ks, vs, scale)
    for o in od:
        assert_parity(host_f64(o), want, "decode worker output")
    assert_parity(host_f64(op), OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale), "prefill beside the decode worker")
    # a failing step ends the worker and is reported
    bad = gp.pool.make_decode_batch([987654], [5], tqd, od[0], L.n_q_heads, scale)
    worker = gp.pool.decode_worker_start([bad])
    with pytest.raises(S.SpdError) as e:
        gp.pool.decode_worker_stop(worker)
    assert e.value.status == S.SPD_ENOENT
    gp.close()


def test_long_context_decode_and_long_prompt_prefill():
    """The largest sizes the workloads name: a 131 072-token context (Llama-3.1's limit) decoded with
    split-K over ~8000 pages, and a 32 768-token prompt prefilled; sampled against the oracle."""
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    scale = 1.0 / math.sqrt(128)
    n = 131072
    gp = GpuPool(layer, n // 16 + 2048 + 64)
    rng = np.random.default_rng(77)
    k = W.normal_bf16(rng, (n, 2, 128))
    v = W.normal_bf16(rng, (n, 2, 128))
    qd = W.normal_bf16(rng, (2, 8, 128))
    gp.pool.kv_reserve(1, n)
    gp.pool.kv_reserve(2, 1)                       # a one-token context beside the long one
    for a in range(0, n, 32768):                   # written in four pieces
        gp.pool.kv_write(DEC, 1, a, 32768, dev_bf16(k[a:a + 32768]), dev_bf16(v[a:a + 32768]))
    gp.pool.kv_write(DEC, 2, 0, 1, dev_bf16(k[:1]), dev_bf16(v[:1]))
    od = torch.empty((2, 8, 128), dtype=torch.bfloat16, device=DEV)
    gp.pool.decode_step([1, 2], [n, 1], dev_bf16(qd), od, 8, scale)
    gp.ctx.phase_sync(DEC)
    want = np.stack([OA.decode_attention(f64(qd[0]), f64(k), f64(v), scale), OA.decode_attention(f64(qd[1]), f64(k[:1]), f64(v[:1]), scale)])
    assert_parity(host_f64(od), want, "decode over 131072 tokens")
    gp.pool.kv_free(1)
    # 32768-token prompt: rows sampled through the decode oracle (row i attends to rows 0..i)
    L = 32768
    q = W.normal_bf16(rng, (L, 8, 128))
    out = torch.empty((L, 8, 128), dtype=torch.bfloat16, device=DEV)
    gp.pool.prefill_step([3], [0, L], dev_bf16(q), dev_bf16(k[:L]), dev_bf16(v[:L]), out, 8, 2, 128, 128, scale)
    gp.ctx.phase_sync(PRE)
    got = host_f64(out)
    for i in (0, 63, 64, 4095, 16384, 32767):
        want_i = OA.decode_attention(f64(q[i]), f64(k[:i + 1]), f64(v[:i + 1]), scale)
        assert_parity(got[i], want_i, f"prefill row {i} of 32768")
    gp.close()
