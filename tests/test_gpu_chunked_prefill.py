"""GPU parity of chunked prefill: a prompt processed piece by piece, each piece attending to the
pages written by the pieces before it, against the fp64 oracle (chunk_attention, which is pinned
to the rows of whole-prompt causal attention)."""
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


def run_chunks(gp, q, k, v, cu, cuts_per_req, ids, scale):
    """Feed each request's rows in the pieces given by its cut list; all requests advance together,
    a request that has run out of pieces simply drops out of the later steps.  Returns the outputs
    [T, H, dv] assembled from the steps."""
    L = gp.layer
    out_all = torch.zeros((q.shape[0], L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
    n_steps = max(len(c) - 1 for c in cuts_per_req)
    for s in range(n_steps):
        rows, step_ids, pre, lens = [], [], [], []
        for r, cuts in enumerate(cuts_per_req):
            if s + 1 < len(cuts):
                a, b = cu[r] + cuts[s], cu[r] + cuts[s + 1]
                rows.append(np.arange(a, b))
                step_ids.append(ids[r])
                pre.append(cuts[s])
                lens.append(b - a)
        idx = np.concatenate(rows)
        step_cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        out = torch.empty((len(idx), L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=DEV)
        gp.pool.prefill_step(step_ids, step_cu, dev_bf16(q[idx]), dev_bf16(k[idx]), dev_bf16(v[idx]), out, L.n_q_heads,
                             L.n_kv_heads, L.dim_qk, L.dim_v, scale, prefix_lens=pre)
        gp.ctx.phase_sync(PRE)
        out_all[torch.from_numpy(idx).to(DEV)] = out
    return out_all


@pytest.mark.parametrize("H,Hkv,d", [(8, 2, 128), (16, 2, 128), (3, 3, 64)])
def test_chunked_prefill_matches_oracle_and_pages(H, Hkv, d):
    layer = W.LayerShape("gqa", H, Hkv, d, d, 16)
    lens = (300, 77, 513, 16)
    # cut points inside each request: pieces that end mid-tile, mid-page, of one token, and one request in a single piece
    cuts = [[0, 64, 65, 130, 300], [0, 5, 77], [0, 100, 101, 357, 513], [0, 16]]
    gp = GpuPool(layer, 128, poison=True)
    ora = BlockAllocator(128, 16)
    for op, r, n in W.scramble_ops(60, 16, seed=7):
        (gp.pool.kv_reserve(r, n), ora.reserve(r, n)) if op == "reserve" else (gp.pool.kv_free(r), ora.free(r))
    q, k, v, cu = W.prefill_inputs(layer, lens, seed=51 + H)
    scale = 1.0 / math.sqrt(d)
    ids = [11, 12, 13, 14]
    out = run_chunks(gp, q, k, v, cu, cuts, ids, scale)
    got = host_f64(out)
    for r in range(len(lens)):
        for a, b in zip(cuts[r][:-1], cuts[r][1:]):
            want = OA.chunk_attention(f64(q[cu[r] + a:cu[r] + b]), f64(k[cu[r]:cu[r] + b]), f64(v[cu[r]:cu[r] + b]), scale)
            assert_parity(got[cu[r] + a:cu[r] + b], want, f"request {r} piece [{a},{b})")
    # the pages hold the whole prompt, bit for bit, and the tables grew like the oracle's
    for step in range(max(len(c) - 1 for c in cuts)):          # same order as the steps took them
        for r, rid in enumerate(ids):
            if step + 1 < len(cuts[r]):
                ora.reserve(rid, cuts[r][step + 1])
    for r, rid in enumerate(ids):
        assert gp.pool.kv_block_table(rid) == ora.block_table(rid)
        kb = torch.empty((lens[r], Hkv, d), dtype=torch.bfloat16, device=DEV)
        vb = torch.empty((lens[r], Hkv, d), dtype=torch.bfloat16, device=DEV)
        gp.pool.kv_gather(PRE, rid, lens[r], kb, vb)
        gp.ctx.phase_sync(PRE)
        np.testing.assert_array_equal(host_bits(kb), k[cu[r]:cu[r + 1]])
        np.testing.assert_array_equal(host_bits(vb), v[cu[r]:cu[r + 1]])
    # and a decode step over them sees the same context
    qd, _, _ = W.decode_inputs(layer, (1,) * len(lens), seed=99)
    od = torch.empty((len(lens), H, d), dtype=torch.bfloat16, device=DEV)
    gp.ctx.phase_wait_for(DEC, PRE)
    gp.pool.decode_step(ids, lens, dev_bf16(qd), od, H, scale)
    gp.ctx.phase_sync(DEC)
    want_d = np.stack([OA.decode_attention(f64(qd[r]), f64(k[cu[r]:cu[r + 1]]), f64(v[cu[r]:cu[r + 1]]), scale) for r in range(len(lens))])
    assert_parity(host_f64(od), want_d, "decode after chunked prefill")
    gp.close()


def test_chunked_prefill_long_prefix_and_argument_checks():
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    gp = GpuPool(layer, 400, poison=True)
    n = 4096 + 37
    q, k, v, cu = W.prefill_inputs(layer, (n,), seed=77)
    scale = 1.0 / math.sqrt(128)
    out = run_chunks(gp, q, k, v, cu, [[0, 4000, n]], [5], scale)
    a = 4000
    want = OA.chunk_attention(f64(q[a:n]), f64(k[:n]), f64(v[:n]), scale)
    assert_parity(host_f64(out)[a:n], want, "piece of 133 rows after a prefix of 4000")
    # a prefix that is not there
    one = dev_bf16(q[:8])
    kk, vv = dev_bf16(k[:8]), dev_bf16(v[:8])
    o = torch.empty((8, 8, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(S.SpdError) as e:
        gp.pool.prefill_step([99], [0, 8], one, kk, vv, o, 8, 2, 128, 128, scale, prefix_lens=[32])
    assert e.value.status == S.SPD_ENOENT
    gp.pool.kv_reserve(98, 16)
    with pytest.raises(S.SpdError) as e:
        gp.pool.prefill_step([98], [0, 8], one, kk, vv, o, 8, 2, 128, 128, scale, prefix_lens=[32])
    assert e.value.status == S.SPD_EINVAL
    with pytest.raises(S.SpdError):
        gp.pool.prefill_step([98], [0, 8], one, kk, vv, o, 8, 2, 128, 128, scale, prefix_lens=[-1])
    # exhaustion changes nothing: 400 pages cannot take another 4096-token piece
    free_before = gp.pool.kv_free_list()
    big = dev_bf16(q[:4096])
    ob = torch.empty((4096, 8, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(S.PoolExhausted):
        gp.pool.prefill_step([5], [0, 4096], big, dev_bf16(k[:4096]), dev_bf16(v[:4096]), ob, 8, 2, 128, 128, scale, prefix_lens=[n])
    assert gp.pool.kv_free_list() == free_before
    gp.close()


def test_workspace_grows_between_steps_in_flight():
    """Two chunked steps issued back to back without a wait between them, the second with a context that
    no longer fits the gather workspace of the first (16 MiB to start with): the first step still reads the
    old workspace when the second takes a new one, and both come out right."""
    layer = W.LayerShape("gqa", 8, 2, 64, 64, 16)              # 512 bytes of K and V per cached row
    small, big = 600, 33000                                     # 0.3 MiB, then 16.9 MiB of gathered context
    gp = GpuPool(layer, (small + big) // 16 + 8, poison=True)
    scale = 1.0 / math.sqrt(64)
    qs, ks, vs, _ = W.prefill_inputs(layer, (small,), seed=311)
    qb, kb, vb, _ = W.prefill_inputs(layer, (big,), seed=312)
    cut_s, cut_b = small - 40, big - 24
    # the prefixes, each in one un-chunked step (no workspace), then drained
    for rid, (q, k, v, cut) in ((1, (qs, ks, vs, cut_s)), (2, (qb, kb, vb, cut_b))):
        o = torch.empty((cut, 8, 64), dtype=torch.bfloat16, device=DEV)
        gp.pool.prefill_step([rid], [0, cut], dev_bf16(q[:cut]), dev_bf16(k[:cut]), dev_bf16(v[:cut]), o, 8, 2, 64, 64, scale)
    gp.ctx.phase_sync(PRE)
    out_s = torch.empty((small - cut_s, 8, 64), dtype=torch.bfloat16, device=DEV)
    out_b = torch.empty((big - cut_b, 8, 64), dtype=torch.bfloat16, device=DEV)
    args_s = [dev_bf16(x[cut_s:]) for x in (qs, ks, vs)]
    args_b = [dev_bf16(x[cut_b:]) for x in (qb, kb, vb)]
    gp.pool.prefill_step([1], [0, small - cut_s], *args_s, out_s, 8, 2, 64, 64, scale, prefix_lens=[cut_s])
    gp.pool.prefill_step([2], [0, big - cut_b], *args_b, out_b, 8, 2, 64, 64, scale, prefix_lens=[cut_b])
    gp.ctx.phase_sync(PRE)
    want_s = OA.chunk_attention(f64(qs[cut_s:]), f64(ks), f64(vs), scale)
    want_b = OA.chunk_attention(f64(qb[cut_b:]), f64(kb), f64(vb), scale)
    assert_parity(host_f64(out_s), want_s, "step that read the workspace before it grew")
    assert_parity(host_f64(out_b), want_b, "step that made it grow")
    gp.close()
