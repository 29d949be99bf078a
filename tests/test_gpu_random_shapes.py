"""Seeded random shapes through the whole path (reserve, prefill in pieces, decode with append, free)
against the fp64 oracle: catches indexing mistakes that the hand-picked cases above happen to miss."""
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


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_shape_end_to_end(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 16]))
    H = Hkv * G
    P = int(rng.choice([16, 32, 64, 128]))
    layer = W.LayerShape("gqa", H, Hkv, d, d, P)
    n_req = int(rng.integers(1, 6))
    lens = [int(rng.integers(1, 420)) for _ in range(n_req)]
    num_pages = sum((n + 8 + P - 1) // P for n in lens) + int(rng.integers(0, 6))
    gp = GpuPool(layer, num_pages + 8, poison=True)
    ora = BlockAllocator(num_pages + 8, P)
    # scatter the free list
    for op, r, n in W.scramble_ops(min(6, num_pages), P, seed=seed):
        (gp.pool.kv_reserve(r, n), ora.reserve(r, n)) if op == "reserve" else (gp.pool.kv_free(r), ora.free(r))
    scale = float(rng.uniform(0.05, 0.3))
    q, k, v, cu = W.prefill_inputs(layer, lens, seed=2000 + seed)
    ids = [int(x) for x in rng.choice(10_000, size=n_req, replace=False) + 50_000]
    # every request in one or two pieces
    cuts = [[0, n] if (n < 2 or rng.random() < 0.4) else [0, int(rng.integers(1, n)), n] for n in lens]
    out = torch.zeros((q.shape[0], H, d), dtype=torch.bfloat16, device=DEV)
    for step in range(2):
        rows, sid, pre, ln = [], [], [], []
        for r, c in enumerate(cuts):
            if step + 1 < len(c):
                rows.append(np.arange(cu[r] + c[step], cu[r] + c[step + 1]))
                sid.append(ids[r]); pre.append(c[step]); ln.append(c[step + 1] - c[step])
                ora.reserve(ids[r], c[step + 1])
        if not rows:
            continue
        idx = np.concatenate(rows)
        o = torch.empty((len(idx), H, d), dtype=torch.bfloat16, device=DEV)
        gp.pool.prefill_step(sid, np.concatenate([[0], np.cumsum(ln)]), dev_bf16(q[idx]), dev_bf16(k[idx]), dev_bf16(v[idx]), o,
                             H, Hkv, d, d, scale, prefix_lens=pre if step else None)
        gp.ctx.phase_sync(PRE)
        out[torch.from_numpy(idx).to(DEV)] = o
    want = OA.prefill_attention(f64(q), f64(k), f64(v), cu, scale)
    assert_parity(host_f64(out), want, f"prefill seed {seed}: H={H} Hkv={Hkv} d={d} P={P} lens={lens} cuts={cuts}")
    for r, rid in enumerate(ids):
        assert gp.pool.kv_block_table(rid) == ora.block_table(rid)
    # three decode steps with append
    ks = [k[cu[r]:cu[r + 1]].copy() for r in range(n_req)]
    vs = [v[cu[r]:cu[r + 1]].copy() for r in range(n_req)]
    gp.ctx.phase_wait_for(DEC, PRE)
    cur = list(lens)
    for t in range(3):
        cur = [n + 1 for n in cur]
        kn, vn = W.normal_bf16(rng, (n_req, Hkv, d)), W.normal_bf16(rng, (n_req, Hkv, d))
        qn = W.normal_bf16(rng, (n_req, H, d))
        od = torch.empty((n_req, H, d), dtype=torch.bfloat16, device=DEV)
        gp.pool.decode_step(ids, cur, dev_bf16(qn), od, H, scale, k_new=dev_bf16(kn), v_new=dev_bf16(vn))
        gp.ctx.phase_sync(DEC)
        for r in range(n_req):
            ks[r] = np.concatenate([ks[r], kn[r][None]])
            vs[r] = np.concatenate([vs[r], vn[r][None]])
            ora.reserve(ids[r], cur[r])
        want_d = np.stack([OA.decode_attention(f64(qn[r]), f64(ks[r]), f64(vs[r]), scale) for r in range(n_req)])
        assert_parity(host_f64(od), want_d, f"decode step {t} seed {seed}")
    for r, rid in enumerate(ids):
        assert gp.pool.kv_block_table(rid) == ora.block_table(rid)
        gp.pool.kv_free(rid)
        ora.free(rid)
    assert gp.pool.kv_free_list() == ora.free_stack
    gp.close()
