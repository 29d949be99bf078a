"""GPU tests of two state rules of the library: a request's pages cannot be freed while a step that was given
the request may still be running (they would be handed out again and overwritten under the reader), and a step
that fails leaves a staged partition staged."""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as OA
from paper_2504_19867_amd import semipd as S
from gpu_util import DEV, GpuPool, assert_parity, dev_bf16, f64, host_f64

pytestmark = pytest.mark.gpu
PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE


def test_free_is_refused_while_a_step_may_still_read_the_pages():
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    scale = 1.0 / math.sqrt(128)
    gp = GpuPool(layer, 4096, poison=True)
    # request 5: a cached context for the decode phase
    n = 300
    qd, ks, vs = W.decode_inputs(layer, (n,), seed=81)
    gp.pool.kv_reserve(5, n)
    gp.pool.kv_write(DEC, 5, 0, n, dev_bf16(ks[0]), dev_bf16(vs[0]))
    gp.ctx.phase_sync(DEC)
    gp.pool.kv_free(5)                                   # its write has finished: freed at once ...
    gp.pool.kv_reserve(5, n)                             # ... and the same pages come back
    gp.pool.kv_write(DEC, 5, 0, n, dev_bf16(ks[0]), dev_bf16(vs[0]))
    gp.ctx.phase_sync(DEC)
    table5 = gp.pool.kv_block_table(5)

    # a prefill step that keeps its partition busy for milliseconds, and a decode step queued behind it
    L = 32768
    rng = np.random.default_rng(82)
    q = dev_bf16(W.normal_bf16(rng, (L, 8, 128)))
    k = dev_bf16(W.normal_bf16(rng, (L, 2, 128)))
    v = dev_bf16(W.normal_bf16(rng, (L, 2, 128)))
    out = torch.empty((L, 8, 128), dtype=torch.bfloat16, device=DEV)
    od = torch.empty((1, 8, 128), dtype=torch.bfloat16, device=DEV)
    tq = dev_bf16(qd)
    torch.cuda.synchronize()
    gp.pool.prefill_step([1], [0, L], q, k, v, out, 8, 2, 128, 128, scale)
    gp.ctx.phase_wait_for(DEC, PRE)
    gp.pool.decode_step([5], [n], tq, od, 8, scale)
    before = (gp.pool.kv_free_list(), gp.pool.stats())
    for rid in (5, 1):                                   # both are still being read or written on the GPU
        with pytest.raises(S.SpdError) as e:
            gp.pool.kv_free(rid)
        assert e.value.status == S.SPD_ESTATE, rid
    assert (gp.pool.kv_free_list(), gp.pool.stats()) == before
    assert gp.pool.kv_block_table(5) == table5
    gp.ctx.phase_sync(PRE)
    gp.pool.kv_free(1)                                   # the prefill phase has drained
    assert gp.ctx.phase_query(DEC) in (True, False)
    gp.ctx.phase_sync(DEC)
    assert_parity(host_f64(od), np.stack([OA.decode_attention(f64(qd[0]), f64(ks[0]), f64(vs[0]), scale)]), "decode before the free")
    gp.pool.kv_free(5)
    # the freed pages are handed out again and overwritten: the new owner reads its own data
    q2, ks2, vs2 = W.decode_inputs(layer, (n,), seed=83)
    gp.pool.kv_reserve(6, n)
    assert gp.pool.kv_block_table(6) == table5
    gp.pool.kv_write(DEC, 6, 0, n, dev_bf16(ks2[0]), dev_bf16(vs2[0]))
    gp.pool.decode_step([6], [n], dev_bf16(q2), od, 8, scale)
    gp.ctx.phase_sync(DEC)
    assert_parity(host_f64(od), np.stack([OA.decode_attention(f64(q2[0]), f64(ks2[0]), f64(vs2[0]), scale)]), "decode over re-used pages")
    gp.close()


def test_a_failing_step_leaves_the_staged_partition_staged():
    layer = W.LayerShape("gqa", 2, 2, 64, 64, 16)
    gp = GpuPool(layer, 4)
    total, _, _ = gp.ctx.device_info()
    half = total // 2
    q, k, v, cu = W.prefill_inputs(layer, (40, 40), seed=91)       # needs 3 + 3 pages, the pool has 4
    out = torch.empty((80, 2, 64), dtype=torch.bfloat16, device=DEV)
    tq, tk, tv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    gp.ctx.set_partition(half, half)
    staged = (total, total, half, half)
    assert gp.ctx.get_partition() == staged
    with pytest.raises(S.PoolExhausted):
        gp.pool.prefill_step([1, 2], cu, tq, tk, tv, out, 2, 2, 64, 64, 0.125)
    assert gp.ctx.get_partition() == staged
    with pytest.raises(S.SpdError) as e:
        gp.pool.decode_step([77], [5], tq[:1], out, 2, 0.125)      # unknown request
    assert e.value.status == S.SPD_ENOENT
    assert gp.ctx.get_partition() == staged
    with pytest.raises(S.SpdError) as e:
        gp.pool.kv_write(DEC, 77, 0, 4, tk, tv)
    assert e.value.status == S.SPD_ENOENT
    assert gp.ctx.get_partition() == staged
    # steps that succeed adopt it, each phase at its own step
    gp.pool.prefill_step([1], cu[:2], tq, tk, tv, out, 2, 2, 64, 64, 0.125)
    assert gp.ctx.get_partition() == (half, total, half, half)
    gp.ctx.phase_wait_for(DEC, PRE)
    gp.pool.decode_step([1], [40], tq[:1], out[:1], 2, 0.125)
    assert gp.ctx.get_partition() == (half,) * 4
    gp.ctx.phase_sync(PRE)
    gp.ctx.phase_sync(DEC)
    gp.close()


def test_read_only_yardsticks_take_any_multiple_of_16_bytes():
    """The two streaming-read kernels of the measurement aids: sizes below one load instruction per wave, ragged
    tails and a few MiB all run to completion on either phase; sizes and pointers off the 16-byte grid are refused."""
    ctx = S.Context(0)
    total, _, _ = ctx.device_info()
    ctx.set_partition(total // 2, total // 2)
    buf = torch.zeros((8 << 20) + 64, dtype=torch.uint8, device=DEV)
    for read in (ctx.phase_read, ctx.phase_read_lds):
        for phase in (PRE, DEC):
            for nbytes in (16, 1024, 1040, (1 << 20) + 48, 8 << 20):
                read(phase, buf, nbytes)
            ctx.phase_sync(phase)
        for bad in (0, 8, 1000):
            with pytest.raises(S.SpdError) as e:
                read(DEC, buf, bad)
            assert e.value.status == S.SPD_EINVAL
        with pytest.raises(S.SpdError) as e:
            read(DEC, buf[8:], 1024)
        assert e.value.status == S.SPD_EINVAL
    ctx.close()
