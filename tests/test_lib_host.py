"""Host logic of libsemipd through the C ABI, no GPU: exports, allocator == oracle bit for bit,
the two-worker atomicity scenario, partition masks, error behaviour."""
import os
import re
import threading

import numpy as np
import pytest

import workloads as W
from oracle.allocator import BlockAllocator, PoolExhausted
from paper_2504_19867_amd import semipd as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def host_pool(num_pages=64, P=16, kind=S.SPD_KV_GQA, hkv=2, dk=64, dv=64):
    ctx = S.Context(-1)
    return ctx, S.Pool(ctx, None, 0, kind, P, hkv, dk, dv, num_pages)


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "semipd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(spd_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(S.EXPORTS)
    for name in declared:
        assert hasattr(S.lib, name), f"{name} declared in semipd.h but not exported"


def test_policy_trace_matches_golden_fixture():
    ctx, pool = host_pool(8, 4 * 4)        # the fixture uses 4 tokens / page; the library needs P % 16 == 0
    scale = 4                              # so token counts are multiplied by 4 (same page counts)
    for line in open(os.path.join(GOLDEN, "allocator_policy_trace.txt")):
        if not line.strip() or line[0] == "#":
            continue
        op, want, nfree = (p.strip() for p in line.split("|"))
        name, req, n = op.split()
        req, n = int(req), int(n)
        before = (pool.kv_free_list(), pool.stats())
        if want == "ENOMEM":
            with pytest.raises(S.PoolExhausted):
                pool.kv_reserve(req, (n - 1) * scale + 1)
            assert (pool.kv_free_list(), pool.stats()) == before
        elif want == "ENOENT":
            with pytest.raises(S.SpdError) as e:
                pool.kv_free(req)
            assert e.value.status == S.SPD_ENOENT
            assert (pool.kv_free_list(), pool.stats()) == before
        elif name == "reserve":
            pool.kv_reserve(req, (n - 1) * scale + 1)      # same ceil(n / 4) pages
            assert pool.kv_block_table(req) == [int(x) for x in want.split()]
        else:
            pool.kv_free(req)
        assert pool.stats()[1] == int(nfree)


def test_random_churn_is_bit_exact_with_oracle():
    rng = np.random.default_rng(1)
    ctx, pool = host_pool(97, 16)
    ora = BlockAllocator(97, 16)
    live = {}
    for step in range(3000):
        r = int(rng.integers(0, 30))
        if r in live and rng.random() < 0.3:
            assert pool.kv_free(r) == ora.free(r)
            del live[r]
        else:
            n = live.get(r, 0) + int(rng.integers(1, 90))
            try:
                want = ora.reserve(r, n)
            except PoolExhausted:
                with pytest.raises(S.PoolExhausted):
                    pool.kv_reserve(r, n)
                continue
            assert pool.kv_reserve(r, n) == want
            live[r] = n
        if step % 100 == 0:
            assert pool.kv_free_list() == ora.free_stack
            for r2 in live:
                assert pool.kv_block_table(r2) == ora.block_table(r2)
            total, free, nlive, seq = pool.stats()
            assert (total, free, nlive, seq) == (97, ora.n_free, len(ora.tables), ora.op_seq)
    assert pool.kv_free_list() == ora.free_stack


def test_two_workers_allocate_atomically_and_replay_matches_oracle():
    """The paper's write-after-read hazard: two asynchronous workers query / get / update at once.
    Each call's sequence number gives the linearised order; the oracle replays it and must land
    in exactly the same tables and free list, and no block may ever be owned twice."""
    ctx, pool = host_pool(512, 16)
    logs = [[], []]

    def worker(wid):
        rng = np.random.default_rng(100 + wid)
        mine = {}
        for _ in range(4000):
            r = wid * 1000 + int(rng.integers(0, 20))
            if r in mine and rng.random() < 0.4:
                logs[wid].append((pool.kv_free(r), "free", r, 0))
                del mine[r]
            else:
                n = mine.get(r, 0) + int(rng.integers(1, 200))
                try:
                    logs[wid].append((pool.kv_reserve(r, n), "reserve", r, n))
                    mine[r] = n
                except S.PoolExhausted:
                    pass

    ts = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    ops = sorted(logs[0] + logs[1])
    seqs = [o[0] for o in ops]
    assert seqs == list(range(1, len(ops) + 1)), "sequence numbers are not a gap-free linear order"
    ora = BlockAllocator(512, 16)
    for _, op, r, n in ops:
        ora.reserve(r, n) if op == "reserve" else ora.free(r)
    assert pool.kv_free_list() == ora.free_stack
    owned = []
    for r in ora.tables:
        t = pool.kv_block_table(r)
        assert t == ora.block_table(r)
        owned += t
    assert len(owned) == len(set(owned))
    assert pool.stats() == (512, ora.n_free, len(ora.tables), ora.op_seq)


def test_scramble_ops_same_on_both_sides():
    ctx, pool = host_pool(256, 16)
    ora = BlockAllocator(256, 16)
    for op, r, n in W.scramble_ops(200, 16, seed=3):
        if op == "reserve":
            pool.kv_reserve(r, n), ora.reserve(r, n)
        else:
            pool.kv_free(r), ora.free(r)
    assert pool.kv_free_list() == ora.free_stack
    pool.kv_reserve(1, 16 * 50)
    ora.reserve(1, 16 * 50)
    assert pool.kv_block_table(1) == ora.block_table(1) != list(range(50))


def test_allocator_argument_errors_change_nothing():
    ctx, pool = host_pool(4, 16)
    pool.kv_reserve(1, 20)
    snap = (pool.kv_free_list(), pool.stats(), pool.kv_block_table(1))
    for bad in (0, -5):
        with pytest.raises(S.SpdError) as e:
            pool.kv_reserve(2, bad)
        assert e.value.status == S.SPD_EINVAL
    with pytest.raises(S.PoolExhausted):
        pool.kv_reserve(1, 16 * 5)
    with pytest.raises(S.SpdError) as e:
        pool.kv_block_table(99)
    assert e.value.status == S.SPD_ENOENT
    assert (pool.kv_free_list(), pool.stats(), pool.kv_block_table(1)) == snap


def test_pool_geometry_and_validation():
    c2 = W.get_config("c2").layer
    assert S.pool_bytes(S.SPD_KV_GQA, 16, c2.n_kv_heads, 128, 128, 10) == 10 * c2.page_bytes
    c4 = W.get_config("c4").layer
    assert S.pool_bytes(S.SPD_KV_MLA_LATENT, 64, 1, 576, 512, 3) == 3 * c4.page_bytes
    for bad in ((S.SPD_KV_GQA, 15, 8, 128, 128, 4), (S.SPD_KV_GQA, 16, 8, 96, 96, 4), (S.SPD_KV_GQA, 16, 8, 128, 64, 4),
                (S.SPD_KV_GQA, 16, 8, 128, 128, 0), (S.SPD_KV_MLA_LATENT, 64, 2, 576, 512, 4), (7, 16, 8, 128, 128, 4)):
        with pytest.raises(S.SpdError) as e:
            S.pool_bytes(*bad)
        assert e.value.status == S.SPD_EINVAL


def bits(words):
    return {32 * i + b for i, w in enumerate(words) for b in range(32) if (w >> b) & 1}


def test_fp8_latent_pool_geometry():
    """656 bytes per cached token (512 codes, 4 scales, 64 bf16 rope entries) against 1152 for the bf16 latent pool;
    the same shape rules; the allocator does not care."""
    assert S.pool_bytes(S.SPD_KV_MLA_LATENT_FP8, 64, 1, 576, 512, 10) == 10 * 64 * 656
    assert S.pool_bytes(S.SPD_KV_MLA_LATENT, 64, 1, 576, 512, 10) == 10 * 64 * 1152
    ctx = S.Context(-1)
    for bad in ((48, 1, 576, 512), (64, 2, 576, 512), (64, 1, 512, 512), (64, 1, 576, 128)):
        with pytest.raises(S.SpdError) as e:
            S.Pool(ctx, None, 0, S.SPD_KV_MLA_LATENT_FP8, *bad, 8)
        assert e.value.status == S.SPD_EINVAL
    pool = S.Pool(ctx, None, 0, S.SPD_KV_MLA_LATENT_FP8, 64, 1, 576, 512, 8)
    pool.kv_reserve(1, 130)
    assert pool.kv_block_table(1) == [0, 1, 2]
    with pytest.raises(S.SpdError) as e:                       # RoPE inside the decode step is not offered here
        pool.decode_step([1], [130], 4096, 4096, 16, 1.0, rope=S.rope_config(rotary_dim=64, rotary_offset=512))
    assert e.value.status == S.SPD_EINVAL


@pytest.mark.parametrize("p,d", [(77, 179), (128, 128), (102, 154), (179, 77), (8, 248), (1, 1)])
def test_partition_masks_disjoint_and_balanced(p, d):
    pm, dm, pr, dr = S.partition_masks(256, 8, p, d)
    pb, db = bits(pm), bits(dm)
    assert len(pb) == pr and len(db) == dr and pr % 8 == 0 and dr % 8 == 0
    assert abs(pr - p) <= 7 and abs(dr - d) <= 7
    assert not (pb & db), "partitions overlap although the counts fit"
    assert pb == set(range(pr)) and db == set(range(256 - dr, 256))
    # consecutive mask bits walk the XCDs, so each XCD contributes equally to each share
    for s in (pb, db):
        per_xcd = [sum(1 for b in s if b % 8 == x) for x in range(8)]
        assert len(set(per_xcd)) == 1


def test_partition_rounding_keeps_disjoint_requests_disjoint():
    for p, d in [(80, 176), (112, 144), (16, 240), (240, 16), (250, 6), (1, 255)]:
        pm, dm, pr, dr = S.partition_masks(256, 32, p, d)
        assert pr % 32 == 0 and dr % 32 == 0 and pr >= 32 and dr >= 32 and pr + dr <= 256, (p, d, pr, dr)
        assert not any(a & b for a, b in zip(pm, dm))
    assert S.partition_masks(256, 32, 80, 176)[2:] == (96, 160)
    assert S.partition_masks(256, 32, 200, 200)[2:] == (192, 192)       # asked to overlap: each rounded on its own


def test_partition_masks_oversubscription_overlaps():
    pm, dm, pr, dr = S.partition_masks(256, 8, 256, 256)      # the paper's (100, 100) setting
    assert pr == dr == 256 and bits(pm) == bits(dm) == set(range(256))
    pm, dm, pr, dr = S.partition_masks(256, 8, 160, 160)
    assert len(bits(pm) & bits(dm)) == 64
    for bad in ((0, 8), (8, 0), (-1, 5)):
        with pytest.raises(S.SpdError):
            S.partition_masks(256, 8, *bad)
    with pytest.raises(S.SpdError):
        S.partition_masks(250, 8, 10, 10)


def test_host_only_context_stages_partition_and_refuses_gpu_work():
    ctx, pool = host_pool(16, 16)
    assert ctx.device_info() == (256, 8, 32)
    assert ctx.get_partition() == (256, 256, 256, 256)
    ctx.set_partition(102, 154)
    # delayed switching: staged, not adopted until the phase's next step
    assert ctx.get_partition() == (256, 256, 96, 160)
    assert bits(ctx.phase_cu_mask(S.SPD_PHASE_PREFILL)) == set(range(256))
    pool.kv_reserve(1, 16)
    for fn in (lambda: ctx.phase_sync(0), lambda: ctx.phase_stream(1), lambda: pool.kv_write(0, 1, 0, 4, 4096, 4096),
               lambda: pool.decode_step([1], [4], 4096, 4096, 2, 1.0),
               lambda: pool.prefill_step([2], [0, 8], 4096, 4096, 4096, 4096, 2, 2, 64, 64, 1.0)):
        with pytest.raises(S.SpdError) as e:
            fn()
        assert e.value.status == S.SPD_ESTATE
    assert pool.stats()[2] == 1          # the refused prefill reserved nothing


def test_step_argument_validation():
    ctx, pool = host_pool(16, 16)
    pool.kv_reserve(1, 16)
    cases = [
        lambda: pool.decode_step([1], [0], 4096, 4096, 2, 1.0),                    # empty context
        lambda: pool.decode_step([1], [4], 4096, 4096, 3, 1.0),                    # heads not a multiple of KV heads
        lambda: pool.decode_step([1], [4], 4096, 4096, 64, 1.0),                   # > 16 query heads per KV head
        lambda: pool.decode_step([1], [4], None, 4096, 2, 1.0),
        lambda: pool.prefill_step([2], [0, 0], 4096, 4096, 4096, 4096, 2, 2, 64, 64, 1.0),   # zero-length prompt
        lambda: pool.prefill_step([2, 2], [0, 4, 8], 4096, 4096, 4096, 4096, 2, 2, 64, 64, 1.0),  # duplicate id
        lambda: pool.prefill_step([2], [0, 8], 4096, 4096, 4096, 4096, 2, 2, 128, 128, 1.0),  # dims differ from pool
        lambda: pool.prefill_step([2], [0, 8], 4096, 4096, 4096, 4096, 2, 2, 64, 64, 1.0, latent=4096),
        lambda: pool.decode_step([1], [4], 4096, 4096, 2, 0.0),                    # scale must be > 0
        lambda: pool.prefill_step([2], [0, 8], 4096, 4096, 4096, 4096, 2, 2, 64, 64, -1.0),
        lambda: pool.kv_write(0, 1, 0, 0, 4096, 4096),
        lambda: pool.kv_write(0, 1, 0, 4, 4096, None),
    ]
    for fn in cases:
        with pytest.raises(S.SpdError) as e:
            fn()
        assert e.value.status == S.SPD_EINVAL
    assert pool.stats()[2] == 1


def test_misaligned_device_tensors_are_refused():
    """Every tensor a step is given must start on a 16-byte boundary (the kernels move 16 bytes per lane): a view
    that starts 2, 4 or 8 bytes into one is SPD_EINVAL; the same call with aligned addresses gets as far as
    SPD_ESTATE on a host-only context."""
    ctx, pool = host_pool(16, 16)
    pool.kv_reserve(1, 16)
    A = 4096

    def prefill(q=A, k=A, v=A, out=A):
        pool.prefill_step([2], [0, 8], q, k, v, out, 2, 2, 64, 64, 1.0)

    def decode(q=A, out=A, k_new=None, v_new=None):
        pool.decode_step([1], [4], q, out, 2, 1.0, k_new=k_new, v_new=v_new)

    for off in (2, 4, 8):
        bad = A + off
        cases = [lambda: prefill(q=bad), lambda: prefill(k=bad), lambda: prefill(v=bad), lambda: prefill(out=bad),
                 lambda: decode(q=bad), lambda: decode(out=bad), lambda: decode(k_new=bad, v_new=A),
                 lambda: decode(k_new=A, v_new=bad), lambda: pool.kv_write(0, 1, 0, 4, bad, A),
                 lambda: pool.kv_write(0, 1, 0, 4, A, bad), lambda: pool.kv_gather(0, 1, 4, bad, A),
                 lambda: pool.decode_step_noalloc_batch(pool.make_decode_batch([1], [4], bad, A, 2, 1.0))]
        for i, fn in enumerate(cases):
            with pytest.raises(S.SpdError) as e:
                fn()
            assert e.value.status == S.SPD_EINVAL, (off, i)
    for fn in (prefill, decode, lambda: decode(k_new=A, v_new=A), lambda: pool.kv_write(0, 1, 0, 4, A, A)):
        with pytest.raises(S.SpdError) as e:
            fn()
        assert e.value.status == S.SPD_ESTATE
    assert pool.stats()[2] == 1
    # the MLA side: the latent rows of a prefill step
    ctx2 = S.Context(-1)
    mla = S.Pool(ctx2, None, 0, S.SPD_KV_MLA_LATENT, 64, 1, 576, 512, 8)
    with pytest.raises(S.SpdError) as e:
        mla.prefill_step([1], [0, 8], A, A, A, A, 4, 4, 192, 128, 1.0, latent=A + 8)
    assert e.value.status == S.SPD_EINVAL
    with pytest.raises(S.SpdError) as e:
        mla.prefill_step([1], [0, 8], A, A, A, A, 4, 4, 192, 128, 1.0, latent=A)
    assert e.value.status == S.SPD_ESTATE


def test_free_needs_no_wait_when_no_step_took_the_table():
    """The lifetime rule of spd_kv_free concerns steps in flight on the GPU; a request that no step was ever given
    (all a host-only context can have) is freed at once, and its pages are the next ones handed out."""
    ctx, pool = host_pool(8, 16)
    pool.kv_reserve(1, 40)
    table = pool.kv_block_table(1)
    pool.kv_free(1)
    with pytest.raises(S.SpdError) as e:
        pool.kv_free(1)
    assert e.value.status == S.SPD_ENOENT
    pool.kv_reserve(2, 40)
    assert pool.kv_block_table(2) == table


# ---------------------------------------------------------------- SLO-aware partition adjuster
def _feed(adj, ora, ttfts, tpots):
    for v in ttfts:
        adj.observe_ttft(v)
        ora.observe_ttft(v)
    for v in tpots:
        adj.observe_tpot(v)
        ora.observe_tpot(v)


def test_adjuster_matches_hand_worked_trace_and_oracle():
    import os
    from oracle import controller as OC
    golden = os.path.join(os.path.dirname(__file__), "golden", "controller_trace.txt")
    runs = {}
    for line in open(golden):
        line = line.split("#")[0].split()
        if not line:
            continue
        run, it, x0, y0, ttft, tpot, x, y = line[0], *[float(v) for v in line[1:]]
        if run not in runs:
            runs[run] = (S.Adjuster(100.0, 20.0, 90.0, 1, 4, 10), OC.Adjuster(100.0, 20.0, 90.0, 1, 4, 10))
        adj, ora = runs[run]
        _feed(adj, ora, [ttft * 0.5] * 8 + [ttft, ttft * 3], [tpot * 0.5] * 8 + [tpot, tpot * 3])
        got = adj.step(int(it), int(x0), int(y0))
        assert got == (int(x), int(y)) == ora.step(int(it), int(x0), int(y0)), f"run {run} window {int(it)}"
    for adj, _ in runs.values():
        adj.close()


def test_adjuster_from_the_overlapping_start_takes_every_step():
    """Points are recorded at the raw share and Eq. 4 is evaluated at the normalised one (Algorithm 1 updates with x
    and estimates with x'): from the library's initial (100, 100) the model fitted at share 100 is asked about share
    50 and predicts twice the observed latency, so a phase that misses its objective by 1 % still takes all max_step
    steps; the other share pays, since 100 cannot be passed.  Library and oracle agree on it."""
    from oracle import controller as OC
    for which in ("ttft", "tpot"):
        adj, ora = S.Adjuster(100.0, 20.0, 90.0, 1, 4, 10), OC.Adjuster(100.0, 20.0, 90.0, 1, 4, 10)
        ttft, tpot = (101.0, 10.0) if which == "ttft" else (50.0, 20.2)
        _feed(adj, ora, [ttft] * 10, [tpot] * 10)
        got = adj.step(0, 100, 100)
        assert got == ora.step(0, 100, 100)
        assert got == ((100, 60) if which == "ttft" else (60, 100))
        # the next window, observed at the new partition, gives the fit a second share and the model its slope
        _feed(adj, ora, [ttft * 0.7] * 10, [tpot * 0.7] * 10)
        assert adj.step(1, *got) == ora.step(1, *got) == got


def test_adjuster_decisions_bit_exact_and_model_close_on_random_streams():
    import random
    from oracle import controller as OC
    rnd = random.Random(5)
    moved = 0
    for trial in range(150):
        ss = rnd.choice((5, 10, 20))
        kw = dict(slo_ttft=rnd.uniform(50, 400), slo_tpot=rnd.uniform(5, 60), p_slo=rnd.choice((50.0, 90.0, 99.0)),
                  window_size=rnd.choice((1, 3, 8)), max_step=rnd.choice((1, 2, 4)), step_size=ss, history=rnd.choice((2, 8, 64)))
        adj, ora = S.Adjuster(**kw), OC.Adjuster(**kw)
        x, y = rnd.choice(range(ss, 101, ss)), rnd.choice(range(ss, 101, ss))
        # latencies follow a hidden model of the shares plus noise, as a served system's would
        a1, lam, b1, a2, b2 = rnd.uniform(2e3, 2e4), rnd.uniform(0, 4), rnd.uniform(0, 30), rnd.uniform(200, 3000), rnd.uniform(0, 8)
        for it in range(60):
            n = rnd.randint(0, 5)
            _feed(adj, ora, [max(0.0, a1 / (100.0 * x / (x + y) - lam) + b1 + rnd.gauss(0, 5)) for _ in range(n)],
                  [max(0.0, a2 / (100.0 * y / (x + y)) + b2 + rnd.gauss(0, 1)) for _ in range(n)])
            got, want = adj.step(it, x, y), ora.step(it, x, y)
            assert got == want, f"trial {trial} iter {it}: {got} vs {want}"
            moved += got != (x, y)
            x, y = got
            m = adj.model()
            for g, w in zip(m, (*ora.model_ttft, *ora.model_tpot)):
                assert abs(g - w) <= 1e-9 * max(1.0, abs(w)), (m, ora.model_ttft, ora.model_tpot)
        adj.close()
    assert moved > 100          # the streams do exercise the adjusting branches


def test_adjuster_argument_checks():
    with pytest.raises(S.SpdError):
        S.Adjuster(0.0, 20.0)
    with pytest.raises(S.SpdError):
        S.Adjuster(100.0, 20.0, p_slo=0.0)
    with pytest.raises(S.SpdError):
        S.Adjuster(100.0, 20.0, step_size=60)
    adj = S.Adjuster(100.0, 20.0, step_size=10)
    with pytest.raises(S.SpdError):
        adj.observe_ttft(float("nan"))
    with pytest.raises(S.SpdError):
        adj.step(0, 5, 50)          # below one step
    with pytest.raises(S.SpdError):
        adj.step(-1, 50, 50)
    assert adj.step(0, 50, 50) == (50, 50)      # empty window: unchanged
    assert adj.model() == (0.0, 0.0, 0.0, 0.0, 0.0)
    adj.close()


# ----------------------------------------------------------------------------- rotary embedding (host side)
def test_rope_frequency_table_equals_the_oracle():
    from oracle import rope as R
    cases = [
        (S.rope_config(theta=10000.0, rotary_dim=64), R.RopeConfig(theta=10000.0, rotary_dim=64)),
        (S.rope_config(factor=8.0), R.LLAMA31),
        (S.rope_config(theta=1e6, factor=32.0, low_freq_factor=2.0, high_freq_factor=8.0, original_max_pos=4096, rotary_dim=96),
         R.RopeConfig(theta=1e6, factor=32.0, low_freq_factor=2.0, high_freq_factor=8.0, original_max_pos=4096, rotary_dim=96)),
    ]
    for c, o in cases:
        got, want = np.array(S.rope_inv_freq(c)), R.inv_freq(o)
        np.testing.assert_allclose(got, want, rtol=1e-15, atol=0)


def test_rope_argument_checks():
    import ctypes as C
    bad = [
        S.rope_config(theta=0.0), S.rope_config(factor=0.5), S.rope_config(rotary_dim=0), S.rope_config(rotary_dim=6 + 1),
        S.rope_config(rotary_offset=-8), S.rope_config(factor=8.0, high_freq_factor=1.0), S.rope_config(factor=8.0, original_max_pos=0),
    ]
    buf = (C.c_double * 256)()
    for c in bad:
        assert S.lib.spd_rope_inv_freq(C.byref(c), buf, 256) == S.SPD_EINVAL
    ok = S.rope_config(rotary_dim=64)
    assert S.lib.spd_rope_inv_freq(C.byref(ok), buf, 31) == S.SPD_EINVAL          # room for fewer than 32
    assert S.lib.spd_rope_inv_freq(C.byref(ok), None, 64) == S.SPD_EINVAL
    # the device call: every violated condition is refused before anything is enqueued (a null context too)
    pos = (C.c_int32 * 4)(0, 1, 2, 3)
    assert S.lib.spd_rope_qk(None, 0, C.byref(ok), pos, 4, 16, 2, None, 0, 64) == S.SPD_EINVAL


def test_ffn_argument_checks_on_a_host_only_context():
    ctx, pool = host_pool(16, 16)
    lib = S.lib
    bad = [(31, 128), (64, 100), (0, 128), (64, 0), (64, -128)]
    for hidden, inter in bad:
        assert lib.spd_ffn_gate_up(ctx.h, 0, 4096, 4096, 4096, 4, hidden, inter) == S.SPD_EINVAL
        assert lib.spd_ffn_pack_gate_up(ctx.h, 0, 4096, 4096, 4096, hidden, inter) == S.SPD_EINVAL
    assert lib.spd_ffn_gate_up(ctx.h, 2, 4096, 4096, 4096, 4, 64, 128) == S.SPD_EINVAL          # no such phase
    assert lib.spd_ffn_gate_up(ctx.h, 0, 4096, 4096, 4096, -1, 64, 128) == S.SPD_EINVAL
    assert lib.spd_ffn_gate_up(ctx.h, 0, 4100, 4096, 4096, 4, 64, 128) == S.SPD_EINVAL          # x not 16-byte aligned
    assert lib.spd_ffn_gate_up(ctx.h, 0, None, 4096, 4096, 4, 64, 128) == S.SPD_EINVAL
    # well-formed, but this context has no device
    assert lib.spd_ffn_gate_up(ctx.h, 0, 4096, 4096, 4096, 4, 64, 128) == S.SPD_ESTATE
    assert lib.spd_ffn_pack_gate_up(ctx.h, 1, 4096, 4096, 4096, 64, 128) == S.SPD_ESTATE
