"""The allocator in POSIX shared memory (C-ABI spd_shm_*), no GPU: same policy as the in-process one, bit for bit the
oracle's; two worker PROCESSES storming one segment, their logged operations replayed through the oracle in the
order of the operation numbers the library handed out; error behaviour."""
import multiprocessing as mp
import os

import numpy as np
import pytest

from oracle.allocator import BlockAllocator, PoolExhausted
from paper_2504_19867_amd import semipd as S


def _name(tag):
    return f"/spd_test_{os.getpid()}_{tag}"


def test_single_process_matches_the_oracle_bit_for_bit():
    name = _name("one")
    pool = S.ShmPool(name, 96, 16, 40, create=True)
    try:
        ora = BlockAllocator(96, 16)
        rng = np.random.default_rng(5)
        live = {}
        for step in range(4000):
            r = rng.integers(100)
            if not live or r < 30:
                req, n = int(rng.integers(1 << 40)), int(rng.integers(1, 200))
            elif r < 65:
                req = list(live)[int(rng.integers(len(live)))]
                n = live[req] + int(rng.integers(1, 40))
            else:
                req = list(live)[int(rng.integers(len(live)))]
                assert pool.kv_free(req) == ora.free(req)
                del live[req]
                continue
            if req not in live and len(live) >= 40:
                with pytest.raises(S.PoolExhausted):          # the request table is full: nothing changes
                    pool.kv_reserve(req, n)
                continue
            try:
                want = ora.reserve(req, n)
            except PoolExhausted:
                before = (pool.kv_free_list(), pool.stats())
                with pytest.raises(S.PoolExhausted):
                    pool.kv_reserve(req, n)
                assert (pool.kv_free_list(), pool.stats()) == before
                continue
            assert pool.kv_reserve(req, n) == want
            live[req] = max(live.get(req, 0), n)
            if step % 50 == 0:
                assert pool.kv_block_table(req) == ora.block_table(req)
        assert pool.kv_free_list() == ora.free_stack
        for req in live:
            assert pool.kv_block_table(req) == ora.block_table(req)
        assert pool.stats() == (96, ora.n_free, len(live), ora.op_seq)
    finally:
        pool.close()
        pool.unlink()


def _worker(name, who, n_ops, seed, out_q, start):
    """One worker process: opens the segment by name and runs a seeded mix of new requests, growth and frees on its
    own requests, logging every successful operation with the number the library gave it."""
    from paper_2504_19867_amd import semipd as S2
    pool = S2.ShmPool(name)
    rng = np.random.default_rng(seed)
    live = {}
    log = []
    next_id = (who + 1) << 32
    start.wait(timeout=120)                            # both processes have mapped the segment: go
    for _ in range(n_ops):
        r = rng.integers(100)
        try:
            if not live or r < 35:
                n = int(rng.integers(1, 600 if who == 0 else 60))        # prompts are long, decode contexts grow slowly
                log.append((pool.kv_reserve(next_id, n), "reserve", next_id, n))
                live[next_id] = n
                next_id += 1
            elif r < 75:
                req = list(live)[int(rng.integers(len(live)))]
                n = live[req] + int(rng.integers(1, 20))
                log.append((pool.kv_reserve(req, n), "reserve", req, n))
                live[req] = n
            else:
                req = list(live)[int(rng.integers(len(live)))]
                log.append((pool.kv_free(req), "free", req, 0))
                del live[req]
        except S2.PoolExhausted:
            pass
    tables = {req: pool.kv_block_table(req) for req in live}
    pool.close()
    out_q.put((who, log, tables))


def test_two_processes_allocate_atomically_and_replay_matches_the_oracle():
    name = _name("two")
    num_pages, P = 2048, 16
    pool = S.ShmPool(name, num_pages, P, 4096, create=True)
    try:
        ctx = mp.get_context("spawn")                  # fresh interpreters: nothing is inherited but the name
        q = ctx.Queue()
        start = ctx.Barrier(2)
        procs = [ctx.Process(target=_worker, args=(name, who, 6000, 100 + who, q, start)) for who in range(2)]
        for p in procs:
            p.start()
        results = [q.get(timeout=240) for _ in procs]
        for p in procs:
            p.join(timeout=60)
            assert p.exitcode == 0
        log = sorted(op for _, ops, _ in results for op in ops)
        assert len(log) > 6000, "the workers hardly allocated anything"
        assert [op[0] for op in log] == list(range(1, len(log) + 1))      # every operation number handed out exactly once
        # both workers were active in every quarter of the sequence: the processes really interleaved
        by = {who: {op[0] for op in ops} for who, ops, _ in results}
        n = len(log)
        for quarter in range(4):
            lo, hi = quarter * n // 4, (quarter + 1) * n // 4
            assert all(any(lo < s <= hi for s in by[who]) for who in by)
        ora = BlockAllocator(num_pages, P)
        ora.replay([(op, req, n_tok) for _, op, req, n_tok in log])
        assert pool.kv_free_list() == ora.free_stack
        assert pool.stats() == (num_pages, ora.n_free, len(ora.tables), ora.op_seq)
        for _, _, tables in results:                   # what each worker saw at its end is what the replay gives
            for req, t in tables.items():
                assert t == ora.block_table(req) == pool.kv_block_table(req)
        owned = [b for t in ora.tables.values() for b in t]
        assert len(owned) == len(set(owned)) and not set(owned) & set(ora.free_stack)
    finally:
        pool.close()
        pool.unlink()


def test_names_and_errors():
    name = _name("err")
    with pytest.raises(S.SpdError) as e:
        S.ShmPool(name)                                 # nothing to open
    assert e.value.status == S.SPD_ENOENT
    for bad in (dict(num_pages=0, page_tokens=16, max_requests=4), dict(num_pages=8, page_tokens=0, max_requests=4),
                dict(num_pages=8, page_tokens=16, max_requests=0)):
        with pytest.raises(S.SpdError) as e:
            S.ShmPool(name, create=True, **bad)
        assert e.value.status == S.SPD_EINVAL
    with pytest.raises(S.SpdError) as e:
        S.ShmPool("no_slash", 8, 16, 4, create=True)
    assert e.value.status == S.SPD_EINVAL
    pool = S.ShmPool(name, 8, 16, 4, create=True)
    try:
        with pytest.raises(S.SpdError) as e:
            S.ShmPool(name, 8, 16, 4, create=True)      # the name is taken
        assert e.value.status == S.SPD_ESTATE
        other = S.ShmPool(name)                         # a second mapping in the same process sees the same state
        pool.kv_reserve(7, 40)
        assert other.kv_block_table(7) == [0, 1, 2]
        with pytest.raises(S.SpdError) as e:
            other.kv_free(8)
        assert e.value.status == S.SPD_ENOENT
        with pytest.raises(S.SpdError) as e:
            other.kv_reserve(7, 0)
        assert e.value.status == S.SPD_EINVAL
        other.kv_free(7)
        assert pool.stats() == (8, 8, 0, 2)
        other.close()
    finally:
        pool.close()
        pool.unlink()
    with pytest.raises(S.SpdError):
        S.ShmPool(name)                                 # unlinked
