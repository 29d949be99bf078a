"""Pins for the allocator oracle (CPU only).

Pinned by (a) a hand-worked trace of the stated policy, (b) invariants that the
paper's "Unified Memory Manager" requires of any paged pool shared by two
workers (no block owned twice, utilisation = blocks handed out, conservation),
and (c) an exhaustive model check on tiny pools against a set-based model that
knows nothing about the stack order.
"""
import itertools
import os

import numpy as np
import pytest

import workloads as W
from oracle.allocator import BlockAllocator, PoolExhausted

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_policy_trace():
    steps = []
    for line in open(os.path.join(GOLDEN, "allocator_policy_trace.txt")):
        if not line.strip() or line[0] == "#":
            continue
        op, want, nfree = (p.strip() for p in line.split("|"))
        name, req, n = op.split()
        steps.append((name, int(req), int(n), want, int(nfree)))
    return steps


def check_invariants(a: BlockAllocator):
    owned = [b for t in a.tables.values() for b in t]
    assert len(owned) == len(set(owned)), "a physical block is owned twice"
    assert len(a.free_stack) == len(set(a.free_stack)), "free list holds a duplicate"
    assert not set(owned) & set(a.free_stack), "a block is both free and owned"
    assert set(owned) | set(a.free_stack) == set(range(a.num_pages)), "a block leaked"
    assert a.used == len(owned) and a.n_free + a.used == a.num_pages


def test_hand_worked_policy_trace():
    a = BlockAllocator(8, 4)
    seq = 0
    for name, req, n, want, nfree in read_policy_trace():
        before = a.state()
        if want == "ENOMEM":
            with pytest.raises(PoolExhausted):
                a.reserve(req, n)
            assert a.state() == before
        elif want == "ENOENT":
            with pytest.raises(KeyError):
                a.free(req)
            assert a.state() == before
        elif name == "reserve":
            seq += 1
            assert a.reserve(req, n) == seq
            assert a.block_table(req) == [int(x) for x in want.split()]
        else:
            seq += 1
            assert a.free(req) == seq
            assert req not in a.tables
        assert a.n_free == nfree
        check_invariants(a)


def test_first_pops_are_sequential_and_refree_returns_same_table():
    a = BlockAllocator(32, 16)
    a.reserve(1, 16 * 5)
    assert a.block_table(1) == [0, 1, 2, 3, 4]
    a.reserve(2, 1)
    a.free(1)
    a.reserve(3, 16 * 5)
    assert a.block_table(3) == [0, 1, 2, 3, 4]
    a.reserve(2, 17)
    assert a.block_table(2) == [5, 6]


def test_reserve_boundaries():
    a = BlockAllocator(4, 16)
    for n, pages in ((1, 1), (16, 1), (17, 2), (32, 2), (33, 3)):
        a.reserve(9, n)
        assert len(a.block_table(9)) == pages
    a.reserve(9, 5)                       # shrinking request is a no-op, never frees
    assert len(a.block_table(9)) == 3
    with pytest.raises(ValueError):
        a.reserve(9, 0)
    with pytest.raises(PoolExhausted):
        a.reserve(9, 16 * 5)
    assert len(a.block_table(9)) == 3 and a.n_free == 1


def test_invariants_under_random_churn():
    rng = np.random.default_rng(0)
    a = BlockAllocator(97, 16)
    live = {}
    for step in range(4000):
        r = int(rng.integers(0, 40))
        if r in live and rng.random() < 0.3:
            a.free(r)
            del live[r]
        else:
            n = live.get(r, 0) + int(rng.integers(1, 80))
            before = a.state()
            try:
                a.reserve(r, n)
                live[r] = n
            except PoolExhausted:
                assert a.state() == before
        if step % 50 == 0:
            check_invariants(a)
            for r2, n2 in live.items():
                assert len(a.block_table(r2)) == -(-n2 // 16)
    check_invariants(a)


def test_exhaustive_small_pool_against_set_model():
    """All op sequences of length 5 over a 4-page pool, 2 tokens/page, 2 request ids."""
    P, N = 2, 4
    alphabet = [("reserve", r, n) for r in (0, 1) for n in (1, 3, 5, 9)] + [("free", r, 0) for r in (0, 1)]
    for seq in itertools.product(alphabet, repeat=5):
        a = BlockAllocator(N, P)
        model = {}                                  # req -> page count (set model: counts only)
        for op, r, n in seq:
            before = a.state()
            if op == "reserve":
                want_pages = max(-(-n // P), model.get(r, 0))
                grow = want_pages - model.get(r, 0)
                if grow > N - sum(model.values()):
                    with pytest.raises(PoolExhausted):
                        a.reserve(r, n)
                    assert a.state() == before
                else:
                    a.reserve(r, n)
                    model[r] = want_pages
            else:
                if r in model:
                    a.free(r)
                    del model[r]
                else:
                    with pytest.raises(KeyError):
                        a.free(r)
                    assert a.state() == before
            assert {k: len(t) for k, t in a.tables.items()} == model
        check_invariants(a)


def test_scramble_ops_leave_a_permuted_free_list():
    a = BlockAllocator(64, 16)
    a.replay(W.scramble_ops(48, 16, seed=5))
    check_invariants(a)
    assert a.used == 0 and not a.tables
    a.reserve(1, 16 * 48)
    t = a.block_table(1)
    assert sorted(t) == list(range(48)) and t != list(range(48))
    a2 = BlockAllocator(64, 16)
    a2.replay(W.scramble_ops(48, 16, seed=5))
    a2.reserve(1, 16 * 48)
    assert a2.block_table(1) == t
