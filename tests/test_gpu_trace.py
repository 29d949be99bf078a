"""Dynamic trace replay (config 5, reduced): allocator churn through the steps, a mid-run CU-split
resize, and the library's allocator state bit-exact against the oracle replaying the same ops."""
import numpy as np
import pytest

import workloads as W
from oracle.allocator import BlockAllocator
from paper_2504_19867_amd import trace_replay

pytestmark = pytest.mark.gpu


def test_reduced_trace_replay_matches_oracle_allocator_and_resizes():
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    tr = W.trace(160, rate_per_s=8.0, seed=77, in_median=96, in_cap=400, out_median=24, out_cap=80)
    num_pages = 700                                        # small enough that the pool runs dry at times
    stats, ops, snapshots, free_list = trace_replay.replay(
        layer, tr.arrival_s, tr.input_len, tr.output_len, num_pages, max_decode_batch=48, max_prefill_tokens=1024,
        time_scale=2000.0, seed=5, log_ops=True)
    assert stats["pool"]["final"][1] == num_pages and stats["pool"]["final"][2] == 0      # everything freed
    assert stats["decode_outputs_finite"]
    assert stats["decode_step_ms"]["n"] >= int(tr.output_len.max())
    # the resize happened, both phases adopted it, and the pool survived it
    total = stats["resize"]["active_cus_after"]
    assert stats["resize"]["at_step"] is not None and total[0] > total[1]
    # oracle replay of the logged operations: same tables at every snapshot, same final free list
    ora = BlockAllocator(num_pages, layer.page_tokens)
    done = 0
    for n_ops, tables in snapshots:
        ora.replay(ops[done:n_ops])
        done = n_ops
        for r, t in tables.items():
            assert ora.block_table(r) == t
    ora.replay(ops[done:])
    assert ora.free_stack == free_list
    assert ora.op_seq == stats["pool"]["final"][3] == len(ops)
    assert not ora.tables


def test_trace_replay_with_slo_aware_adjuster_decisions_match_oracle():
    """The adjusting algorithm drives spd_set_partition inside the replay; the oracle, fed the logged
    observations, must take the same decisions at every iteration (bit-exact integers)."""
    from oracle import controller as OC
    layer = W.LayerShape("gqa", 8, 2, 128, 128, 16)
    tr = W.trace(200, rate_per_s=8.0, seed=78, in_median=96, in_cap=400, out_median=24, out_cap=80)
    cfg = dict(slo_ttft=0.05, slo_tpot=0.2, p_slo=90.0, window_size=20, max_step=2, step_size=10, history=16)
    stats, ops, snapshots, free_list = trace_replay.replay(
        layer, tr.arrival_s, tr.input_len, tr.output_len, 4000, split_before=(30, 70), max_decode_batch=48,
        max_prefill_tokens=1024, time_scale=2000.0, seed=6, log_ops=True, adjuster=cfg)
    assert stats["pool"]["final"][1] == 4000 and stats["pool"]["final"][2] == 0
    assert stats["decode_outputs_finite"]
    a = stats["adjuster"]
    ora = OC.Adjuster(**cfg)
    share = tuple(a["start"])
    steps = moved = 0
    for ev in a["log"]:
        if ev[0] == "ttft":
            ora.observe_ttft(ev[1])
        elif ev[0] == "tpot":
            ora.observe_tpot(ev[1])
        else:
            _, it, x0, y0, x, y = ev
            assert (x0, y0) == share
            assert ora.step(it, x0, y0) == (x, y), f"iteration {it}"
            moved += (x, y) != share
            share = (x, y)
            steps += 1
    assert steps == stats["decode_step_ms"]["n"] and moved == a["adjustments"] and list(share) == a["final_share"]
    # the tight TTFT objective makes the prefill share grow from its small start
    assert a["adjustments"] >= 1 and a["final_share"][0] > a["start"][0]
    for g, w in zip(a["model_a1_lambda_b1_a2_b2"], (*ora.model_ttft, *ora.model_tpot)):
        assert abs(g - w) <= 1e-9 * max(1.0, abs(w))
    # allocator state still replays exactly
    alloc = BlockAllocator(4000, layer.page_tokens)
    alloc.replay(ops)
    assert alloc.free_stack == free_list and not alloc.tables
