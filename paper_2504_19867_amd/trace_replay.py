"""Dynamic mixed-trace replay over the semi-PD hot path (benchmark configs[4]).

Drives the library the way the paper's two workers do ("Prefill and Decode Workers"): requests
arrive (Poisson), wait FCFS for a prefill batch, are prefilled (K, V written into the unified
pool), join the decode batch (max_batch_size, FCFS), append one token per decode step with block
reservations growing page by page, and free their blocks when they finish.  Midway the CU split is
resized (`spd_set_partition`), and the cost of the switch is measured.

Only one attention layer runs, so a step takes ~1/1000 of a model iteration: the arrival clock is
virtual (wall time x `time_scale`); when nothing is runnable the clock jumps to the next arrival
instead of sleeping, so the GPU is never idled on purpose.

All method arithmetic is in the library's kernels; this module only schedules calls.
"""
from __future__ import annotations

import json
import math
import time
from collections import deque
from typing import Dict, List, Optional, Tuple

from . import semipd as S

PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE


def _pct(xs: List[float], p: float) -> Optional[float]:
    if not xs:
        return None
    s = sorted(xs)
    return s[min(len(s) - 1, int(math.ceil(p / 100.0 * len(s))) - 1)]


def _summary(xs: List[float]) -> Dict[str, Optional[float]]:
    return {"n": len(xs), "p50": _pct(xs, 50), "p90": _pct(xs, 90), "p99": _pct(xs, 99),
            "mean": (sum(xs) / len(xs)) if xs else None}


def replay(layer, arrival_s, input_len, output_len, num_pages: int, *, split_before=(40, 60), split_after=(60, 40),
           resize_after_requests: Optional[int] = None, max_decode_batch: int = 512, max_prefill_tokens: int = 16384,
           time_scale: float = 128.0, seed: int = 0, device: int = 0, log_ops: bool = False,
           adjuster: Optional[dict] = None):
    """Replay a trace; returns (stats dict, allocator op log, table snapshots, final free list).

    The op log lists, in execution order, ("reserve", req, n_tokens) / ("free", req, 0) exactly as
    the library performed them, so an independent allocator can replay it.

    `adjuster` (keyword arguments of semipd.Adjuster, latencies in virtual seconds) replaces the one
    fixed mid-run resize by the SLO-aware adjusting algorithm (paper, "Dynamic Adjusting Method"):
    TTFT = virtual time from arrival to the end of the request's first prefill step, TPOT = virtual
    duration of a decode step, one adjusting iteration per decode step.  stats["adjuster"] then
    holds the partition history and, with log_ops, the exact observation / decision stream.
    """
    import torch

    dev = torch.device(f"cuda:{device}")
    torch.cuda.init()
    n_req = len(arrival_s)
    ctx = S.Context(device)
    total_cus, _, _ = ctx.device_info()
    nbytes = S.pool_bytes(S.SPD_KV_GQA, layer.page_tokens, layer.n_kv_heads, layer.dim_qk, layer.dim_v, num_pages)
    mem = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pool = S.Pool(ctx, mem, nbytes, S.SPD_KV_GQA, layer.page_tokens, layer.n_kv_heads, layer.dim_qk, layer.dim_v, num_pages)
    scale = 1.0 / math.sqrt(layer.dim_qk)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)

    H, Hkv, d, dv = layer.n_q_heads, layer.n_kv_heads, layer.dim_qk, layer.dim_v
    cap_tokens = max(max_prefill_tokens, int(max(input_len)) + int(max(output_len)))
    pq, pk, pv = randn(cap_tokens, H, d), randn(cap_tokens, Hkv, d), randn(cap_tokens, Hkv, dv)
    pout = torch.empty((cap_tokens, H, dv), dtype=torch.bfloat16, device=dev)
    dq, dk, dvn = randn(max_decode_batch, H, d), randn(max_decode_batch, Hkv, d), randn(max_decode_batch, Hkv, dv)
    dout = torch.zeros((max_decode_batch, H, dv), dtype=torch.bfloat16, device=dev)

    def cus(pct):
        return max(1, round(total_cus * pct / 100))

    ctx.set_partition(cus(split_before[0]), cus(split_before[1]))
    ctx.set_kernel_timing(True)
    if resize_after_requests is None:
        resize_after_requests = n_req // 2

    ops: List[Tuple[str, int, int]] = []
    waiting: deque = deque()            # arrived, not yet prefilled
    ready: deque = deque()              # prefilled, waiting for a decode slot
    running: List[int] = []             # in the decode batch
    ctx_len = [0] * n_req
    generated = [0] * n_req
    next_arrival = 0
    finished = 0
    prefill_inflight: Optional[List[int]] = None
    decode_inflight: Optional[List[int]] = None
    pre_ms: List[float] = []
    dec_ms: List[float] = []
    pre_tokens: List[int] = []
    dec_batch: List[int] = []
    resized_at_step = None              # (prefill steps, decode steps) issued before the resize
    resize_call_ms = None
    issued_pre = issued_dec = 0
    snapshots = []                      # (ops so far, {request: block table}) for the allocator cross-check
    peak_used = 0
    exhausted_events = 0
    preemptions = 0
    prompt_len = [int(x) for x in input_len]     # grows when a preempted request is re-prefilled with its output so far
    prefill_cap = 64                             # requests per prefill batch; halved while the pool is short
    adj = S.Adjuster(**adjuster) if adjuster else None
    adj_log: List[tuple] = []
    adj_history: List[tuple] = []                # (decode iteration, x, y, set_partition call ms)
    share = [int(split_before[0]), int(split_before[1])]
    first_prefill_done = [False] * n_req
    t0 = time.perf_counter()
    vt_offset = 0.0

    def vt():
        return (time.perf_counter() - t0) * time_scale + vt_offset

    while finished < n_req:
        now = vt()
        while next_arrival < n_req and arrival_s[next_arrival] <= now:
            waiting.append(next_arrival)
            next_arrival += 1
        progressed = False

        # ---- prefill worker
        if prefill_inflight is not None and ctx.phase_query(PRE):
            ms = ctx.phase_last_ms(PRE)
            pre_ms.append(ms)
            for r in prefill_inflight:
                ready.append(r)
                if adj is not None and not first_prefill_done[r]:
                    first_prefill_done[r] = True
                    v = max(0.0, vt() - float(arrival_s[r]))
                    adj.observe_ttft(v)
                    if log_ops:
                        adj_log.append(("ttft", v))
            prefill_inflight = None
            progressed = True
        if prefill_inflight is None and waiting:
            batch, toks = [], 0
            while waiting and (not batch or toks + prompt_len[waiting[0]] <= max_prefill_tokens) and len(batch) < prefill_cap:
                r = waiting.popleft()
                batch.append(r)
                toks += prompt_len[r]
            cu = [0]
            for r in batch:
                cu.append(cu[-1] + prompt_len[r])
            try:
                pool.prefill_step(batch, cu, pq, pk, pv, pout, H, Hkv, d, dv, scale)
                for r in batch:
                    ops.append(("reserve", r, prompt_len[r]))
                    ctx_len[r] = prompt_len[r]
                prefill_inflight = batch
                pre_tokens.append(toks)
                issued_pre += 1
                prefill_cap = 64
                progressed = True
            except S.PoolExhausted:                                        # all-or-nothing: nothing was reserved
                exhausted_events += 1
                for r in reversed(batch):
                    waiting.appendleft(r)
                if len(batch) == 1 and not running and not ready and decode_inflight is None:
                    raise RuntimeError(f"request {batch[0]} ({prompt_len[batch[0]]} tokens) can never fit the pool")
                prefill_cap = max(1, len(batch) // 2)

        # ---- decode worker
        if decode_inflight is not None and ctx.phase_query(DEC):
            ms = ctx.phase_last_ms(DEC)
            dec_ms.append(ms)
            still = []
            for r in decode_inflight:
                generated[r] += 1
                if generated[r] >= int(output_len[r]):
                    pool.kv_free(r)
                    ops.append(("free", r, 0))
                    finished += 1
                else:
                    still.append(r)
            running = still
            decode_inflight = None
            progressed = True
            if adj is not None:
                v = ms * 1e-3 * time_scale
                adj.observe_tpot(v)
                x, y = adj.step(len(dec_ms), share[0], share[1])
                if log_ops:
                    adj_log.append(("tpot", v))
                    adj_log.append(("step", len(dec_ms), share[0], share[1], x, y))
                if (x, y) != (share[0], share[1]):
                    t1 = time.perf_counter()
                    ctx.set_partition(cus(x), cus(y))         # delayed + asynchronous: adopted at each phase's next step
                    adj_history.append((len(dec_ms), x, y, (time.perf_counter() - t1) * 1e3))
                    share = [x, y]
        if decode_inflight is None:
            while ready and len(running) < max_decode_batch:
                running.append(ready.popleft())
            if running:
                lens = [ctx_len[r] + 1 for r in running]
                try:
                    # requests join only after the host has seen their prefill step complete, so the
                    # pages they read are already visible: no GPU-side wait on the prefill stream
                    pool.decode_step(running, lens, dq, dout, H, scale, k_new=dk, v_new=dvn)
                    for r, n in zip(running, lens):
                        ops.append(("reserve", r, n))
                        ctx_len[r] = n
                    decode_inflight = list(running)
                    dec_batch.append(len(running))
                    issued_dec += 1
                    if log_ops and issued_dec % 100 == 1:
                        snapshots.append((len(ops), {r: pool.kv_block_table(r) for r in running[:8]}))
                    progressed = True
                except S.PoolExhausted:
                    # no page left for the next token: preempt the youngest running request
                    # (free its blocks; it is prefilled again later with the tokens it has so far)
                    exhausted_events += 1
                    victim = running.pop()
                    pool.kv_free(victim)
                    ops.append(("free", victim, 0))
                    prompt_len[victim] = ctx_len[victim]
                    waiting.appendleft(victim)
                    preemptions += 1
                    progressed = True

        # ---- controller: one resize, delayed + asynchronous (each phase adopts at its next step)
        if adj is None and resized_at_step is None and finished + len(running) + len(ready) >= resize_after_requests and next_arrival >= resize_after_requests:
            t1 = time.perf_counter()
            ctx.set_partition(cus(split_after[0]), cus(split_after[1]))
            resize_call_ms = (time.perf_counter() - t1) * 1e3
            resized_at_step = (issued_pre, issued_dec)

        total, free, live, _ = pool.stats() if (len(dec_ms) % 64 == 0) else (0, 0, 0, 0)
        if total:
            peak_used = max(peak_used, total - free)
        if not progressed and prefill_inflight is None and decode_inflight is None and not waiting and not running and not ready:
            if next_arrival < n_req:
                vt_offset += max(0.0, arrival_s[next_arrival] - vt())     # idle: jump to the next arrival
        elif not progressed:
            time.sleep(0)                                                  # yield; GPU work is in flight

    ctx.phase_sync(PRE)
    ctx.phase_sync(DEC)
    wall_s = time.perf_counter() - t0
    p_act, d_act, _, _ = ctx.get_partition()

    def around(xs, idx):
        before = xs[max(0, idx - 50):idx]
        after = xs[idx + 1:idx + 51]
        return {"median_before": _pct(before, 50), "median_after": _pct(after, 50)}

    stats = {
        "requests": n_req, "wall_s": wall_s, "time_scale": time_scale,
        "prefill_step_ms": _summary(pre_ms), "decode_step_ms": _summary(dec_ms),
        "prefill_tokens_per_step": _summary([float(x) for x in pre_tokens]),
        "decode_batch": _summary([float(x) for x in dec_batch]),
        "prefill_tok_s": (sum(pre_tokens) / (sum(pre_ms) * 1e-3)) if pre_ms else None,
        "decode_tok_s": (sum(dec_batch) / (sum(dec_ms) * 1e-3)) if dec_ms else None,
        "resize": {"from": list(split_before), "to": list(split_after), "set_partition_call_ms": resize_call_ms,
                   "at_step": resized_at_step, "active_cus_after": [p_act, d_act],
                   "prefill": around(pre_ms, resized_at_step[0]) if resized_at_step else None,
                   "decode": around(dec_ms, resized_at_step[1]) if resized_at_step else None,
                   "first_prefill_step_after_ms": pre_ms[resized_at_step[0]] if resized_at_step and resized_at_step[0] < len(pre_ms) else None,
                   "first_decode_step_after_ms": dec_ms[resized_at_step[1]] if resized_at_step and resized_at_step[1] < len(dec_ms) else None},
        "pool": {"pages": num_pages, "peak_used_pages": peak_used, "exhausted_events": exhausted_events, "preemptions": preemptions,
                 "final": pool.stats()},
    }
    if adj is not None:
        stats["adjuster"] = {"config": dict(adjuster), "start": [int(split_before[0]), int(split_before[1])],
                             "adjustments": len(adj_history), "history": [list(h) for h in adj_history], "final_share": share,
                             "model_a1_lambda_b1_a2_b2": list(adj.model()),
                             "set_partition_call_ms": _summary([h[3] for h in adj_history])}
        if log_ops:
            stats["adjuster"]["log"] = adj_log
        adj.close()
    free_list = pool.kv_free_list() if log_ops else None
    out_finite = bool(torch.isfinite(dout.float()).all().item())
    stats["decode_outputs_finite"] = out_finite
    pool.close()
    ctx.close()
    return stats, (ops if log_ops else None), snapshots, free_list


def main():
    import argparse
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import workloads as W

    ap = argparse.ArgumentParser(description="config 5: dynamic mixed trace on the Llama-3-8B layer shape")
    ap.add_argument("--requests", type=int, default=2000)
    ap.add_argument("--rate", type=float, default=8.0)
    ap.add_argument("--pool-frac", type=float, default=0.8, help="fraction of HBM given to the unified pool")
    ap.add_argument("--time-scale", type=float, default=128.0)
    ap.add_argument("--adjust", action="store_true", help="run the SLO-aware adjusting algorithm instead of one fixed resize")
    ap.add_argument("--slo-ttft", type=float, default=0.5, help="TTFT objective, virtual seconds")
    ap.add_argument("--slo-tpot", type=float, default=0.05, help="TPOT objective, virtual seconds")
    ap.add_argument("--window", type=int, default=100)
    args = ap.parse_args()
    import torch
    layer = W.get_config("c2").layer
    tr = W.trace(args.requests, args.rate)
    hbm = torch.cuda.get_device_properties(0).total_memory
    num_pages = int(args.pool_frac * hbm) // layer.page_bytes
    adjuster = dict(slo_ttft=args.slo_ttft, slo_tpot=args.slo_tpot, p_slo=90.0, window_size=args.window, max_step=4, step_size=10) if args.adjust else None
    stats, _, _, _ = replay(layer, tr.arrival_s, tr.input_len, tr.output_len, num_pages, time_scale=args.time_scale,
                            adjuster=adjuster)
    stats["config"] = {"workload": "c5_dynamic_trace", "layer": "Llama-3-8B attention layer", "rate_req_s": args.rate,
                       "pool_bytes": num_pages * layer.page_bytes}
    print(json.dumps(stats))


if __name__ == "__main__":
    main()
