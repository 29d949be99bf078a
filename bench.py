"""bench.py - throughput of the semi-PD hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: one prefill step
(block reservation, K/V page write, causal attention over the prompt batch) on the prefill CU
partition, running concurrently with `decode_per_prefill` decode steps (paged attention of the
decode batch over the unified pool) on the decode CU partition; the ratio is calibrated in the
warm-up so that both partitions stay busy, as the paper's two asynchronous workers do.
Workload: benchmark configs[1] (Llama-3-8B attention layer shape).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PRE, DEC = 0, 1
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.md")


def profiled_traffic(workload):
    """HBM bytes per launch (prefill kernel, decode kernels) of `workload` as the hardware byte counters saw them.
    Counters cannot be read from inside this process: rocprofv3 collects FETCH_SIZE and WRITE_SIZE in two runs of
    this same command, and the summary of those runs holds one row per workload and phase,
    `| traffic | <workload> | <phase> | <read bytes> | <written bytes> |` (calibrated against a plain copy of known
    size).  Read from there, never typed in here; (None, None) where no such run has been summarised."""
    got = {}
    try:
        for line in open(TRAFFIC_TABLE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and cells[0] == "traffic" and cells[1] == workload:
                got[cells[2]] = float(cells[3]) + float(cells[4])
    except OSError:
        pass
    return got.get("prefill"), got.get("decode")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--split", default="50/50", help="prefill%%/decode%% of the CUs for the headline run")
    ap.add_argument("--no-sweep", action="store_true", help="skip the CU-split sweep (solo + concurrent per split)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-extra", action="store_true", help="skip the other single-GPU workloads (configs 3 and 4 at 50/50)")
    ap.add_argument("--no-clock", action="store_true", help="skip the clock probe beside the phases")
    ap.add_argument("--no-solo", action="store_true",
                    help="profiling aid: skip the solo passes, so that every launch of the run is in the headline regime")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="profiling aid: also run a plain 1 GiB copy kernel four times (known traffic for the byte counters)")
    ap.add_argument("--fp8-kv", action="store_true",
                    help="profiling aid: run the headline passes of an MLA config over the FP8 latent cache")
    ap.add_argument("--pool-gb", type=float, default=None, help="override pool size (GB)")
    ap.add_argument("--no-scramble", action="store_true", help="experiment: hand out physical pages in order")
    ap.add_argument("--decode-per-prefill", type=int, default=0,
                    help="fix r (decode steps per prefill step) and skip the solo calibration passes (profiling aid)")
    ap.add_argument("--only", default=None, choices=[None, "prefill", "decode"],
                    help="profiling aid: run only one phase in the timed region")
    return ap.parse_args()


def median(xs):
    s = sorted(xs)
    return s[len(s) // 2] if s else float("nan")


class Bench:
    def __init__(self, cfg, pool_gb=None, scramble=True, fp8=False):
        import torch
        from paper_2504_19867_amd import semipd as S
        self.torch, self.S, self.cfg = torch, S, cfg
        L = cfg.layer
        self.L = L
        self.dev = torch.device("cuda:0")
        self.ctx = S.Context(0)
        self.total_cus, self.xcds, self.gran = self.ctx.device_info()
        num_pages = cfg.num_pages if pool_gb is None else int(pool_gb * 1e9) // L.page_bytes
        self.num_pages = num_pages
        mla = L.kind == "mla"
        assert mla or not fp8, "the FP8 cache is the latent path's"
        kind = (S.SPD_KV_MLA_LATENT_FP8 if fp8 else S.SPD_KV_MLA_LATENT) if mla else S.SPD_KV_GQA
        pk, pv = (L.latent_dim, L.latent_v_dim) if mla else (L.dim_qk, L.dim_v)
        if fp8 and pool_gb is None:
            num_pages = self.num_pages = 40_000_000_000 // (L.page_tokens * 656)      # the same 40 GB hold 1.76 x the tokens
        nbytes = S.pool_bytes(kind, L.page_tokens, L.n_kv_heads, pk, pv, num_pages)
        self.mem = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        self.pool = S.Pool(self.ctx, self.mem, nbytes, kind, L.page_tokens, L.n_kv_heads, pk, pv, num_pages)
        self.scale = 1.0 / math.sqrt(L.dim_qk)
        gen = torch.Generator(device=self.dev)
        gen.manual_seed(cfg.seed)

        def randn(*shape, std=1.0):
            x = torch.randn(*shape, generator=gen, device=self.dev, dtype=torch.float32)
            return (x * std if std != 1.0 else x).to(torch.bfloat16)

        # scattered physical pages, as after long serving
        import workloads as W
        touched = min(num_pages - 8, 4 * sum(-(-n // L.page_tokens) for n in cfg.decode_ctx) * 3)
        for op, r, n in (W.scramble_ops(touched, L.page_tokens, cfg.seed) if scramble else []):
            self.pool.kv_reserve(r, n) if op == "reserve" else self.pool.kv_free(r)

        # decode: 3 disjoint request sets (> 256 MB apart in use) so that no step finds its KV in cache
        self.B = len(cfg.decode_ctx)
        self.n_sets = 3
        self.dec_batches = []
        for s in range(self.n_sets):
            ids = [10_000 * (s + 1) + i for i in range(self.B)]
            for rid, n in zip(ids, cfg.decode_ctx):
                self.pool.kv_reserve(rid, n)
                if mla:
                    self.pool.kv_write(DEC, rid, 0, n, randn(n, L.latent_dim))
                else:
                    k = randn(n, L.n_kv_heads, L.dim_qk)
                    v = randn(n, L.n_kv_heads, L.dim_v)
                    self.pool.kv_write(DEC, rid, 0, n, k, v)
            self.ctx.phase_sync(DEC)
            if mla:
                q = randn(self.B, L.n_q_heads, L.latent_dim)
                q[..., : L.latent_v_dim] *= float(W.MLA_QABS_NOPE_STD)
                out = torch.empty((self.B, L.n_q_heads, L.latent_v_dim), dtype=torch.bfloat16, device=self.dev)
            else:
                q = randn(self.B, L.n_q_heads, L.dim_qk)
                out = torch.empty((self.B, L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=self.dev)
            self.dec_batches.append(self.pool.make_decode_batch(ids, cfg.decode_ctx, q, out, L.n_q_heads, self.scale))
        # prefill: 2 input sets
        self.T = sum(cfg.prefill_lens)
        cu = [0]
        for n in cfg.prefill_lens:
            cu.append(cu[-1] + n)
        self.pre_batches = []
        kvh = L.n_q_heads if mla else L.n_kv_heads          # MLA prefill is the un-absorbed multi-head form
        for s in range(2):
            q = randn(self.T, L.n_q_heads, L.dim_qk)
            k = randn(self.T, kvh, L.dim_qk, std=float(W.MLA_UP_STD) if mla else 1.0)
            v = randn(self.T, kvh, L.dim_v, std=float(W.MLA_UP_STD) if mla else 1.0)
            latent = randn(self.T, L.latent_dim) if mla else None
            out = torch.empty((self.T, L.n_q_heads, L.dim_v), dtype=torch.bfloat16, device=self.dev)
            ids = [100 * (s + 1) + i for i in range(len(cfg.prefill_lens))]
            self.pre_batches.append(self.pool.make_prefill_batch(ids, cu, q, k, v, out, L.n_q_heads, kvh,
                                                                 L.dim_qk, L.dim_v, self.scale, latent=latent))
        torch.cuda.synchronize()
        # algorithmic work
        G = L.n_q_heads
        self.prefill_flops = sum(2.0 * (L.dim_qk + L.dim_v) * G * n * (n + 1) / 2 for n in cfg.prefill_lens)
        if mla:
            kv_bytes = sum(cfg.decode_ctx) * (656 if fp8 else L.latent_dim * 2)      # FP8 rows: 512 codes + 4 scales + 64 bf16
            qo_bytes = self.B * L.n_q_heads * (L.latent_dim + L.latent_v_dim) * 2
        else:
            kv_bytes = sum(cfg.decode_ctx) * L.n_kv_heads * (L.dim_qk + L.dim_v) * 2
            qo_bytes = self.B * L.n_q_heads * (L.dim_qk + L.dim_v) * 2
        self.decode_bytes = float(kv_bytes + qo_bytes)
        self.n_pre = self.n_dec = 0

    def close(self):
        self.sync()
        self.pre_batches = self.dec_batches = None
        self.pool.close()
        self.ctx.close()

    def prefill(self):
        self.pool.prefill_step_batch(self.pre_batches[self.n_pre % 2])
        self.n_pre += 1

    def decode(self):
        self.pool.decode_step_batch(self.dec_batches[self.n_dec % self.n_sets])
        self.n_dec += 1

    def sync(self):
        self.ctx.phase_sync(PRE)
        self.ctx.phase_sync(DEC)

    def set_split(self, p_pct, d_pct):
        self.ctx.set_partition(max(1, round(self.total_cus * p_pct / 100)), max(1, round(self.total_cus * d_pct / 100)))
        self.prefill(); self.decode(); self.sync()          # both phases adopt the new streams
        return self.ctx.get_partition()[:2]

    def read_ceiling(self, phase, nbytes=4 << 30, reps=6):
        """GB/s of the read-only streaming kernels over `nbytes` on the phase's stream, the other phase idle:
        what the phase's CU share can read out of HBM at best, the yardstick of the decode kernels.  Two ways of
        reading (eight 16-byte register loads in flight per lane; 1 KiB loads into LDS, 16 in flight per wave):
        returns (the faster of the two, {"register_loads": GB/s, "lds_loads": GB/s})."""
        torch = self.torch
        if not hasattr(self, "_rd"):
            self._rd = torch.empty(nbytes // 8, dtype=torch.int64, device=self.dev).random_()
        got = {}
        for name, fn in (("register_loads", self.ctx.phase_read), ("lds_loads", self.ctx.phase_read_lds)):
            fn(phase, self._rd, nbytes)
            self.ctx.phase_sync(phase)
            t0 = time.perf_counter()
            for _ in range(reps):
                fn(phase, self._rd, nbytes)
            self.ctx.phase_sync(phase)
            got[name] = nbytes * reps / (time.perf_counter() - t0) / 1e9
        return max(got.values()), got

    def clock_probe(self, load, ms=4.0):
        """The shader clock the chip holds under `load` ("idle", "prefill", "decode", "both"): one wave on a
        stream of its own runs a fixed chain of dependent adds for about `ms` milliseconds while the load runs;
        returns MHz (cycle-counter ticks per tick of the constant 100 MHz counter) and cycles per add."""
        torch = self.torch
        if not hasattr(self, "_clk"):
            self._clk = (torch.cuda.Stream(device=self.dev), torch.zeros(4, dtype=torch.int64, device=self.dev))
        side, buf = self._clk
        iters = int(ms * 1e-3 * 2.0e9 / (64 * 5))          # ~5 cycles per dependent add
        self.sync()
        torch.cuda.synchronize()
        worker = None
        if load == "both":
            worker = self.pool.decode_worker_start(self.dec_batches)
            for _ in range(3):
                self.prefill()
            self.ctx.phase_sync(PRE)
        t_end = time.perf_counter() + ms * 1.5e-3
        self.ctx.clock_probe(side.cuda_stream, iters, buf)
        while time.perf_counter() < t_end:
            if load in ("prefill", "both"):
                self.prefill()
            elif load == "decode":
                self.decode()
            else:
                time.sleep(0.0002)
        if worker is not None:
            self.pool.decode_worker_stop(worker)
        self.sync()
        side.synchronize()
        w, c, _, _ = (int(x) for x in buf.cpu().tolist())
        return {"mhz": 100.0 * c / max(w, 1), "cycles_per_add": c / (64.0 * iters), "probe_ms": w / 1e5}

    def issue_probe(self):
        """Shader cycles per loop iteration of one MFMA, of eight vector instructions, of both from one wave, and of the
        two loops run by two waves of one SIMD beside each other (spd_issue_probe), on an otherwise idle chip."""
        torch = self.torch
        self.sync()
        torch.cuda.synchronize()
        buf = torch.zeros(8, dtype=torch.int64, device=self.dev)
        for _ in range(2):
            self.ctx.issue_probe(0, buf)
            torch.cuda.synchronize()
        v = [int(x) / 100.0 for x in buf.cpu().tolist()]
        return {"mfma_alone": v[0], "valu8_alone": v[1], "mfma_then_valu8_one_wave": v[2],
                "mfma_beside_other_waves_valu8": v[3], "valu8_beside_other_waves_mfma": v[4],
                "unit": "shader cycles per iteration (one 32x32x16 bf16 MFMA; four v_exp_f32 + four v_fma_f32)"}

    def partition_switch(self):
        """Cost of a resize: spd_set_partition for a split never seen (streams are created) and for one seen
        before (streams re-used), on the caller's thread; and what the swap costs the phases: the step that adopts
        the staged partition against a steady step, each timed from the call to the drain of its phase."""
        def one_step(fn, phase):
            t0 = time.perf_counter()
            fn()
            self.ctx.phase_sync(phase)
            return (time.perf_counter() - t0) * 1e3

        def set_ms(p, d):
            t0 = time.perf_counter()
            self.ctx.set_partition(p, d)
            return (time.perf_counter() - t0) * 1e3

        total, half = self.total_cus, self.total_cus // 2
        self.sync()
        a, b = (half, half), (half - self.gran, half + self.gran)       # 128/128 and 96/160 on this chip
        self.ctx.set_partition(*a)
        self.prefill(); self.decode(); self.sync()
        new_ms = set_ms(*b)                                               # 96/160: not used anywhere else in this run
        self.prefill(); self.decode(); self.sync()
        reuse = []
        steady = {"prefill": [], "decode": []}
        swap = {"prefill": [], "decode": []}
        for i in range(6):
            for _ in range(3):
                steady["prefill"].append(one_step(self.prefill, PRE))
                steady["decode"].append(one_step(self.decode, DEC))
            reuse.append(set_ms(*(a if i % 2 == 0 else b)))
            swap["prefill"].append(one_step(self.prefill, PRE))           # these two steps adopt the staged streams
            swap["decode"].append(one_step(self.decode, DEC))
        self.ctx.set_partition(*a)
        self.prefill(); self.decode(); self.sync()
        return {"set_partition_new_split_ms": new_ms, "set_partition_seen_split_ms": median(reuse),
                "steady_step_ms": {k: median(v) for k, v in steady.items()},
                "step_that_adopts_ms": {k: median(v) for k, v in swap.items()},
                "note": "steps timed one at a time, call to drain (host launch latency included in both rows)"}

    def time_solo(self, phase, n):
        """median kernel-level and step-level ms of `n` back-to-back steps of one phase, other phase idle"""
        fn = self.prefill if phase == PRE else self.decode
        self.ctx.set_kernel_timing(False)
        for _ in range(3):
            fn()
        self.ctx.phase_sync(phase)
        gc.collect()
        gc.disable()                  # a full collection of the driver's Python heap is a 6 ms pause
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        self.ctx.phase_sync(phase)
        wall = (time.perf_counter() - t0) * 1e3 / n
        gc.enable()
        self.ctx.set_kernel_timing(True)
        self.ctx.phase_kernel_ms(phase)
        for _ in range(n):
            fn()
        kms = self.ctx.phase_kernel_ms(phase)
        self.ctx.set_kernel_timing(False)
        return median(kms), wall

    def run_concurrent(self, steps, r, only=None, timing=False):
        """`steps` steps of (1 prefill || r decodes); returns wall ms/step and per-phase kernel ms lists
        (the lists are empty unless `timing`: event records slow the pipeline, so the throughput pass runs without)"""
        torch = self.torch
        self.sync()
        self.ctx.set_kernel_timing(timing)
        self.ctx.phase_kernel_ms(PRE); self.ctx.phase_kernel_ms(DEC)
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()                  # keep the Python driver's collector out of the timed region
        t0 = time.perf_counter()
        for _ in range(steps):
            if only != "decode":
                self.prefill()
            if only != "prefill":
                for _ in range(r):
                    self.decode()
        self.sync()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        gc.enable()
        pk, dk = self.ctx.phase_kernel_ms(PRE), self.ctx.phase_kernel_ms(DEC)
        self.ctx.set_kernel_timing(False)
        return wall_ms, pk, dk


def run_async(bench, steps, timing=False):
    """The paper's two asynchronous workers: this thread drives `steps` prefill steps back to back while the
    library's decode worker thread drives decode steps as fast as the decode partition takes them.  Returns wall
    ms per prefill step (K steps, from the first call to the prefill partition's drain, the decode worker running
    throughout), the number of decode steps issued meanwhile, the kernel ms lists."""
    torch = bench.torch
    bench.sync()
    bench.ctx.set_kernel_timing(timing)
    bench.ctx.phase_kernel_ms(PRE); bench.ctx.phase_kernel_ms(DEC)
    torch.cuda.synchronize()
    gc.collect()
    gc.disable()                        # keep the Python driver's collector out of the timed region
    # both workers are running before the clock starts (the decode worker's thread start-up is not part of a
    # step); the decode steps of the timed region are those issued between its two ends
    worker = bench.pool.decode_worker_start(bench.dec_batches)
    for _ in range(4):
        bench.prefill()
    while bench.pool.decode_worker_steps(worker) < 4:
        time.sleep(0.0005)
    bench.ctx.phase_sync(PRE)
    n0 = bench.pool.decode_worker_steps(worker)
    t0 = time.perf_counter()
    for _ in range(steps):
        bench.prefill()
    bench.ctx.phase_sync(PRE)
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    n_dec = bench.pool.decode_worker_steps(worker) - n0
    bench.pool.decode_worker_stop(worker)
    bench.ctx.phase_sync(DEC)
    torch.cuda.synchronize()
    gc.enable()
    pk, dk = bench.ctx.phase_kernel_ms(PRE), bench.ctx.phase_kernel_ms(DEC)
    bench.ctx.set_kernel_timing(False)
    return wall_ms, n_dec, pk, dk


def cpu_baseline(cfg, r):
    """The fp64 oracle, as it stands, timed on this host on a bounded sample of the same workload."""
    import numpy as np
    import workloads as W
    from oracle import attention as OA
    L = cfg.layer
    scale = 1.0 / math.sqrt(L.dim_qk)
    G = L.n_q_heads // L.n_kv_heads
    f = lambda b: W.bf16_bits_to_f32(b).astype(np.float64)
    mla = L.kind == "mla"
    # prefill sample: request 0, all heads
    n0 = cfg.prefill_lens[0]
    if mla:
        q, k, v, _, cu = W.mla_prefill_inputs(L, (n0,), cfg.seed)
    else:
        q, k, v, cu = W.prefill_inputs(L, (n0,), cfg.seed)
    t0 = time.perf_counter()
    OA.prefill_attention(f(q), f(k), f(v), cu, scale)
    t_p = (time.perf_counter() - t0) * (sum(cfg.prefill_lens) / n0)                   # whole prefill batch
    # decode sample: first quarter (MLA) or half (GQA) of the requests, all heads
    ns = cfg.decode_ctx[: max(1, len(cfg.decode_ctx) // (4 if mla else 2))]
    if mla:
        qd, cs = W.mla_decode_inputs(L, ns, cfg.seed + 1)
        t0 = time.perf_counter()
        for i in range(len(ns)):
            OA.mla_decode_latent(f(qd[i]), f(cs[i]), scale, L.latent_v_dim)
    else:
        qd, ks, vs = W.decode_inputs(L, ns, cfg.seed + 1)
        t0 = time.perf_counter()
        for i in range(len(ns)):
            OA.decode_attention(f(qd[i]), f(ks[i]), f(vs[i]), scale)
    t_d = (time.perf_counter() - t0) * (sum(cfg.decode_ctx) / sum(ns))                # whole decode batch
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    tokens = sum(cfg.prefill_lens) + r * len(cfg.decode_ctx)
    return {"value": tokens / (t_p + r * t_d), "unit": "tokens/s (one attention layer)", "cores": int(cores),
            "kind": "oracle",
            "sample": f"prefill: request 0 of {len(cfg.prefill_lens)}, all heads ({n0} tokens), scaled by tokens; "
                      f"decode: first {len(ns)} of {len(cfg.decode_ctx)} requests, all heads, scaled by context tokens; same "
                      f"1 prefill : {r} decode step mix as the GPU run",
            "prefill_tok_s": sum(cfg.prefill_lens) / t_p, "decode_tok_s": len(cfg.decode_ctx) / t_d}


def measure_config(cfg, args, steps, warmup, sweep, clock, fp8=False):
    """All figures of one workload: the headline split (solo passes, then the two asynchronous workers), optionally
    the split sweep and the clock probe; returns the workload's part of the JSON line."""
    bench = Bench(cfg, args.pool_gb, not args.no_scramble, fp8)
    p_pct, d_pct = (int(x) for x in args.split.split("/"))

    def measure_split(pp, dp, steps, warmup, only=None):
        p_cus, d_cus = bench.set_split(pp, dp)
        read_gbs, read_by = bench.read_ceiling(DEC)
        if args.decode_per_prefill > 0 or only:
            # fixed mix in lockstep (profiling aid), or one phase alone
            r = max(1, args.decode_per_prefill)
            solo_p_k = solo_p_w = solo_d_k = solo_d_w = float("nan")
            bench.run_concurrent(warmup, r, only)
            wall_ms, _, _ = bench.run_concurrent(steps, r, only)                       # the timed region: K steps
            _, pk, dk = bench.run_concurrent(min(steps, 64), r, only, timing=True)     # same steps again, kernels bracketed by events
        else:
            solo_p_k = solo_p_w = solo_d_k = solo_d_w = float("nan")
            if not args.no_solo:
                solo_p_k, solo_p_w = bench.time_solo(PRE, max(5, steps // 4))
                solo_d_k, solo_d_w = bench.time_solo(DEC, max(10, steps))
            run_async(bench, warmup)
            wall_ms, n_dec, _, _ = run_async(bench, steps)                              # the timed region: K prefill steps, decode free-running
            r = n_dec / steps
            _, _, pk, dk = run_async(bench, min(steps, 64), timing=True)               # again, kernels bracketed by events
        dec_gbs = bench.decode_bytes / (median(dk) * 1e-3) / 1e9 if dk else None
        solo_dec_gbs = bench.decode_bytes / (solo_d_k * 1e-3) / 1e9
        return {"split": f"{pp}/{dp}", "prefill_cus": p_cus, "decode_cus": d_cus, "decode_per_prefill": r,
                "ms_per_step": wall_ms, "decode_share_read_gbs": read_gbs, "decode_share_read_gbs_by_method": read_by,
                "prefill_tok_s": bench.T / wall_ms * 1e3 if only != "decode" else 0.0,
                "decode_tok_s": r * bench.B / wall_ms * 1e3 if only != "prefill" else 0.0,
                "prefill_kernel_ms": median(pk), "decode_kernel_ms": median(dk),
                "prefill_tflops": bench.prefill_flops / (median(pk) * 1e-3) / 1e12 if pk else None,
                "decode_gbs": dec_gbs, "decode_frac_of_share_read": dec_gbs / read_gbs if dec_gbs else None,
                "solo": {"prefill_kernel_ms": solo_p_k, "prefill_step_ms": solo_p_w, "decode_kernel_ms": solo_d_k,
                         "decode_step_ms": solo_d_w,
                         "prefill_tflops": bench.prefill_flops / (solo_p_k * 1e-3) / 1e12,
                         "decode_gbs": solo_dec_gbs, "decode_frac_of_share_read": solo_dec_gbs / read_gbs}}

    if args.calibrate_copy:
        torch = bench.torch
        a = torch.empty(1 << 30, dtype=torch.uint8, device=bench.dev).random_()
        b = torch.empty_like(a)
        for _ in range(4):
            bench.ctx.phase_copy(DEC, b, a, 1 << 30)
        bench.ctx.phase_sync(DEC)
        del a, b
    head = measure_split(p_pct, d_pct, steps, warmup, args.only)
    splits = [head]
    if sweep:
        for pp, dp in list(cfg.cu_splits) + [(100, 100)]:
            if (pp, dp) != (p_pct, d_pct):
                splits.append(measure_split(pp, dp, max(10, steps // 2), 2))
    clocks = switch = issue = None
    if clock:
        bench.set_split(p_pct, d_pct)
        clocks = {load: bench.clock_probe(load) for load in ("idle", "prefill", "decode", "both")}
        switch = bench.partition_switch()
        issue = bench.issue_probe()

    r = head["decode_per_prefill"]
    tokens_per_step = (bench.T if args.only != "decode" else 0) + (r * bench.B if args.only != "prefill" else 0)
    traffic_p, traffic_d = profiled_traffic(cfg.name + ("_fp8kv" if fp8 else ""))
    L = cfg.layer
    part = {
        "value": tokens_per_step / head["ms_per_step"] * 1e3,
        "ms_per_step": head["ms_per_step"],
        "config": {"workload": cfg.name, "note": cfg.note, "prefill_batch": list(cfg.prefill_lens),
                   "decode_batch": bench.B, "decode_ctx_mean": sum(cfg.decode_ctx) / bench.B,
                   "q_heads": L.n_q_heads, "kv_heads": L.n_kv_heads, "head_dim": L.dim_qk,
                   "page_tokens": L.page_tokens, "pool_pages": bench.num_pages,
                   "cu_split": head["split"], "prefill_cus": head["prefill_cus"], "decode_cus": head["decode_cus"],
                   "step": (f"1 prefill step || {r} decode steps (lockstep)" if isinstance(r, int) else
                            f"1 prefill step, the decode worker free-running beside it ({r:.2f} decode steps per prefill step)"),
                   "only": args.only},
        "prefill_tok_s": head["prefill_tok_s"], "decode_tok_s": head["decode_tok_s"],
        "roofline": {"bound": "mfma", "kernel": f"prefill_kernel<{L.dim_qk},{L.dim_v}>", "achieved": head["prefill_tflops"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": (head["prefill_tflops"] or 0.0) / PEAK_BF16_TFLOPS,
                     "traffic": traffic_p, "traffic_source": "profiles/hbm_traffic_pmc.md" if traffic_p else None,
                     "kernel_ms": head["prefill_kernel_ms"], "flops_per_launch": bench.prefill_flops,
                     "share_cus": head["prefill_cus"],
                     "frac_of_share_peak": (head["prefill_tflops"] or 0.0) / (PEAK_BF16_TFLOPS * head["prefill_cus"] / bench.total_cus)},
        "roofline_decode": {"bound": "hbm", "kernel": (("decode_mla_kernel<fp8 pages>" if fp8 else "decode_mla_kernel") if L.kind == "mla" else f"decode_gqa_kernel<{L.dim_qk}>") + " (+combine)", "achieved": head["decode_gbs"],
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": (head["decode_gbs"] or 0.0) / PEAK_HBM_GBS,
                            "traffic": traffic_d, "traffic_source": "profiles/hbm_traffic_pmc.md" if traffic_d else None,
                            "kernel_ms": head["decode_kernel_ms"],
                            "bytes_per_launch": bench.decode_bytes, "share_cus": head["decode_cus"],
                            "share_read_ceiling_gbs": head["decode_share_read_gbs"],
                            "share_read_ceiling_gbs_by_method": head["decode_share_read_gbs_by_method"],
                            "frac_of_share_read_ceiling": head["decode_frac_of_share_read"],
                            "solo_frac_of_share_read_ceiling": head["solo"]["decode_frac_of_share_read"]},
        "splits": splits,
    }
    if clocks:
        part["clock_probe"] = clocks
        # the same fractions against the share's peak at the shader clock the probe measured under that load
        # (the published peak is at 2.4 GHz; under load the chip runs below it)
        rf = part["roofline"]
        nominal = clocks["idle"]["mhz"]
        rf["frac_of_share_peak_at_measured_clock"] = rf["frac_of_share_peak"] * nominal / clocks["both"]["mhz"]
        if head["solo"].get("prefill_tflops"):
            rf["solo_frac_of_share_peak"] = head["solo"]["prefill_tflops"] / (PEAK_BF16_TFLOPS * head["prefill_cus"] / bench.total_cus)
            rf["solo_frac_of_share_peak_at_measured_clock"] = rf["solo_frac_of_share_peak"] * nominal / clocks["prefill"]["mhz"]
        part["partition_switch"] = switch
        part["issue_probe"] = issue
    bench.close()
    del bench
    gc.collect()
    return part, r


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the hot path of one MI355X; --gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import workloads as W
    cfg = W.get_config(args.config)
    part, r = measure_config(cfg, args, args.steps, args.warmup, not args.no_sweep, not args.no_clock, fp8=args.fp8_kv)
    result = {
        "metric": "prefill tok/s + decode tok/s at CU split; % MFMA peak / % HBM BW",
        "value": part.pop("value"),
        "unit": "tokens/s (prefill + decode tokens, one attention layer)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": part.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    result.update(part)
    if not args.no_extra and args.only is None:
        # the other workloads that fit one GPU, each with rooflines of its own, at the headline split
        result["configs"] = {}
        for name in ("c3", "c4"):
            other = W.get_config(name)
            if other.name == cfg.name:
                continue
            steps = max(10, args.steps // 2)
            sub, _ = measure_config(other, args, steps, 2, False, False)
            sub["steps"] = steps
            sub["unit"] = result["unit"]
            result["configs"][other.name] = sub
            if other.layer.kind == "mla":
                # the same workload over the FP8 latent cache (656 instead of 1152 bytes per cached token)
                sub8, _ = measure_config(other, args, steps, 2, False, False, fp8=True)
                sub8["steps"] = steps
                sub8["unit"] = result["unit"]
                sub8["config"]["kv_cache"] = "fp8 e4m3, one fp32 scale per 128 latent entries, rope entries bf16"
                result["configs"][other.name + "_fp8kv"] = sub8
        if cfg.name == "c2_llama3_8b":
            # config 5: the dynamic trace (2000 requests, Poisson 8/s, resize 40/60 -> 60/40 mid-run) replayed over a
            # 40 GB pool of the same layer shape; a failure is reported in the line, it does not take the line away
            try:
                import torch
                from paper_2504_19867_amd.trace_replay import replay
                torch.cuda.empty_cache()
                tr = W.trace(2000, 8.0)
                st, _, _, _ = replay(cfg.layer, tr.arrival_s, tr.input_len, tr.output_len, 40_000_000_000 // cfg.layer.page_bytes)
                result["configs"]["c5_dynamic_trace"] = {
                    "requests": st["requests"], "wall_s": st["wall_s"], "time_scale": st["time_scale"],
                    "prefill_tok_s": st["prefill_tok_s"], "decode_tok_s": st["decode_tok_s"],
                    "prefill_step_ms_p50": st["prefill_step_ms"]["p50"], "decode_step_ms_p50": st["decode_step_ms"]["p50"],
                    "decode_batch_mean": st["decode_batch"].get("mean"), "decode_batch_p50": st["decode_batch"]["p50"],
                    "resize": {k: st["resize"][k] for k in ("from", "to", "set_partition_call_ms", "active_cus_after",
                                                            "first_prefill_step_after_ms", "first_decode_step_after_ms")},
                    "preemptions": st["pool"]["preemptions"], "peak_used_pages": st["pool"]["peak_used_pages"],
                    "decode_outputs_finite": st["decode_outputs_finite"],
                    "unit": "step times from the phases' own events; tokens/s = tokens of the steps / summed step times"}
            except Exception as e:          # noqa: BLE001 (whatever it is, it goes into the line)
                result["configs"]["c5_dynamic_trace"] = {"error": repr(e)}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, r)
    print(json.dumps(result))
    sys.stdout.flush()


if __name__ == "__main__":
    main()
