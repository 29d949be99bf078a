"""RoPE step on the Llama-3-8B layer shape (32 query heads, 8 KV heads, 128 dims, Llama-3.1 scaling):
kernel time by HIP events on the prefill partition for a prompt batch and on the decode partition for a
decode batch, against the bytes it has to move (every q and k row read once and written once).
Run as `python -m paper_2504_19867_amd.rope_bench`."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import torch

from paper_2504_19867_amd import semipd as S

PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE
HQ, HKV, D = 32, 8, 128


def main():
    dev = torch.device("cuda:0")
    ctx = S.Context(0)
    total, _, _ = ctx.device_info()
    cfg = S.rope_config(theta=500000.0, factor=8.0)
    ctx.set_kernel_timing(True)
    for split in ((total // 2, total // 2), (total, total)):
        ctx.set_partition(*split)
        for phase, name, T in ((PRE, "prompt batch 4 x 2048", 8192), (PRE, "prompt batch 8 x 4096", 32768), (DEC, "decode batch", 64)):
            q = torch.randn((T, HQ, D), device=dev, dtype=torch.bfloat16)
            k = torch.randn((T, HKV, D), device=dev, dtype=torch.bfloat16)
            pos = [i % 4096 for i in range(T)] if phase == PRE else [2000 + 31 * i for i in range(T)]
            for _ in range(3):
                ctx.rope_qk(phase, cfg, pos, q, HQ, k, HKV, D)
            ctx.phase_sync(phase)
            ctx.phase_kernel_ms(phase)
            for _ in range(20):
                ctx.rope_qk(phase, cfg, pos, q, HQ, k, HKV, D)
            ctx.phase_sync(phase)
            ms = sorted(ctx.phase_kernel_ms(phase))
            med = ms[len(ms) // 2]
            nbytes = 2 * T * (HQ + HKV) * D * 2
            cus = split[0] if phase == PRE else split[1]
            print(f"{name:24s} on {cus:3d} CUs: {med * 1e3:7.1f} us  {nbytes / 1e6:7.1f} MB moved  {nbytes / med / 1e6:6.0f} GB/s", flush=True)
    # RoPE inside the prefill step (`rope` on the batch: keys rotated on their way into the pages) against the
    # rotation as a pass of its own before the step: wall time per step, 4 x 2048 tokens, page write included
    import math
    import time
    import workloads as W
    L = W.get_config("c2").layer
    ctx.set_kernel_timing(False)
    num_pages = 4096
    nbytes = S.pool_bytes(S.SPD_KV_GQA, L.page_tokens, L.n_kv_heads, L.dim_qk, L.dim_v, num_pages)
    mem = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pool = S.Pool(ctx, mem, nbytes, S.SPD_KV_GQA, L.page_tokens, L.n_kv_heads, L.dim_qk, L.dim_v, num_pages)
    lens = [2048] * 4
    T = sum(lens)
    cu = [0, 2048, 4096, 6144, 8192]
    pos = [i % 2048 for i in range(T)]
    q = torch.randn((T, HQ, D), device=dev, dtype=torch.bfloat16)
    k = torch.randn((T, HKV, D), device=dev, dtype=torch.bfloat16)
    v = torch.randn((T, HKV, D), device=dev, dtype=torch.bfloat16)
    out = torch.empty_like(q)
    scale = 1.0 / math.sqrt(D)
    plain = pool.make_prefill_batch([1, 2, 3, 4], cu, q, k, v, out, HQ, HKV, D, D, scale)
    inside = pool.make_prefill_batch([1, 2, 3, 4], cu, q, k, v, out, HQ, HKV, D, D, scale, rope=cfg)
    for split in ((total // 2, total // 2), (total, total)):
        ctx.set_partition(*split)
        row = []
        for name, fn in (("no RoPE", lambda: pool.prefill_step_batch(plain)),
                         ("RoPE pass + step", lambda: (ctx.rope_qk(PRE, cfg, pos, q, HQ, k, HKV, D), pool.prefill_step_batch(plain))),
                         ("RoPE inside the step", lambda: pool.prefill_step_batch(inside))):
            for _ in range(5):
                fn()
            ctx.phase_sync(PRE)
            t0 = time.perf_counter()
            for _ in range(40):
                fn()
            ctx.phase_sync(PRE)
            row.append(f"{name} {(time.perf_counter() - t0) / 40 * 1e6:6.1f} us")
        print(f"prefill step 4 x 2048 on {split[0]:3d} CUs: " + ", ".join(row), flush=True)
    pool.close()
    ctx.close()


if __name__ == "__main__":
    main()
