"""Chunked prefill on the Llama-3-8B layer shape: step time of 4 requests x `chunk` new tokens each over
`prefix` cached tokens (page write + gather of the context + attention), attention kernel time by HIP events.
Run as `python -m paper_2504_19867_amd.chunked_prefill_bench`."""
import math
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import torch

import workloads as W
from paper_2504_19867_amd import semipd as S

PRE = S.SPD_PHASE_PREFILL
R = 4                       # requests per step


def main():
    L = W.get_config("c2").layer
    dev = torch.device("cuda:0")
    ctx = S.Context(0)
    num_pages = 20000
    nbytes = S.pool_bytes(S.SPD_KV_GQA, L.page_tokens, L.n_kv_heads, L.dim_qk, L.dim_v, num_pages)
    mem = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pool = S.Pool(ctx, mem, nbytes, S.SPD_KV_GQA, L.page_tokens, L.n_kv_heads, L.dim_qk, L.dim_v, num_pages)
    scale = 1 / math.sqrt(L.dim_qk)
    ids = list(range(100, 100 + R))
    live = False
    for prefix, chunk in ((0, 2048), (1536, 512), (3584, 512), (7680, 512), (0, 512)):
        T = R * chunk
        q = torch.randn((T, L.n_q_heads, L.dim_qk), device=dev, dtype=torch.bfloat16)
        k = torch.randn((T, L.n_kv_heads, L.dim_qk), device=dev, dtype=torch.bfloat16)
        v = torch.randn((T, L.n_kv_heads, L.dim_v), device=dev, dtype=torch.bfloat16)
        out = torch.empty_like(q)
        for r in ids:
            if live:
                pool.kv_free(r)             # the steps of the case before have drained (phase_sync below)
            if prefix:
                pool.kv_reserve(r, prefix)
        live = True
        cu = [i * chunk for i in range(R + 1)]
        b = pool.make_prefill_batch(ids, cu, q, k, v, out, L.n_q_heads, L.n_kv_heads, L.dim_qk, L.dim_v, scale,
                                    prefix_lens=[prefix] * R if prefix else None)
        ctx.set_kernel_timing(True)
        for _ in range(3):
            pool.prefill_step_batch(b)
        ctx.phase_sync(PRE)
        ctx.phase_kernel_ms(PRE)
        n = 20
        t0 = time.perf_counter()
        for _ in range(n):
            pool.prefill_step_batch(b)
        ctx.phase_sync(PRE)
        wall = (time.perf_counter() - t0) / n * 1e3
        kms = sorted(ctx.phase_kernel_ms(PRE))
        km = kms[len(kms) // 2]
        flops = R * L.n_q_heads * 2 * (L.dim_qk + L.dim_v) * (chunk * prefix + chunk * (chunk + 1) / 2)
        print(f"prefix {prefix:5d} chunk {chunk:5d} x {R}: step wall {wall:.3f} ms, attention kernel {km:.3f} ms "
              f"({flops / km / 1e9:.0f} TFLOP/s), rest (page write + gather + launches) {wall - km:.3f} ms", flush=True)
    pool.close()
    ctx.close()


if __name__ == "__main__":
    main()
