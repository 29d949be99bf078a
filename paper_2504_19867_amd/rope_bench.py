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
    ctx.close()


if __name__ == "__main__":
    main()
