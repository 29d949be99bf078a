"""Gate/up GEMM of the gated FFN (one product, activation on the accumulators) on the Llama-3-8B layer shape
(hidden 4096, inter 14336) and on one tensor-parallel quarter of the Llama-3-70B one (hidden 8192, inter 7168):
kernel time by HIP events on the prefill partition for a prompt batch (matrix-core bound: 4 T hidden inter flops)
and on the decode partition for a decode batch (bound by reading the weights once: 4 hidden inter bytes).
Inputs are normally distributed (constant operands would let the matrix cores clock higher).
Then both at once on the two halves of the chip: prompt-batch GEMMs on the prefill partition while the decode
partition runs decode-batch GEMMs back to back (the paper's point: a compute-bound and a bandwidth-bound phase
share one GPU).
Run as `python -m paper_2504_19867_amd.ffn_bench` (`--quick`: the Llama-3-8B prompt batch on half the chip only,
three launches, for counter runs)."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import torch

from paper_2504_19867_amd import semipd as S

PRE, DEC = S.SPD_PHASE_PREFILL, S.SPD_PHASE_DECODE
PEAK_TFLOPS, PEAK_GBS = 2500.0, 8000.0
SHAPES = (("llama-3-8b", 4096, 14336), ("llama-3-70b / TP4", 8192, 7168))


def main():
    dev = torch.device("cuda:0")
    ctx = S.Context(0)
    total, _, _ = ctx.device_info()
    quick = "--quick" in sys.argv
    ctx.set_kernel_timing(True)
    for split in ((total // 2, total // 2), (total, total))[:1 if quick else 2]:
        ctx.set_partition(*split)
        for model, K, I in SHAPES[:1 if quick else 2]:
            wg = torch.randn((I, K), device=dev, dtype=torch.float32).mul_(K ** -0.5).to(torch.bfloat16)
            wu = torch.randn((I, K), device=dev, dtype=torch.float32).mul_(K ** -0.5).to(torch.bfloat16)
            w_gu = torch.empty((2 * I, K), device=dev, dtype=torch.bfloat16)
            ctx.ffn_pack_gate_up(PRE, wg, wu, w_gu, K, I)
            ctx.phase_sync(PRE)
            # decode batches cycle over four copies of the weights (four layers' worth, 0.9 GB): one copy would stay
            # in the 256 MB memory-side cache from call to call, which a model with many layers never sees
            w_layers = [w_gu] + ([w_gu.clone() for _ in range(3)] if not quick else [])
            for phase, name, T in ((PRE, "prompt batch 4 x 2048", 8192), (DEC, "decode batch 64", 64), (DEC, "decode batch 256", 256))[:1 if quick else 3]:
                x = torch.randn((T, K), device=dev, dtype=torch.bfloat16)
                out = torch.empty((T, I), device=dev, dtype=torch.bfloat16)
                for i in range(1 if quick else 3):
                    ctx.ffn_gate_up(phase, x, w_layers[i % len(w_layers)] if phase == DEC else w_gu, out, T, K, I)
                ctx.phase_sync(phase)
                ctx.phase_kernel_ms(phase)
                for i in range(2 if quick else 12):
                    ctx.ffn_gate_up(phase, x, w_layers[i % len(w_layers)] if phase == DEC else w_gu, out, T, K, I)
                ctx.phase_sync(phase)
                ms = sorted(ctx.phase_kernel_ms(phase))
                med = ms[len(ms) // 2]
                cus = split[0] if phase == PRE else split[1]
                flops = 4.0 * T * K * I
                nbytes = 4.0 * K * I + 2.0 * T * K + 2.0 * T * I
                tf, gbs = flops / med / 1e9, nbytes / med / 1e6
                share = cus / total
                print(f"{model:18s} {name:22s} on {cus:3d} CUs: {med * 1e3:8.1f} us  {tf:7.1f} TFLOP/s ({100 * tf / (PEAK_TFLOPS * share):4.1f} % of the "
                      f"share's MFMA peak)  {gbs:6.0f} GB/s ({100 * gbs / PEAK_GBS:4.1f} % of HBM)", flush=True)
    if not quick:
        concurrent(ctx, dev, total)
    ctx.close()


def concurrent(ctx, dev, total):
    """Llama-3-8B shape: 8 prompt-batch GEMMs on the prefill half, decode-batch GEMMs on the other half meanwhile."""
    model, K, I = SHAPES[0]
    ctx.set_partition(total // 2, total // 2)
    wg = torch.randn((I, K), device=dev, dtype=torch.float32).mul_(K ** -0.5).to(torch.bfloat16)
    wu = torch.randn((I, K), device=dev, dtype=torch.float32).mul_(K ** -0.5).to(torch.bfloat16)
    w_gu = torch.empty((2 * I, K), device=dev, dtype=torch.bfloat16)
    ctx.ffn_pack_gate_up(PRE, wg, wu, w_gu, K, I)
    xp = torch.randn((8192, K), device=dev, dtype=torch.bfloat16)
    op = torch.empty((8192, I), device=dev, dtype=torch.bfloat16)
    xd = torch.randn((64, K), device=dev, dtype=torch.bfloat16)
    od = torch.empty((64, I), device=dev, dtype=torch.bfloat16)
    w_layers = [w_gu] + [w_gu.clone() for _ in range(3)]
    n_dec = [0]

    def dec():
        ctx.ffn_gate_up(DEC, xd, w_layers[n_dec[0] % 4], od, 64, K, I)
        n_dec[0] += 1
    res = {}
    for mode in ("solo", "concurrent"):
        for _ in range(2):
            ctx.ffn_gate_up(PRE, xp, w_gu, op, 8192, K, I)
            dec()
        ctx.phase_sync(PRE); ctx.phase_sync(DEC)
        ctx.phase_kernel_ms(PRE); ctx.phase_kernel_ms(DEC)
        if mode == "solo":
            for _ in range(8):
                ctx.ffn_gate_up(PRE, xp, w_gu, op, 8192, K, I)
            ctx.phase_sync(PRE)
            for _ in range(200):
                dec()
            ctx.phase_sync(DEC)
        else:
            for _ in range(8):                   # about 35 decode GEMMs fit beside one prompt-batch GEMM
                ctx.ffn_gate_up(PRE, xp, w_gu, op, 8192, K, I)
                for _ in range(30):
                    dec()
            ctx.phase_sync(PRE); ctx.phase_sync(DEC)
        pk, dk = sorted(ctx.phase_kernel_ms(PRE)), sorted(ctx.phase_kernel_ms(DEC))
        res[mode] = (pk[len(pk) // 2], dk[len(dk) // 2])
    for mode, (p, d) in res.items():
        print(f"{model} on {total // 2} + {total // 2} CUs, {mode:10s}: prompt-batch GEMM {p * 1e3:7.1f} us ({4.0 * 8192 * K * I / p / 1e9:6.1f} TFLOP/s)   "
              f"decode-batch GEMM {d * 1e3:6.1f} us ({4.0 * K * I / d / 1e6:5.0f} GB/s of weights)", flush=True)


if __name__ == "__main__":
    main()
