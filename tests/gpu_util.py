"""Helpers shared by the GPU parity tests: tensor marshalling and the parity bar."""
import numpy as np
import torch

import workloads as W
from paper_2504_19867_amd import semipd as S

MAX_ABS, MEAN_ABS = 2e-2, 2e-3      # bf16 outputs vs the fp64 oracle (the benchmark spec)
DEV = "cuda:0"


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def f64(bits: np.ndarray) -> np.ndarray:
    return W.bf16_bits_to_f32(bits).astype(np.float64)


def assert_parity(got: np.ndarray, want: np.ndarray, what: str):
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, \
        f"{what}: max abs {err.max():.3e} (bar {MAX_ABS}), mean abs {err.mean():.3e} (bar {MEAN_ABS})"
    return float(err.max()), float(err.mean())


class GpuPool:
    """A context + pool over a torch-owned byte buffer (optionally pre-filled with NaN patterns)."""

    def __init__(self, layer: W.LayerShape, num_pages: int, poison: bool = False, ctx: S.Context = None, kind: int = None):
        self.layer = layer
        self.kind = kind if kind is not None else (S.SPD_KV_GQA if layer.kind == "gqa" else S.SPD_KV_MLA_LATENT)
        self.dim_k = layer.dim_qk if layer.kind == "gqa" else layer.latent_dim
        self.dim_v = layer.dim_v if layer.kind == "gqa" else layer.latent_v_dim
        self.ctx = ctx or S.Context(0)
        self.own_ctx = ctx is None
        nbytes = S.pool_bytes(self.kind, layer.page_tokens, layer.n_kv_heads, self.dim_k, self.dim_v, num_pages)
        if poison:      # 0x7fc0 = bf16 quiet NaN in every slot: stale page contents must never leak
            self.mem = torch.full((nbytes // 2,), 0x7FC0, dtype=torch.int16, device=DEV).view(torch.uint8)
        else:
            self.mem = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        self.pool = S.Pool(self.ctx, self.mem, nbytes, self.kind, layer.page_tokens, layer.n_kv_heads, self.dim_k,
                           self.dim_v, num_pages)

    def close(self):
        self.pool.close()
        if self.own_ctx:
            self.ctx.close()
