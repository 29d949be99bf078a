"""TEST INFRASTRUCTURE ONLY: plain fp64 reference of the gated FFN's first step.

Nothing in the product path imports this module; only tests, the smoke check and the CPU baseline
of a bench may.  It shares no code with the HIP kernels.

Paper, Evaluation, "Implementation based on DistServe": the first two matrix multiplications of the
gated FFN are fused into one.  The paper gives no formula; what is computed here is the published
definition of the gated (SwiGLU) FFN of the Llama models it serves (the readings are listed in the
design notes):

    g = x W_gate^T        u = x W_up^T        (x: [T, hidden], W_gate, W_up: [inter, hidden])
    out = silu(g) * u     silu(z) = z / (1 + exp(-z))

"One GEMM" means that both products come out of a single multiplication of x with the two weight
matrices laid together; `pack_gate_up` is that joint matrix in the row order the library documents
(blocks of 32 gate rows followed by the 32 up rows of the same output columns).

Results are fp64 and NOT rounded: a comparison with a bf16 kernel allows for the output rounding.
"""
from __future__ import annotations

import numpy as np

PACK_BLOCK = 32


def silu(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    return z / (1.0 + np.exp(-z))


def gate_up(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray) -> np.ndarray:
    """x: [T, hidden], w_gate, w_up: [inter, hidden] (any float dtype).  Returns fp64 [T, inter]."""
    x = np.asarray(x, dtype=np.float64)
    w_gate = np.asarray(w_gate, dtype=np.float64)
    w_up = np.asarray(w_up, dtype=np.float64)
    if x.ndim != 2 or w_gate.ndim != 2 or w_gate.shape != w_up.shape or w_gate.shape[1] != x.shape[1]:
        raise ValueError("x must be [T, hidden], the weights [inter, hidden]")
    g = x @ w_gate.T
    u = x @ w_up.T
    return silu(g) * u


def joint_rows(w_gate: np.ndarray, w_up: np.ndarray) -> np.ndarray:
    """The joint [2 inter, hidden] matrix: rows 64 b .. 64 b + 31 are gate rows 32 b .. 32 b + 31, rows
    64 b + 32 .. 64 b + 63 the up rows with the same numbers.  inter must be a multiple of 32."""
    w_gate = np.asarray(w_gate)
    w_up = np.asarray(w_up)
    inter, hidden = w_gate.shape
    if w_up.shape != (inter, hidden) or inter % PACK_BLOCK:
        raise ValueError("weights must have equal shapes and inter a multiple of 32")
    out = np.empty((2 * inter, hidden), dtype=w_gate.dtype)
    for b in range(inter // PACK_BLOCK):
        out[64 * b:64 * b + 32] = w_gate[32 * b:32 * b + 32]
        out[64 * b + 32:64 * b + 64] = w_up[32 * b:32 * b + 32]
    return out


def gate_up_joint(x: np.ndarray, w_joint: np.ndarray) -> np.ndarray:
    """The same result from the joint matrix: ONE product y = x W_joint^T, then out column 32 b + j is
    silu(y[:, 64 b + j]) * y[:, 64 b + 32 + j]."""
    x = np.asarray(x, dtype=np.float64)
    w_joint = np.asarray(w_joint, dtype=np.float64)
    if w_joint.shape[0] % 64 or w_joint.shape[1] != x.shape[1]:
        raise ValueError("joint matrix must be [2 inter, hidden] with inter a multiple of 32")
    y = x @ w_joint.T
    inter = w_joint.shape[0] // 2
    out = np.empty((x.shape[0], inter), dtype=np.float64)
    for b in range(inter // PACK_BLOCK):
        out[:, 32 * b:32 * b + 32] = silu(y[:, 64 * b:64 * b + 32]) * y[:, 64 * b + 32:64 * b + 64]
    return out


def pack_gate_up(w_gate: np.ndarray, w_up: np.ndarray) -> np.ndarray:
    """The library's packed weight format, as a flat array of 2 inter * hidden elements (the layout is part of
    the interface: it is written out in the header).  The joint matrix is cut into tiles of 256 joint rows x 32
    hidden entries; tile (tn, ks) starts at element (tn * (hidden / 32) + ks) * 8192; inside a tile, joint row
    256 tn + r keeps 64 bytes at element r * 32, and its 16-byte piece number s (8 elements) holds the hidden
    entries 32 ks + 8 (s ^ ((r >> 2) & 3)) .. + 7.  inter a multiple of 128, hidden a multiple of 32."""
    j = joint_rows(w_gate, w_up)
    rows, hidden = j.shape
    if rows % 256 or hidden % 32:
        raise ValueError("inter must be a multiple of 128 and hidden a multiple of 32")
    out = np.empty(rows * hidden, dtype=j.dtype)
    n_ks = hidden // 32
    for tn in range(rows // 256):
        for ks in range(n_ks):
            base = (tn * n_ks + ks) * 8192
            for r in range(256):
                for s_ in range(4):
                    c = s_ ^ ((r >> 2) & 3)
                    out[base + r * 32 + s_ * 8:base + r * 32 + s_ * 8 + 8] = j[256 * tn + r, 32 * ks + 8 * c:32 * ks + 8 * c + 8]
    return out


def unpack_gate_up(packed: np.ndarray, hidden: int):
    """Inverse of pack_gate_up, written as the element-wise index formula: (w_gate, w_up)."""
    packed = np.asarray(packed)
    rows = packed.size // hidden
    inter = rows // 2
    n_ks = hidden // 32
    w_gate = np.empty((inter, hidden), dtype=packed.dtype)
    w_up = np.empty((inter, hidden), dtype=packed.dtype)
    for R in range(rows):
        tn, r = divmod(R, 256)
        blk, jj = divmod(R, 64)
        dst = w_gate if jj < 32 else w_up
        n = 32 * blk + (jj & 31)
        for k in range(hidden):
            ks, kk = divmod(k, 32)
            c, e = divmod(kk, 8)
            s_ = c ^ ((r >> 2) & 3)
            dst[n, k] = packed[(tn * n_ks + ks) * 8192 + r * 32 + s_ * 8 + e]
    return w_gate, w_up
