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
matrices laid together; `joint_rows` is that joint matrix in the row order the library documents
(blocks of 32 gate rows followed by the 32 up rows of the same output columns).  How the library
stores that matrix in memory (its tiled byte layout) is not this module's business: the tests read
it back with an inverse of their own, written from the header's index formula.

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
