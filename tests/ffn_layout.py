"""Test-side reader of the library's packed gate/up weight format, written from the index formula in
include/semipd.h (spd_ffn_gate_up): tiles of 256 joint rows x 32 hidden entries (8192 elements), tile
(tn, ks) at element (tn * hidden / 32 + ks) * 8192; inside a tile joint row 256 tn + r keeps 32 elements
at r * 32, and its 8-element piece number s holds the hidden entries 32 ks + 8 (s ^ ((r >> 2) & 3)) .. + 7.
Joint row 64 b + j is gate row 32 b + j for j < 32, up row 32 b + j - 32 otherwise."""
import numpy as np


def unpack_gate_up(packed: np.ndarray, hidden: int):
    """(w_gate, w_up), each [inter, hidden], from the flat packed array: one element at a time."""
    packed = np.asarray(packed).ravel()
    rows = packed.size // hidden
    inter = rows // 2
    n_ks = hidden // 32
    w_gate = np.empty((inter, hidden), dtype=packed.dtype)
    w_up = np.empty((inter, hidden), dtype=packed.dtype)
    for joint in range(rows):
        tn, r = divmod(joint, 256)
        b, j = divmod(joint, 64)
        dst, n = (w_gate, 32 * b + j) if j < 32 else (w_up, 32 * b + j - 32)
        for k in range(hidden):
            ks, kk = divmod(k, 32)
            c, e = divmod(kk, 8)
            s = c ^ ((r >> 2) & 3)
            dst[n, k] = packed[(tn * n_ks + ks) * 8192 + r * 32 + s * 8 + e]
    return w_gate, w_up
