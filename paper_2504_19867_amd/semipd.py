"""Thin ctypes binding of libsemipd.so: same names as include/semipd.h, argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels.  Device buffers are passed
as integer addresses (e.g. ``tensor.data_ptr()``); PyTorch is only the caller's way to own
device memory.  There is no CPU fallback: if the library is missing the import fails.

PyTorch ships its own copy of the HIP runtime.  A process must use ONE runtime for the tensors
and for this library (a second copy finds no device), so when PyTorch is installed it is imported
first: the library's dependency on libamdhip64 then resolves to the copy PyTorch has loaded.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SEMIPD_LIB", os.path.join(_HERE, "libsemipd.so"))   # override: a differently built library

SPD_OK, SPD_EINVAL, SPD_ENOMEM, SPD_ENOENT, SPD_EHIP, SPD_ESTATE, SPD_ETOOBIG = 0, -1, -2, -3, -5, -6, -7
SPD_PHASE_PREFILL, SPD_PHASE_DECODE = 0, 1
SPD_KV_GQA, SPD_KV_MLA_LATENT, SPD_KV_MLA_LATENT_FP8 = 0, 1, 2

EXPORTS = [
    "spd_ctx_create", "spd_ctx_destroy", "spd_device_info", "spd_pool_bytes", "spd_pool_create",
    "spd_pool_destroy", "spd_pool_stats", "spd_kv_reserve", "spd_kv_free", "spd_kv_block_table",
    "spd_kv_free_list", "spd_kv_write", "spd_kv_gather", "spd_prefill_step", "spd_decode_step",
    "spd_phase_sync", "spd_phase_query", "spd_phase_wait_for", "spd_phase_stream", "spd_phase_last_ms",
    "spd_set_partition", "spd_get_partition", "spd_phase_cu_mask", "spd_partition_masks",
    "spd_phase_probe_cus", "spd_strerror", "spd_last_hip_error", "spd_set_kernel_timing", "spd_phase_kernel_ms", "spd_phase_copy",
    "spd_decode_worker_start", "spd_decode_worker_stop", "spd_decode_worker_steps",
    "spd_ctrl_create", "spd_ctrl_destroy", "spd_ctrl_observe_ttft", "spd_ctrl_observe_tpot", "spd_ctrl_step", "spd_ctrl_model",
    "spd_rope_inv_freq", "spd_rope_qk", "spd_ffn_gate_up", "spd_ffn_pack_gate_up",
    "spd_decode_step_noalloc", "spd_noalloc_limits", "spd_phase_read", "spd_phase_read_lds", "spd_clock_probe", "spd_issue_probe",
    "spd_shm_pool_create", "spd_shm_pool_open", "spd_shm_pool_close", "spd_shm_pool_unlink", "spd_shm_pool_stats",
    "spd_shm_kv_reserve", "spd_shm_kv_free", "spd_shm_kv_block_table", "spd_shm_kv_free_list",
]


class SpdError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} (status {status}, hip error {last_hip_error()})")


class PoolExhausted(SpdError):
    pass


class spd_pool_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("page_tokens", C.c_int32), ("n_kv_heads", C.c_int32),
                ("dim_k", C.c_int32), ("dim_v", C.c_int32), ("num_pages", C.c_int64)]


class spd_ctrl_config(C.Structure):
    _fields_ = [("slo_ttft", C.c_double), ("slo_tpot", C.c_double), ("p_slo", C.c_double), ("window_size", C.c_int32),
                ("max_step", C.c_int32), ("step_size", C.c_int32), ("history", C.c_int32)]


class spd_rope_config(C.Structure):
    _fields_ = [("theta", C.c_double), ("factor", C.c_double), ("low_freq_factor", C.c_double),
                ("high_freq_factor", C.c_double), ("original_max_pos", C.c_int32), ("rotary_dim", C.c_int32),
                ("rotary_offset", C.c_int32), ("interleaved", C.c_int32)]


class spd_prefill_batch(C.Structure):
    _fields_ = [("n_req", C.c_int32), ("req_ids", C.POINTER(C.c_uint64)), ("cu_seqlens", C.POINTER(C.c_int32)),
                ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("latent", C.c_void_p),
                ("out", C.c_void_p), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("dim_qk", C.c_int32), ("dim_v", C.c_int32), ("scale", C.c_float),
                ("prefix_lens", C.POINTER(C.c_int32)), ("rope", C.POINTER(spd_rope_config))]


class spd_decode_batch(C.Structure):
    _fields_ = [("n_req", C.c_int32), ("req_ids", C.POINTER(C.c_uint64)), ("ctx_lens", C.POINTER(C.c_int32)),
                ("q", C.c_void_p), ("k_new", C.c_void_p), ("v_new", C.c_void_p), ("out", C.c_void_p),
                ("n_q_heads", C.c_int32), ("scale", C.c_float), ("rope", C.POINTER(spd_rope_config))]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    try:
        import torch  # noqa: F401  (loads PyTorch's HIP runtime first, see the module docstring)
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    P = C.POINTER
    sig = {
        "spd_ctx_create": [C.c_int, P(vp)],
        "spd_ctx_destroy": [vp],
        "spd_device_info": [vp, P(C.c_int), P(C.c_int), P(C.c_int)],
        "spd_pool_bytes": [P(spd_pool_desc), P(u64)],
        "spd_pool_create": [vp, vp, u64, P(spd_pool_desc), P(vp)],
        "spd_pool_destroy": [vp],
        "spd_pool_stats": [vp, P(i64), P(i64), P(i64), P(u64)],
        "spd_kv_reserve": [vp, u64, i32, P(u64)],
        "spd_kv_free": [vp, u64, P(u64)],
        "spd_kv_block_table": [vp, u64, P(i32), i32, P(i32)],
        "spd_kv_free_list": [vp, P(i32), i64, P(i64)],
        "spd_kv_write": [vp, vp, C.c_int, u64, i32, i32, vp, vp],
        "spd_kv_gather": [vp, vp, C.c_int, u64, i32, vp, vp],
        "spd_prefill_step": [vp, vp, P(spd_prefill_batch)],
        "spd_decode_step": [vp, vp, P(spd_decode_batch)],
        "spd_decode_step_noalloc": [vp, vp, P(spd_decode_batch)],
        "spd_noalloc_limits": [P(u64), P(u64)],
        "spd_phase_sync": [vp, C.c_int],
        "spd_phase_query": [vp, C.c_int, P(C.c_int)],
        "spd_phase_wait_for": [vp, C.c_int, C.c_int],
        "spd_phase_stream": [vp, C.c_int, P(vp)],
        "spd_phase_last_ms": [vp, C.c_int, P(C.c_float)],
        "spd_set_partition": [vp, C.c_int, C.c_int],
        "spd_get_partition": [vp, P(C.c_int), P(C.c_int), P(C.c_int), P(C.c_int)],
        "spd_phase_cu_mask": [vp, C.c_int, P(C.c_uint32), i32, P(i32)],
        "spd_partition_masks": [C.c_int, C.c_int, C.c_int, C.c_int, P(C.c_uint32), P(C.c_uint32), P(C.c_int), P(C.c_int)],
        "spd_phase_probe_cus": [vp, C.c_int, i32, P(i32), i32, P(i32)],
        "spd_last_hip_error": [],
        "spd_phase_copy": [vp, C.c_int, vp, vp, u64],
        "spd_phase_read": [vp, C.c_int, vp, u64],
        "spd_phase_read_lds": [vp, C.c_int, vp, u64],
        "spd_clock_probe": [vp, vp, u64, vp],
        "spd_issue_probe": [vp, vp, vp],
        "spd_set_kernel_timing": [vp, C.c_int],
        "spd_phase_kernel_ms": [vp, C.c_int, P(C.c_float), i32, P(i32)],
        "spd_decode_worker_start": [vp, vp, P(P(spd_decode_batch)), i32, P(vp)],
        "spd_decode_worker_stop": [vp, P(i64), P(C.c_int)],
        "spd_decode_worker_steps": [vp, P(i64)],
        "spd_ctrl_create": [P(spd_ctrl_config), P(vp)],
        "spd_ctrl_destroy": [vp],
        "spd_ctrl_observe_ttft": [vp, C.c_double],
        "spd_ctrl_observe_tpot": [vp, C.c_double],
        "spd_ctrl_step": [vp, i64, i32, i32, P(i32), P(i32)],
        "spd_ctrl_model": [vp, P(C.c_double)],
        "spd_rope_inv_freq": [P(spd_rope_config), P(C.c_double), i32],
        "spd_rope_qk": [vp, C.c_int, P(spd_rope_config), P(i32), i32, vp, i32, vp, i32, i32],
        "spd_ffn_gate_up": [vp, C.c_int, vp, vp, vp, i32, i32, i32],
        "spd_ffn_pack_gate_up": [vp, C.c_int, vp, vp, vp, i32, i32],
        "spd_shm_pool_create": [C.c_char_p, i64, i32, i32, P(vp)],
        "spd_shm_pool_open": [C.c_char_p, P(vp)],
        "spd_shm_pool_close": [vp],
        "spd_shm_pool_unlink": [C.c_char_p],
        "spd_shm_pool_stats": [vp, P(i64), P(i64), P(i64), P(u64)],
        "spd_shm_kv_reserve": [vp, u64, i32, P(u64)],
        "spd_shm_kv_free": [vp, u64, P(u64)],
        "spd_shm_kv_block_table": [vp, u64, P(i32), i32, P(i32)],
        "spd_shm_kv_free_list": [vp, P(i32), i64, P(i64)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.spd_strerror.argtypes = [C.c_int]
    lib.spd_strerror.restype = C.c_char_p
    return lib


lib = _load()


def strerror(status: int) -> str:
    return lib.spd_strerror(status).decode()


def last_hip_error() -> int:
    return lib.spd_last_hip_error()


def _check(status: int, what: str) -> None:
    if status == SPD_ENOMEM:
        raise PoolExhausted(status, what)
    if status != SPD_OK:
        raise SpdError(status, what)


def _ptr(x) -> Optional[int]:
    """Device address of a tensor-like (has data_ptr()), an int address, or None."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def rope_config(theta: float = 500000.0, factor: float = 1.0, low_freq_factor: float = 1.0, high_freq_factor: float = 4.0,
                original_max_pos: int = 8192, rotary_dim: int = 128, rotary_offset: int = 0,
                interleaved: bool = False) -> spd_rope_config:
    return spd_rope_config(theta, factor, low_freq_factor, high_freq_factor, original_max_pos, rotary_dim, rotary_offset,
                           int(interleaved))


def rope_inv_freq(cfg: spd_rope_config) -> List[float]:
    n = max(cfg.rotary_dim // 2, 1)
    buf = (C.c_double * n)()
    _check(lib.spd_rope_inv_freq(C.byref(cfg), buf, n), "spd_rope_inv_freq")
    return [float(buf[i]) for i in range(cfg.rotary_dim // 2)]


# ----------------------------------------------------------------------------- thin object wrappers
class Context:
    """spd_ctx: device=-1 makes a host-only context (allocator and partition state only)."""

    def __init__(self, device: int = 0):
        h = C.c_void_p()
        _check(lib.spd_ctx_create(device, C.byref(h)), "spd_ctx_create")
        self.h = h
        self.device = device

    def close(self) -> None:
        if self.h:
            _check(lib.spd_ctx_destroy(self.h), "spd_ctx_destroy")
            self.h = None

    def device_info(self) -> Tuple[int, int, int]:
        a, b, c = C.c_int(), C.c_int(), C.c_int()
        _check(lib.spd_device_info(self.h, C.byref(a), C.byref(b), C.byref(c)), "spd_device_info")
        return a.value, b.value, c.value

    def set_partition(self, prefill_cus: int, decode_cus: int) -> None:
        _check(lib.spd_set_partition(self.h, prefill_cus, decode_cus), "spd_set_partition")

    def get_partition(self) -> Tuple[int, int, int, int]:
        v = [C.c_int() for _ in range(4)]
        _check(lib.spd_get_partition(self.h, *[C.byref(x) for x in v]), "spd_get_partition")
        return tuple(x.value for x in v)

    def phase_cu_mask(self, phase: int) -> List[int]:
        words = (C.c_uint32 * 32)()
        n = C.c_int32()
        _check(lib.spd_phase_cu_mask(self.h, phase, words, 32, C.byref(n)), "spd_phase_cu_mask")
        return [int(words[i]) for i in range(n.value)]

    def phase_sync(self, phase: int) -> None:
        _check(lib.spd_phase_sync(self.h, phase), "spd_phase_sync")

    def phase_query(self, phase: int) -> bool:
        d = C.c_int()
        _check(lib.spd_phase_query(self.h, phase, C.byref(d)), "spd_phase_query")
        return bool(d.value)

    def phase_wait_for(self, phase: int, other: int) -> None:
        _check(lib.spd_phase_wait_for(self.h, phase, other), "spd_phase_wait_for")

    def phase_stream(self, phase: int) -> int:
        s = C.c_void_p()
        _check(lib.spd_phase_stream(self.h, phase, C.byref(s)), "spd_phase_stream")
        return s.value or 0

    def phase_last_ms(self, phase: int) -> float:
        ms = C.c_float()
        _check(lib.spd_phase_last_ms(self.h, phase, C.byref(ms)), "spd_phase_last_ms")
        return ms.value

    def phase_copy(self, phase: int, dst, src, nbytes: int) -> None:
        _check(lib.spd_phase_copy(self.h, phase, _ptr(dst), _ptr(src), nbytes), "spd_phase_copy")

    def phase_read(self, phase: int, src, nbytes: int) -> None:
        _check(lib.spd_phase_read(self.h, phase, _ptr(src), nbytes), "spd_phase_read")

    def phase_read_lds(self, phase: int, src, nbytes: int) -> None:
        _check(lib.spd_phase_read_lds(self.h, phase, _ptr(src), nbytes), "spd_phase_read_lds")

    def clock_probe(self, hip_stream: int, iters: int, dev_out) -> None:
        _check(lib.spd_clock_probe(self.h, hip_stream or None, iters, _ptr(dev_out)), "spd_clock_probe")

    def issue_probe(self, hip_stream: int, dev_out) -> None:
        _check(lib.spd_issue_probe(self.h, hip_stream or None, _ptr(dev_out)), "spd_issue_probe")

    def rope_qk(self, phase: int, cfg: "spd_rope_config", positions: Sequence[int], q, n_q_heads: int, k, n_kv_heads: int,
                dim: int) -> None:
        """In-place rotary embedding of q [T, n_q_heads, dim] and k [T, n_kv_heads, dim] on `phase`'s stream."""
        n = len(positions)
        pos = (C.c_int32 * max(n, 1))(*positions)
        _check(lib.spd_rope_qk(self.h, phase, C.byref(cfg), pos, n, _ptr(q), n_q_heads, _ptr(k), n_kv_heads, dim), "spd_rope_qk")

    def ffn_gate_up(self, phase: int, x, w_gu, out, n_tokens: int, hidden: int, inter: int) -> None:
        """out [T, inter] = silu(x W_gate^T) * (x W_up^T) from the joint matrix w_gu [2 inter, hidden], on `phase`'s stream."""
        _check(lib.spd_ffn_gate_up(self.h, phase, _ptr(x), _ptr(w_gu), _ptr(out), n_tokens, hidden, inter), "spd_ffn_gate_up")

    def ffn_pack_gate_up(self, phase: int, w_gate, w_up, w_gu, hidden: int, inter: int) -> None:
        """The joint matrix [2 inter, hidden] (blocks of 32 gate rows + their 32 up rows) from the two weight matrices."""
        _check(lib.spd_ffn_pack_gate_up(self.h, phase, _ptr(w_gate), _ptr(w_up), _ptr(w_gu), hidden, inter), "spd_ffn_pack_gate_up")

    def set_kernel_timing(self, on: bool) -> None:
        _check(lib.spd_set_kernel_timing(self.h, int(on)), "spd_set_kernel_timing")

    def phase_kernel_ms(self, phase: int) -> List[float]:
        buf = (C.c_float * 256)()
        n = C.c_int32()
        _check(lib.spd_phase_kernel_ms(self.h, phase, buf, 256, C.byref(n)), "spd_phase_kernel_ms")
        return [float(buf[i]) for i in range(n.value)]

    def phase_probe_cus(self, phase: int, n_blocks: int = 4096) -> List[int]:
        ids = (C.c_int32 * 2048)()
        n = C.c_int32()
        _check(lib.spd_phase_probe_cus(self.h, phase, n_blocks, ids, 2048, C.byref(n)), "spd_phase_probe_cus")
        return [int(ids[i]) for i in range(n.value)]


class Adjuster:
    """SLO-aware partition adjuster (spd_ctrl_*): marshalling only."""

    def __init__(self, slo_ttft: float, slo_tpot: float, p_slo: float = 90.0, window_size: int = 100, max_step: int = 4,
                 step_size: int = 10, history: int = 64):
        cfg = spd_ctrl_config(slo_ttft, slo_tpot, p_slo, window_size, max_step, step_size, history)
        h = C.c_void_p()
        _check(lib.spd_ctrl_create(C.byref(cfg), C.byref(h)), "spd_ctrl_create")
        self._h = h

    def close(self):
        if self._h:
            lib.spd_ctrl_destroy(self._h)
            self._h = None

    def observe_ttft(self, latency: float):
        _check(lib.spd_ctrl_observe_ttft(self._h, latency), "spd_ctrl_observe_ttft")

    def observe_tpot(self, latency: float):
        _check(lib.spd_ctrl_observe_tpot(self._h, latency), "spd_ctrl_observe_tpot")

    def step(self, it: int, x0: int, y0: int):
        x, y = C.c_int32(), C.c_int32()
        _check(lib.spd_ctrl_step(self._h, it, x0, y0, C.byref(x), C.byref(y)), "spd_ctrl_step")
        return x.value, y.value

    def model(self):
        out = (C.c_double * 5)()
        _check(lib.spd_ctrl_model(self._h, out), "spd_ctrl_model")
        return tuple(out)


def partition_masks(total_cus: int, granularity: int, prefill_cus: int, decode_cus: int):
    words = (total_cus + 31) // 32
    pm, dm = (C.c_uint32 * words)(), (C.c_uint32 * words)()
    p, d = C.c_int(), C.c_int()
    _check(lib.spd_partition_masks(total_cus, granularity, prefill_cus, decode_cus, pm, dm, C.byref(p), C.byref(d)),
           "spd_partition_masks")
    return list(pm), list(dm), p.value, d.value


def noalloc_limits() -> Tuple[int, int]:
    a, b = C.c_uint64(), C.c_uint64()
    _check(lib.spd_noalloc_limits(C.byref(a), C.byref(b)), "spd_noalloc_limits")
    return a.value, b.value


def pool_bytes(kind: int, page_tokens: int, n_kv_heads: int, dim_k: int, dim_v: int, num_pages: int) -> int:
    desc = spd_pool_desc(kind, page_tokens, n_kv_heads, dim_k, dim_v, num_pages)
    out = C.c_uint64()
    _check(lib.spd_pool_bytes(C.byref(desc), C.byref(out)), "spd_pool_bytes")
    return out.value


class ShmPool:
    """The allocator in POSIX shared memory (spd_shm_*): marshalling only.  `create=True` makes the segment,
    otherwise an existing one is opened (by another process, say)."""

    def __init__(self, name: str, num_pages: int = 0, page_tokens: int = 0, max_requests: int = 0, create: bool = False):
        h = C.c_void_p()
        self.name = name.encode()
        if create:
            _check(lib.spd_shm_pool_create(self.name, num_pages, page_tokens, max_requests, C.byref(h)), "spd_shm_pool_create")
        else:
            _check(lib.spd_shm_pool_open(self.name, C.byref(h)), "spd_shm_pool_open")
        self.h = h

    def close(self) -> None:
        if self.h:
            _check(lib.spd_shm_pool_close(self.h), "spd_shm_pool_close")
            self.h = None

    def unlink(self) -> None:
        _check(lib.spd_shm_pool_unlink(self.name), "spd_shm_pool_unlink")

    def stats(self) -> Tuple[int, int, int, int]:
        t, f, l, s = C.c_int64(), C.c_int64(), C.c_int64(), C.c_uint64()
        _check(lib.spd_shm_pool_stats(self.h, C.byref(t), C.byref(f), C.byref(l), C.byref(s)), "spd_shm_pool_stats")
        return t.value, f.value, l.value, s.value

    def kv_reserve(self, req_id: int, n_tokens_total: int) -> int:
        seq = C.c_uint64()
        _check(lib.spd_shm_kv_reserve(self.h, req_id, n_tokens_total, C.byref(seq)), "spd_shm_kv_reserve")
        return seq.value

    def kv_free(self, req_id: int) -> int:
        seq = C.c_uint64()
        _check(lib.spd_shm_kv_free(self.h, req_id, C.byref(seq)), "spd_shm_kv_free")
        return seq.value

    def kv_block_table(self, req_id: int) -> List[int]:
        n = C.c_int32()
        rc = lib.spd_shm_kv_block_table(self.h, req_id, None, 0, C.byref(n))
        if rc not in (SPD_OK, SPD_EINVAL):
            _check(rc, "spd_shm_kv_block_table")
        buf = (C.c_int32 * max(n.value, 1))()
        _check(lib.spd_shm_kv_block_table(self.h, req_id, buf, n.value, C.byref(n)), "spd_shm_kv_block_table")
        return [int(buf[i]) for i in range(n.value)]

    def kv_free_list(self) -> List[int]:
        n = C.c_int64()
        lib.spd_shm_kv_free_list(self.h, None, 0, C.byref(n))
        buf = (C.c_int32 * max(n.value, 1))()
        _check(lib.spd_shm_kv_free_list(self.h, buf, n.value, C.byref(n)), "spd_shm_kv_free_list")
        return [int(buf[i]) for i in range(n.value)]


class Pool:
    """spd_pool over caller-owned device memory (`dev_mem`: tensor or address; None with a host-only ctx)."""

    def __init__(self, ctx: Context, dev_mem, nbytes: int, kind: int, page_tokens: int, n_kv_heads: int,
                 dim_k: int, dim_v: int, num_pages: int):
        self.ctx = ctx
        self.desc = spd_pool_desc(kind, page_tokens, n_kv_heads, dim_k, dim_v, num_pages)
        self._mem = dev_mem                       # keep the tensor alive
        h = C.c_void_p()
        _check(lib.spd_pool_create(ctx.h, _ptr(dev_mem), nbytes, C.byref(self.desc), C.byref(h)), "spd_pool_create")
        self.h = h

    def close(self) -> None:
        if self.h:
            _check(lib.spd_pool_destroy(self.h), "spd_pool_destroy")
            self.h = None

    def stats(self) -> Tuple[int, int, int, int]:
        t, f, l, s = C.c_int64(), C.c_int64(), C.c_int64(), C.c_uint64()
        _check(lib.spd_pool_stats(self.h, C.byref(t), C.byref(f), C.byref(l), C.byref(s)), "spd_pool_stats")
        return t.value, f.value, l.value, s.value

    def kv_reserve(self, req_id: int, n_tokens_total: int) -> int:
        seq = C.c_uint64()
        _check(lib.spd_kv_reserve(self.h, req_id, n_tokens_total, C.byref(seq)), "spd_kv_reserve")
        return seq.value

    def kv_free(self, req_id: int) -> int:
        seq = C.c_uint64()
        _check(lib.spd_kv_free(self.h, req_id, C.byref(seq)), "spd_kv_free")
        return seq.value

    def kv_block_table(self, req_id: int) -> List[int]:
        n = C.c_int32()
        st = lib.spd_kv_block_table(self.h, req_id, None, 0, C.byref(n))
        if st not in (SPD_OK, SPD_EINVAL):
            _check(st, "spd_kv_block_table")
        buf = (C.c_int32 * max(1, n.value))()
        _check(lib.spd_kv_block_table(self.h, req_id, buf, n.value, C.byref(n)), "spd_kv_block_table")
        return [int(buf[i]) for i in range(n.value)]

    def kv_free_list(self) -> List[int]:
        import numpy as np
        total = self.stats()[0]
        buf = np.empty(total, dtype=np.int32)
        n = C.c_int64()
        _check(lib.spd_kv_free_list(self.h, buf.ctypes.data_as(C.POINTER(C.c_int32)), total, C.byref(n)),
               "spd_kv_free_list")
        return buf[: n.value].tolist()

    def kv_write(self, phase: int, req_id: int, start_pos: int, n_tokens: int, k, v=None) -> None:
        _check(lib.spd_kv_write(self.ctx.h, self.h, phase, req_id, start_pos, n_tokens, _ptr(k), _ptr(v)),
               "spd_kv_write")

    def kv_gather(self, phase: int, req_id: int, n_tokens: int, k_out, v_out=None) -> None:
        _check(lib.spd_kv_gather(self.ctx.h, self.h, phase, req_id, n_tokens, _ptr(k_out), _ptr(v_out)),
               "spd_kv_gather")

    def prefill_step(self, req_ids: Sequence[int], cu_seqlens: Sequence[int], q, k, v, out, n_q_heads: int,
                     n_kv_heads: int, dim_qk: int, dim_v: int, scale: float, latent=None, prefix_lens=None,
                     rope: Optional[spd_rope_config] = None) -> None:
        self.prefill_step_batch(self.make_prefill_batch(req_ids, cu_seqlens, q, k, v, out, n_q_heads, n_kv_heads,
                                                        dim_qk, dim_v, scale, latent, prefix_lens, rope))

    def make_prefill_batch(self, req_ids: Sequence[int], cu_seqlens: Sequence[int], q, k, v, out, n_q_heads: int,
                           n_kv_heads: int, dim_qk: int, dim_v: int, scale: float, latent=None, prefix_lens=None,
                           rope: Optional[spd_rope_config] = None):
        """Marshal once; the returned object can be passed to prefill_step_batch repeatedly."""
        n = len(req_ids)
        ids = (C.c_uint64 * n)(*req_ids)
        cu = (C.c_int32 * (n + 1))(*[int(x) for x in cu_seqlens])
        pre = (C.c_int32 * n)(*[int(x) for x in prefix_lens]) if prefix_lens is not None else None
        rp = C.pointer(rope) if rope is not None else None
        b = spd_prefill_batch(n, ids, cu, _ptr(q), _ptr(k), _ptr(v), _ptr(latent), _ptr(out), n_q_heads,
                              n_kv_heads, dim_qk, dim_v, scale, pre, rp)
        b._keep = (ids, cu, q, k, v, out, latent, pre, rope, rp)
        return b

    def prefill_step_batch(self, batch) -> None:
        _check(lib.spd_prefill_step(self.ctx.h, self.h, C.byref(batch)), "spd_prefill_step")

    def make_decode_batch(self, req_ids: Sequence[int], ctx_lens: Sequence[int], q, out, n_q_heads: int,
                          scale: float, k_new=None, v_new=None, rope: Optional[spd_rope_config] = None):
        """Marshal once; the returned object can be passed to decode_step_batch repeatedly."""
        n = len(req_ids)
        ids = (C.c_uint64 * n)(*req_ids)
        lens = (C.c_int32 * n)(*[int(x) for x in ctx_lens])
        rp = C.pointer(rope) if rope is not None else None
        b = spd_decode_batch(n, ids, lens, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), n_q_heads, scale, rp)
        b._keep = (ids, lens, q, out, k_new, v_new, rope, rp)
        return b

    def decode_worker_start(self, batches):
        """Start the library's decode worker thread cycling over `batches` (from make_decode_batch); returns a handle."""
        n = len(batches)
        arr = (C.POINTER(spd_decode_batch) * n)(*[C.pointer(b) for b in batches])
        h = C.c_void_p()
        _check(lib.spd_decode_worker_start(self.ctx.h, self.h, arr, n, C.byref(h)), "spd_decode_worker_start")
        return (h, arr, list(batches))

    def decode_worker_steps(self, worker) -> int:
        """Decode steps the running worker has issued so far."""
        steps = C.c_int64()
        _check(lib.spd_decode_worker_steps(worker[0], C.byref(steps)), "spd_decode_worker_steps")
        return steps.value

    def decode_worker_stop(self, worker) -> int:
        """Stop and join the worker; returns the number of decode steps it issued (raises on a failed step)."""
        steps, status = C.c_int64(), C.c_int()
        _check(lib.spd_decode_worker_stop(worker[0], C.byref(steps), C.byref(status)), "spd_decode_worker_stop")
        _check(status.value, "decode worker step")
        return steps.value

    def decode_step_batch(self, batch) -> None:
        _check(lib.spd_decode_step(self.ctx.h, self.h, C.byref(batch)), "spd_decode_step")

    def decode_step_noalloc_batch(self, batch) -> None:
        _check(lib.spd_decode_step_noalloc(self.ctx.h, self.h, C.byref(batch)), "spd_decode_step_noalloc")

    def decode_step(self, req_ids, ctx_lens, q, out, n_q_heads: int, scale: float, k_new=None, v_new=None, rope=None) -> None:
        self.decode_step_batch(self.make_decode_batch(req_ids, ctx_lens, q, out, n_q_heads, scale, k_new, v_new, rope))
