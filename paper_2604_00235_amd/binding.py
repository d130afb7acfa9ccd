"""ctypes binding of libmacattn.so: the same entry points as include/mac_attn.h, argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI; there is no Python or CPU fallback.
If the shared library has not been built (paper_2604_00235_amd/build.py), importing a symbol from it fails
loudly.  torch appears here only as the owner of device memory and streams (data_ptr / cuda_stream).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmacattn.so")

MAC_ATTN_OK = 0
MAC_ATTN_ERR_INVALID_ARG = -1
MAC_ATTN_ERR_UNSUPPORTED = -2
MAC_ATTN_ERR_HIP = -3
MAC_ATTN_ERR_OOM = -4
MAC_ATTN_ERR_CORRUPT = -5
MAC_ATTN_ERR_TOO_LARGE = -6
MAC_ATTN_STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = (
    "mac_attn_init", "mac_attn_decode_step", "mac_attn_full_decode", "mac_attn_stats", "mac_attn_reset",
    "mac_attn_ring_peek", "mac_attn_ring_entry_bytes", "mac_attn_device_bytes", "mac_attn_set_timing",
    "mac_attn_kernel_us", "mac_attn_destroy", "mac_attn_strerror", "mac_attn_last_hip_error",
    "mac_attn_check_guards", "mac_attn_full_decode_static",
)


class mac_attn_config(C.Structure):
    _fields_ = [
        ("device", C.c_int32), ("max_slots", C.c_int32), ("max_batch", C.c_int32),
        ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("page_size", C.c_int32), ("window", C.c_int32), ("band", C.c_int32),
        ("threshold", C.c_float), ("sm_scale", C.c_float),
        ("max_kv_len", C.c_int32), ("chunk_tokens", C.c_int32), ("fuse_epilogue", C.c_int32),
        ("max_gap", C.c_int32), ("group_match", C.c_int32), ("out_dtype", C.c_int32), ("fused_hit_span", C.c_int32),
    ]


class mac_attn_step_args(C.Structure):
    _fields_ = [
        ("batch", C.c_int32),
        ("slot_ids", C.c_void_p), ("kv_lens", C.c_void_p),
        ("q_pre", C.c_void_p), ("q_rope", C.c_void_p), ("kv_pages", C.c_void_p),
        ("stride_page", C.c_int64), ("stride_kv", C.c_int64), ("stride_head", C.c_int64), ("stride_tok", C.c_int64),
        ("block_table", C.c_void_p), ("block_table_stride", C.c_int32),
        ("out", C.c_void_p), ("out_lse", C.c_void_p), ("match_pos", C.c_void_p), ("match_d2", C.c_void_p),
    ]


class mac_attn_static_geometry(C.Structure):
    _fields_ = [
        ("device", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("page_size", C.c_int32), ("sm_scale", C.c_float), ("max_kv_len", C.c_int32), ("chunk_tokens", C.c_int32),
        ("out_dtype", C.c_int32),
    ]


class mac_attn_stats_t(C.Structure):
    _fields_ = [
        ("steps", C.c_uint64), ("head_steps", C.c_uint64), ("hits", C.c_uint64), ("misses", C.c_uint64),
        ("sum_gap", C.c_uint64), ("kv_tokens_read", C.c_uint64), ("kv_tokens_full", C.c_uint64),
        ("sum_skip_frac", C.c_double), ("kv_tokens_split", C.c_uint64), ("kv_tokens_fused", C.c_uint64),
    ]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class MacAttnError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load_library()
        msg = lib.mac_attn_strerror(code).decode()
        detail = lib.mac_attn_last_hip_error().decode() if code in (MAC_ATTN_ERR_HIP, MAC_ATTN_ERR_OOM) else ""
        super().__init__(f"{where}: {msg} ({code})" + (f": {detail}" if detail else ""))
        self.code = code


_lib = None


PROBE_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmacprobe.so")
PROBE_EXPORTS = ("mac_probe_stream",)
_probe_lib = None


def load_probe_library() -> C.CDLL:
    """Load libmacprobe.so (the read-only streaming probe of include/mac_probe.h) and declare its prototype."""
    global _probe_lib
    if _probe_lib is not None:
        return _probe_lib
    if not os.path.exists(PROBE_LIB_PATH):
        raise FileNotFoundError(f"{PROBE_LIB_PATH} is missing: build it with `python -m paper_2604_00235_amd.build`")
    lib = C.CDLL(PROBE_LIB_PATH)
    lib.mac_probe_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.POINTER(C.c_float)]
    lib.mac_probe_stream.restype = C.c_int
    _probe_lib = lib
    return lib


def mac_probe_stream(buffer_ptr: int, order_ptr: int, n_segments: int, segment_bytes: int, non_temporal: bool,
                     work_groups: int, iterations: int, sink_ptr: int, stream: int) -> float:
    """include/mac_probe.h mac_probe_stream: microseconds per pass over n_segments x segment_bytes."""
    us = C.c_float(0.0)
    rc = load_probe_library().mac_probe_stream(buffer_ptr, order_ptr, n_segments, segment_bytes, int(non_temporal),
                                               work_groups, iterations, sink_ptr, stream, C.byref(us))
    if rc != 0:
        raise RuntimeError(f"mac_probe_stream failed ({rc})")
    return float(us.value)


def load_library() -> C.CDLL:
    """Load libmacattn.so and declare the prototypes.  Raises if the library is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_00235_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    lib.mac_attn_init.argtypes = [P(mac_attn_config), P(C.c_void_p)]
    lib.mac_attn_init.restype = C.c_int
    lib.mac_attn_decode_step.argtypes = [C.c_void_p, P(mac_attn_step_args), C.c_void_p]
    lib.mac_attn_decode_step.restype = C.c_int
    lib.mac_attn_full_decode.argtypes = [C.c_void_p, P(mac_attn_step_args), C.c_void_p]
    lib.mac_attn_full_decode.restype = C.c_int
    lib.mac_attn_full_decode_static.argtypes = [P(mac_attn_static_geometry), P(mac_attn_step_args), C.c_void_p]
    lib.mac_attn_full_decode_static.restype = C.c_int
    lib.mac_attn_stats.argtypes = [C.c_void_p, P(mac_attn_stats_t), C.c_int]
    lib.mac_attn_stats.restype = C.c_int
    lib.mac_attn_reset.argtypes = [C.c_void_p, P(C.c_int32), C.c_int32]
    lib.mac_attn_reset.restype = C.c_int
    lib.mac_attn_ring_peek.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p]
    lib.mac_attn_ring_peek.restype = C.c_int
    lib.mac_attn_ring_entry_bytes.argtypes = [C.c_int32]
    lib.mac_attn_ring_entry_bytes.restype = C.c_int64
    lib.mac_attn_device_bytes.argtypes = [P(mac_attn_config)]
    lib.mac_attn_device_bytes.restype = C.c_int64
    lib.mac_attn_check_guards.argtypes = [C.c_void_p]
    lib.mac_attn_check_guards.restype = C.c_int
    lib.mac_attn_set_timing.argtypes = [C.c_void_p, C.c_int]
    lib.mac_attn_set_timing.restype = C.c_int
    lib.mac_attn_kernel_us.argtypes = [C.c_void_p, P(C.c_double), P(C.c_int64)]
    lib.mac_attn_kernel_us.restype = C.c_int
    lib.mac_attn_destroy.argtypes = [C.c_void_p]
    lib.mac_attn_destroy.restype = None
    lib.mac_attn_strerror.argtypes = [C.c_int]
    lib.mac_attn_strerror.restype = C.c_char_p
    lib.mac_attn_last_hip_error.argtypes = []
    lib.mac_attn_last_hip_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(code: int, where: str):
    if code != MAC_ATTN_OK:
        raise MacAttnError(code, where)


# ----------------------------------------------------------------------------- same names as the C ABI
def mac_attn_init(cfg: mac_attn_config) -> C.c_void_p:
    ctx = C.c_void_p()
    _check(load_library().mac_attn_init(C.byref(cfg), C.byref(ctx)), "mac_attn_init")
    return ctx


def mac_attn_decode_step(ctx, args: mac_attn_step_args, stream: int = 0) -> None:
    _check(load_library().mac_attn_decode_step(ctx, C.byref(args), C.c_void_p(stream)), "mac_attn_decode_step")


def mac_attn_full_decode(ctx, args: mac_attn_step_args, stream: int = 0) -> None:
    _check(load_library().mac_attn_full_decode(ctx, C.byref(args), C.c_void_p(stream)), "mac_attn_full_decode")


def mac_attn_full_decode_static(geo: mac_attn_static_geometry, args: mac_attn_step_args, stream: int = 0) -> None:
    _check(load_library().mac_attn_full_decode_static(C.byref(geo), C.byref(args), C.c_void_p(stream)),
           "mac_attn_full_decode_static")


def mac_attn_stats(ctx, reset: bool = False) -> mac_attn_stats_t:
    st = mac_attn_stats_t()
    _check(load_library().mac_attn_stats(ctx, C.byref(st), int(reset)), "mac_attn_stats")
    return st


def mac_attn_check_guards(ctx) -> None:
    _check(load_library().mac_attn_check_guards(ctx), "mac_attn_check_guards")


def mac_attn_reset(ctx, slot_ids=None) -> None:
    if slot_ids is None:
        _check(load_library().mac_attn_reset(ctx, None, 0), "mac_attn_reset")
    else:
        arr = (C.c_int32 * len(slot_ids))(*[int(s) for s in slot_ids])
        _check(load_library().mac_attn_reset(ctx, arr, len(slot_ids)), "mac_attn_reset")


def mac_attn_ring_peek(ctx, slot: int, j: int, h: int, head_dim: int = 128):
    """Returns (q_pre bits uint16[d], summary float32[d], lse float, n_p int) of one ring entry."""
    import numpy as np
    q = np.zeros(head_dim, np.uint16)
    o = np.zeros(head_dim, np.float32)
    lse = C.c_float()
    n_p = C.c_int32()
    _check(load_library().mac_attn_ring_peek(ctx, slot, j, h, q.ctypes.data, o.ctypes.data,
                                             C.cast(C.byref(lse), C.c_void_p), C.cast(C.byref(n_p), C.c_void_p)),
           "mac_attn_ring_peek")
    return q, o, lse.value, n_p.value


def mac_attn_ring_entry_bytes(head_dim: int) -> int:
    return int(load_library().mac_attn_ring_entry_bytes(head_dim))


def mac_attn_device_bytes(cfg: mac_attn_config) -> int:
    return int(load_library().mac_attn_device_bytes(C.byref(cfg)))


def mac_attn_set_timing(ctx, enable: bool) -> None:
    _check(load_library().mac_attn_set_timing(ctx, int(enable)), "mac_attn_set_timing")


def mac_attn_kernel_us(ctx):
    """(sum_us[4] = match, attention, merge, write-back; n_calls) since the previous query."""
    us = (C.c_double * 4)()
    n = C.c_int64()
    _check(load_library().mac_attn_kernel_us(ctx, us, C.byref(n)), "mac_attn_kernel_us")
    return [us[i] for i in range(4)], n.value


def mac_attn_destroy(ctx) -> None:
    load_library().mac_attn_destroy(ctx)


# ----------------------------------------------------------------------------- torch-tensor convenience
class MacAttention:
    """Owns one context; takes torch tensors on the context's GPU and passes their addresses through."""

    def __init__(self, *, num_q_heads: int, num_kv_heads: int, window: int, band: int, threshold: float,
                 max_kv_len: int, max_slots: int, max_batch: Optional[int] = None, head_dim: int = 128,
                 page_size: int = 16, sm_scale: float = 0.0, chunk_tokens: int = 0, fuse_epilogue: bool = True,
                 max_gap: int = 0, group_match: bool = False, out_bf16: bool = False, fused_hit_span: int = 0,
                 device: int = 0):
        self.cfg = mac_attn_config(device, max_slots, max_batch or max_slots, num_q_heads, num_kv_heads, head_dim,
                                   page_size, window, band, threshold, sm_scale, max_kv_len, chunk_tokens,
                                   int(fuse_epilogue), int(max_gap), int(group_match), int(out_bf16),
                                   int(fused_hit_span))
        self.ctx = mac_attn_init(self.cfg)

    def make_args(self, *, kv_lens, q_rope, kv_pages, strides, block_table, out, slot_ids=None, q_pre=None,
                  out_lse=None, match_pos=None, match_d2=None) -> mac_attn_step_args:
        import torch
        assert kv_lens.dtype == torch.int32 and block_table.dtype == torch.int32
        assert out.dtype == (torch.bfloat16 if self.cfg.out_dtype else torch.float32)
        assert q_rope.dtype == torch.bfloat16 and kv_pages.dtype == torch.bfloat16
        assert q_rope.is_contiguous() and out.is_contiguous() and block_table.stride(1) == 1
        ptr = lambda t: None if t is None else t.data_ptr()
        return mac_attn_step_args(
            q_rope.shape[0], ptr(slot_ids), ptr(kv_lens), ptr(q_pre), ptr(q_rope), ptr(kv_pages),
            int(strides[0]), int(strides[1]), int(strides[2]), int(strides[3]),
            ptr(block_table), int(block_table.stride(0)), ptr(out), ptr(out_lse), ptr(match_pos), ptr(match_d2))

    def decode_step(self, args: mac_attn_step_args, stream: int = 0):
        mac_attn_decode_step(self.ctx, args, stream)

    def full_decode(self, args: mac_attn_step_args, stream: int = 0):
        mac_attn_full_decode(self.ctx, args, stream)

    def stats(self, reset: bool = False) -> dict:
        return mac_attn_stats(self.ctx, reset).as_dict()

    def reset(self, slot_ids=None):
        mac_attn_reset(self.ctx, slot_ids)

    def check_guards(self):
        mac_attn_check_guards(self.ctx)

    def ring_peek(self, slot: int, j: int, h: int):
        return mac_attn_ring_peek(self.ctx, slot, j, h, self.cfg.head_dim)

    def close(self):
        if self.ctx is not None:
            mac_attn_destroy(self.ctx)
            self.ctx = None

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass
