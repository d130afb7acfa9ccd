"""ctypes front end of the fp64 CPU oracle (oracle/mac_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this.
It neither imports nor is imported by the HIP library or its Python binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mac_oracle.c")
_LIB = os.path.join(_HERE, "libmacoracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over (request, head))."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Params(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("page_size", C.c_int32), ("window", C.c_int32), ("band", C.c_int32),
        ("threshold", C.c_double), ("sm_scale", C.c_double),
        ("stride_page", C.c_int64), ("stride_kv", C.c_int64), ("stride_head", C.c_int64), ("stride_tok", C.c_int64),
        ("block_table_stride", C.c_int32), ("num_threads", C.c_int32),
        ("max_gap", C.c_int32), ("group_match", C.c_int32),
    ]


class Stats(C.Structure):
    _fields_ = [
        ("steps", C.c_uint64), ("head_steps", C.c_uint64), ("hits", C.c_uint64), ("misses", C.c_uint64),
        ("sum_gap", C.c_uint64), ("kv_tokens_read", C.c_uint64), ("kv_tokens_full", C.c_uint64),
        ("sum_skip_frac", C.c_double),
    ]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int32
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


class Oracle:
    """Geometry + ring state of one MAC context, all on the host in fp64.

    Ring layout: ring_q u16 [slots, W, Hq, d]; ring_O f64 [slots, W, Hq, d];
    ring_lse f64 [slots, W, Hq]; ring_npos i32 [slots, W] (0 = empty).
    """

    def __init__(self, *, num_q_heads: int, num_kv_heads: int, head_dim: int, page_size: int,
                 window: int, band: int, threshold: float, sm_scale: Optional[float] = None,
                 strides: Tuple[int, int, int, int], max_slots: int, num_threads: int = 0,
                 max_gap: int = 0, group_match: bool = False):
        assert num_q_heads % num_kv_heads == 0 and head_dim <= 1024 and window >= 1 and band >= 0
        self.Hq, self.Hkv, self.d, self.ps = num_q_heads, num_kv_heads, head_dim, page_size
        self.W, self.B = window, band
        # the library receives the threshold and the scale as fp32; keep exactly those values
        self.T = float(np.float32(threshold))
        self.sm_scale = float(np.float32(sm_scale if sm_scale is not None else 1.0 / np.sqrt(head_dim)))
        self.strides = tuple(int(s) for s in strides)
        self.max_slots = max_slots
        self.num_threads = num_threads
        self.max_gap, self.group_match = int(max_gap), int(bool(group_match))
        self.reset()
        self.stats = Stats()

    def reset(self, slots=None):
        if slots is None:
            self.ring_q = np.zeros((self.max_slots, self.W, self.Hq, self.d), np.uint16)
            self.ring_O = np.zeros((self.max_slots, self.W, self.Hq, self.d), np.float64)
            self.ring_lse = np.full((self.max_slots, self.W, self.Hq), -np.inf, np.float64)
            self.ring_npos = np.zeros((self.max_slots, self.W), np.int32)
        else:
            for s in slots:
                self.ring_npos[s] = 0

    def _params(self, batch: int, block_table: np.ndarray) -> _Params:
        sp, skv, sh, st = self.strides
        return _Params(batch, self.Hq, self.Hkv, self.d, self.ps, self.W, self.B, self.T, self.sm_scale,
                       sp, skv, sh, st, block_table.shape[1], self.num_threads, self.max_gap, self.group_match)

    # ------------------------------------------------------------------ definitions
    def summary(self, q_rope, kv_pages, block_table, b: int, h: int, lo: int, hi: int):
        """(O, LSE) of keys [lo, hi) for request b, query head h."""
        q_rope, kv_pages, block_table = _u16(q_rope), _u16(kv_pages), _i32(block_table)
        P = self._params(q_rope.shape[0], block_table)
        O = np.zeros(self.d, np.float64)
        lse = C.c_double()
        _load().oracle_summary(C.byref(P), _p(q_rope), _p(kv_pages), _p(block_table), C.c_int32(b), C.c_int32(h),
                               C.c_int64(lo), C.c_int64(hi), _p(O), C.byref(lse))
        return O, lse.value

    @staticmethod
    def merge(Oa, la, Ob, lb):
        Oa = np.ascontiguousarray(Oa, np.float64)
        Ob = np.ascontiguousarray(Ob, np.float64)
        O = np.zeros_like(Oa)
        l = C.c_double()
        _load().oracle_merge(C.c_int32(Oa.shape[0]), _p(Oa), C.c_double(la), _p(Ob), C.c_double(lb), _p(O), C.byref(l))
        return O, l.value

    def full_decode(self, kv_lens, q_rope, kv_pages, block_table):
        q_rope, kv_pages, block_table, kv_lens = _u16(q_rope), _u16(kv_pages), _i32(block_table), _i32(kv_lens)
        batch = q_rope.shape[0]
        P = self._params(batch, block_table)
        out = np.zeros((batch, self.Hq, self.d), np.float64)
        lse = np.zeros((batch, self.Hq), np.float64)
        _load().oracle_full_decode(C.byref(P), _p(kv_lens), _p(q_rope), _p(kv_pages), _p(block_table), _p(out), _p(lse))
        return out, lse

    def match(self, slot_ids, kv_lens, q_pre):
        q_pre, slot_ids, kv_lens = _u16(q_pre), _i32(slot_ids), _i32(kv_lens)
        batch = q_pre.shape[0]
        P = self._params(batch, np.zeros((batch, 1), np.int32))
        pos = np.zeros((batch, self.Hq), np.int32)
        idx = np.zeros((batch, self.Hq), np.int32)
        d2 = np.zeros((batch, self.Hq), np.float64)
        _load().oracle_match(C.byref(P), _p(slot_ids), _p(kv_lens), _p(q_pre), _p(self.ring_q), _p(self.ring_npos),
                             _p(pos), _p(idx), _p(d2))
        return pos, idx, d2

    def mac_step(self, slot_ids, kv_lens, q_pre, q_rope, kv_pages, block_table):
        """One decode step.  Returns dict(out, lse, match_pos, d2, rect_O, rect_lse); updates rings + stats."""
        q_pre, q_rope, kv_pages = _u16(q_pre), _u16(q_rope), _u16(kv_pages)
        slot_ids, kv_lens, block_table = _i32(slot_ids), _i32(kv_lens), _i32(block_table)
        batch = q_pre.shape[0]
        P = self._params(batch, block_table)
        out = np.zeros((batch, self.Hq, self.d), np.float64)
        lse = np.zeros((batch, self.Hq), np.float64)
        pos = np.zeros((batch, self.Hq), np.int32)
        d2 = np.zeros((batch, self.Hq), np.float64)
        rO = np.zeros((batch, self.Hq, self.d), np.float64)
        rL = np.zeros((batch, self.Hq), np.float64)
        _load().oracle_mac_step(C.byref(P), _p(slot_ids), _p(kv_lens), _p(q_pre), _p(q_rope), _p(kv_pages),
                                _p(block_table), _p(self.ring_q), _p(self.ring_O), _p(self.ring_lse),
                                _p(self.ring_npos), _p(out), _p(lse), _p(pos), _p(d2), _p(rO), _p(rL),
                                C.byref(self.stats))
        return {"out": out, "lse": lse, "match_pos": pos, "d2": d2, "rect_O": rO, "rect_lse": rL}
