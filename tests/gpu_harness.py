"""Runs the HIP library and the CPU oracle side by side on one workload and compares them (GPU tests only).

Tolerances (the benchmark spec): hit/miss decisions and matched positions bit-exact; outputs within max-abs 2e-3 and
relative-L2 1e-3 per (request, head) row (bf16 KV, fp32 accumulation).  Relative L2 is taken against the
oracle's row; rows whose norm is tiny fall back to the absolute bound.
"""
from __future__ import annotations

import sys

import numpy as np
import torch

from paper_2604_00235_amd import binding as mb
from paper_2604_00235_amd.workload import Workload, WorkloadConfig, bf16_bits
from tests.helpers import make_oracle

MAX_ABS = 2e-3
REL_L2 = 1e-3


def say(msg: str):
    print(msg, flush=True)
    sys.stdout.flush()


def check_rows(got: np.ndarray, ref: np.ndarray, what: str):
    """got, ref: [..., d].  Every row within max-abs and relative-L2 of the oracle."""
    got = got.astype(np.float64)
    diff = got - ref
    max_abs = np.abs(diff).max()
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert max_abs <= MAX_ABS, f"{what}: max-abs {max_abs:.3e} > {MAX_ABS}"
    num = np.linalg.norm(diff, axis=-1)
    den = np.linalg.norm(ref, axis=-1)
    rel = num / np.maximum(den, 1e-30)
    bad = (rel > REL_L2) & (num > 1e-6)
    assert not bad.any(), f"{what}: relative-L2 {rel[bad].max():.3e} > {REL_L2} (rows {np.argwhere(bad)[:4].tolist()})"
    return float(max_abs), float(rel[den > 0].max()) if (den > 0).any() else 0.0


class DeviceRun:
    """One library context + device buffers for a workload living on cuda:0."""

    def __init__(self, cfg: WorkloadConfig, wl: Workload, chunk_tokens: int = 0, strides=None, kv_pages=None,
                 max_kv_len=None, fuse_epilogue: bool = True, max_gap: int = 0, group_match: bool = False,
                 out_bf16: bool = False, fused_hit_span: int = 0, sm_scale: float = 0.0):
        self.cfg, self.wl = cfg, wl
        dev = wl.device
        self.mac = mb.MacAttention(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, window=cfg.window,
                                   band=cfg.band, threshold=cfg.threshold, max_kv_len=max_kv_len or cfg.max_kv_len,
                                   max_slots=cfg.batch, page_size=cfg.page_size, head_dim=cfg.head_dim, chunk_tokens=chunk_tokens,
                                   fuse_epilogue=fuse_epilogue, max_gap=max_gap, group_match=group_match,
                                   out_bf16=out_bf16, fused_hit_span=fused_hit_span, sm_scale=sm_scale)
        self.kv_pages = wl.kv_pages if kv_pages is None else kv_pages
        self.strides = wl.strides if strides is None else strides
        B, Hq, d = cfg.batch, cfg.num_q_heads, cfg.head_dim
        # caller-owned outputs sit between guard zones holding a pattern: a write outside an output shows up there
        self._guards = []
        self.out = self._guarded((B, Hq, d), torch.bfloat16 if out_bf16 else torch.float32, dev)
        self.lse = self._guarded((B, Hq), torch.float32, dev)
        self.pos = self._guarded((B, Hq), torch.int32, dev)
        self.d2 = self._guarded((B, Hq), torch.float64, dev)
        self.stream = torch.cuda.current_stream().cuda_stream

    GUARD_BYTES = 4096

    def _guarded(self, shape, dtype, dev):
        n = int(np.prod(shape))
        esz = torch.empty((), dtype=dtype).element_size()
        g = self.GUARD_BYTES // esz
        raw = torch.empty(n + 2 * g, dtype=dtype, device=dev)
        raw.view(torch.uint8).fill_(0xA5)
        view = raw[g:g + n].view(shape)
        view.zero_()
        self._guards.append((raw, g, n))
        return view

    def check_guards(self):
        self.mac.check_guards()          # the library's own buffers (rings, workspace, counters)
        for raw, g, n in self._guards:
            b = raw.view(torch.uint8)
            esz = raw.element_size()
            assert bool((b[:g * esz] == 0xA5).all()) and bool((b[(g + n) * esz:] == 0xA5).all()), "write outside an output buffer"

    def args(self, q_pre, q_rope, kv_lens):
        return self.mac.make_args(kv_lens=kv_lens, q_rope=q_rope, kv_pages=self.kv_pages, strides=self.strides,
                                  block_table=self.wl.block_table, out=self.out, slot_ids=self.wl.slot_ids,
                                  q_pre=q_pre, out_lse=self.lse, match_pos=self.pos, match_d2=self.d2)

    def mac_step(self, q_pre, q_rope, kv_lens):
        self.mac.decode_step(self.args(q_pre, q_rope, kv_lens), self.stream)
        torch.cuda.synchronize()
        self.check_guards()
        return (self.out.float().cpu().numpy().copy(), self.lse.cpu().numpy().copy(), self.pos.cpu().numpy().copy(),
                self.d2.cpu().numpy().copy())

    def full(self, q_rope, kv_lens):
        self.mac.full_decode(self.args(None, q_rope, kv_lens), self.stream)
        torch.cuda.synchronize()
        self.check_guards()
        return self.out.float().cpu().numpy().copy(), self.lse.cpu().numpy().copy()


def run_parity(cfg: WorkloadConfig, chunk_tokens: int = 0, check_full: bool = True, check_ring_every: int = 4,
               label: str = "", fuse_epilogue: bool = True, max_gap: int = 0, group_match: bool = False,
               fused_hit_span: int = 0, sm_scale: float = 0.0):
    """All steps of `cfg` on both sides; returns summary dict.  Oracle inputs are host copies of the same bits."""
    say(f"[parity] {label or cfg.name}: batch={cfg.batch} Hq/Hkv={cfg.num_q_heads}/{cfg.num_kv_heads} "
        f"context={cfg.context} steps={cfg.steps} W={cfg.window} B={cfg.band} T={cfg.threshold:.4g} "
        f"page={cfg.page_size} chunk={chunk_tokens} fused={fuse_epilogue} max_gap={max_gap} group_match={group_match} "
        f"fused_hit_span={fused_hit_span} "
        f"seed={cfg.seed}")
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl, chunk_tokens, fuse_epilogue=fuse_epilogue, max_gap=max_gap, group_match=group_match,
                    fused_hit_span=fused_hit_span, sm_scale=sm_scale)
    orc = make_oracle(cfg, wl, max_gap=max_gap, group_match=group_match, **({"sm_scale": sm_scale} if sm_scale > 0 else {}))
    kvp = bf16_bits(wl.kv_pages)
    bt = wl.block_table.cpu().numpy()
    slots = wl.slot_ids.cpu().numpy()
    worst_abs = worst_rel = 0.0
    hits = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        lens = kv_lens.cpu().numpy()
        if check_full:
            g_out, g_lse = run.full(q_rope, kv_lens)
            o_out, o_lse = orc.full_decode(lens, bf16_bits(q_rope), kvp, bt)
            a, r = check_rows(g_out, o_out, f"step {s} full_decode")
            worst_abs, worst_rel = max(worst_abs, a), max(worst_rel, r)
            assert np.abs(g_lse - o_lse).max() < 1e-3, f"step {s} full_decode lse"
        g_out, g_lse, g_pos, g_d2 = run.mac_step(q_pre, q_rope, kv_lens)
        ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert np.array_equal(g_pos, ref["match_pos"]), (
            f"step {s}: match decisions differ at {np.argwhere(g_pos != ref['match_pos'])[:4].tolist()}")
        fin = np.isfinite(ref["d2"])
        assert np.array_equal(np.isfinite(g_d2), fin), f"step {s}: d2 finiteness"
        assert np.allclose(g_d2[fin], ref["d2"][fin], rtol=1e-13, atol=0), f"step {s}: d2 values"
        a, r = check_rows(g_out, ref["out"], f"step {s} decode_step")
        worst_abs, worst_rel = max(worst_abs, a), max(worst_rel, r)
        assert np.abs(g_lse - ref["lse"]).max() < 1e-3, f"step {s} decode_step lse"
        hits += int((g_pos >= 0).sum())
        if check_ring_every and s % check_ring_every == 0:
            for b in range(cfg.batch):
                n = int(lens[b])
                j = (n - 1) % cfg.window
                for h in {0, cfg.num_q_heads - 1}:
                    q, o, l, n_p = run.mac.ring_peek(int(slots[b]), j, h)
                    assert n_p == n and np.array_equal(q, bf16_bits(q_pre)[b, h]), f"step {s}: ring entry tag/query"
                    check_rows(o[None], ref["rect_O"][b, h][None], f"step {s} ring summary b{b} h{h}")
                    rl = ref["rect_lse"][b, h]
                    assert (l == rl) if np.isinf(rl) else abs(l - rl) < 1e-3, f"step {s}: ring lse"
    gst = run.mac.stats()
    ost = orc.stats.as_dict()
    for k in ("steps", "head_steps", "hits", "misses", "sum_gap", "kv_tokens_read", "kv_tokens_full"):
        assert gst[k] == ost[k], f"stats.{k}: gpu {gst[k]} oracle {ost[k]}"
    assert abs(gst["sum_skip_frac"] - ost["sum_skip_frac"]) <= 1e-9 * max(1.0, ost["sum_skip_frac"])
    # where the work went: heads finished by the matcher read their own range; the split-K kernel never streams more
    # than the method's per-group figure, and exactly that when the matcher finishes nothing
    assert gst["kv_tokens_split"] <= gst["kv_tokens_read"]
    if group_match or fused_hit_span < 0:
        assert gst["kv_tokens_fused"] == 0 and gst["kv_tokens_split"] == gst["kv_tokens_read"]
    run.mac.close()
    say(f"[parity] ok: hits {hits}/{ost['head_steps']} worst max-abs {worst_abs:.2e} rel-L2 {worst_rel:.2e} "
        f"kv read {ost['kv_tokens_read']}/{ost['kv_tokens_full']}")
    return {"hits": hits, "head_steps": ost["head_steps"], "max_abs": worst_abs, "rel_l2": worst_rel,
            "kv_tokens_fused": gst["kv_tokens_fused"], "kv_tokens_split": gst["kv_tokens_split"]}
