"""Seeded synthetic decode workloads (inputs only).

This module plays "the model" around the decode-attention operator: it produces
the paged bf16 KV cache, the block tables, and per step the pre-RoPE query, the
post-RoPE query and the sequence lengths.  It contains none of the operator's
arithmetic (no matching, no softmax, no merging); both the CPU oracle's tests
and the HIP path's tests/benchmarks draw their inputs from here.

Shapes follow the paper's evaluation geometry (Llama-3.1-8B attention: 32 query
heads sharing 8 KV heads, head_dim 128, Sec. 5 and Sec. 5.2 "Setup and metric";
contexts up to 120K+, Sec. 5.1; 16K-token continuous generation).  Value
distributions are synthetic stand-ins for the public suites the paper measures
on: K, V iid N(0,1); pre-RoPE queries follow an AR(1) process per (request,
head) so that consecutive queries are close in pre-RoPE L2 distance, which is
the temporal redundancy the method exploits (Sec. 2 "Exploiting temporal
redundancy").

Everything is generated with torch on the requested device (CPU for the small
parity cases, the GPU for the full-size ones, from where the bits are copied to
the host for the oracle), so both sides always see identical bf16 bit patterns.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Iterator, Optional, Tuple

import torch


@dataclasses.dataclass(frozen=True)
class WorkloadConfig:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    context: int            # tokens already in the cache before the first decode step
    steps: int              # decode steps; step s runs at kv_len = context + s + 1
    window: int             # W: query-ring capacity (paper's K)
    band: int               # B: rectification band (paper's r)
    threshold: float        # T: absolute pre-RoPE L2 distance; hit iff d^2 < T^2
    rho: float              # AR(1) coefficient of the pre-RoPE query process
    head_dim: int = 128
    page_size: int = 16
    seed: int = 0
    rope_theta: float = 1.0e4
    regime_shift_every: int = 0     # >0: add a fresh random mean every this many steps
    use_rope: bool = True
    ragged: int = 0                 # >0: request b is `ragged * b` tokens shorter than request 0
    # second query model ("recurring queries"): the pre-RoPE query of head h repeats a random base sequence with
    # period P_h = period + N(0, period_std) (fixed per head) plus per-step noise, so its nearest neighbour in the
    # window lies one period back (reuse gaps of hundreds of tokens with some skew inside a KV group, as the
    # paper's match-position table reports); with probability jump_prob per step a whole KV group gets fresh
    # random queries instead (a miss for the group).  period = 0 selects the AR(1) model above.
    period: int = 0
    period_std: float = 0.0
    query_noise: float = 0.1
    jump_prob: float = 0.0
    # Recency structure for the error-vs-gap report: a random direction u per (request, KV head) is added, with
    # this weight, to every pre-RoPE key of that head and to every pre-RoPE query of its group.  After RoPE the
    # common part contributes align^2 * sum_j |u_j|^2 cos(omega_j (m - t)) / sqrt(d) to the logit of key t under
    # the query at m: largest for the newest keys and decaying with distance, as in a trained model's heads.
    # 0 = off (drawn from a generator of its own, so the other streams do not move).
    align: float = 0.0

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def max_kv_len(self) -> int:
        return self.context + self.steps

    @property
    def pages_per_request(self) -> int:
        return (self.max_kv_len + self.page_size - 1) // self.page_size


_DEFAULT_T = 0.5 * math.sqrt(128.0)

# Thresholds of the long-context sweep: chosen so that the per-head hit rate of
# the AR(1) stream is roughly 20 / 50 / 90 % (nearest neighbour is almost always
# lag 1, whose squared distance is about 2(1-rho) * chi^2_128).  The figures are the
# quantiles measured on the seeded streams themselves by tests/golden/calibrate_thresholds.py
# (stored in tests/golden/c3_thresholds.json), rounded to 3 digits.
C3_THRESHOLDS: Dict[float, float] = {0.90: 4.78, 0.97: 2.76, 0.99: 1.72}

CONFIGS: Dict[str, WorkloadConfig] = {
    # configs[0]: tiny, the oracle finishes it in seconds
    "C1": WorkloadConfig("C1", batch=1, num_q_heads=8, num_kv_heads=2, context=4096, steps=32,
                         window=32, band=64, threshold=_DEFAULT_T, rho=0.95, seed=0),
    # configs[1]: Llama-3-8B-shaped attention at 32K
    "C2": WorkloadConfig("C2", batch=8, num_q_heads=32, num_kv_heads=8, context=32768, steps=256,
                         window=256, band=64, threshold=_DEFAULT_T, rho=0.97, seed=1),
    # configs[2]: long context, 128K, three (rho, threshold) pairs
    "C3_rho90": WorkloadConfig("C3_rho90", batch=4, num_q_heads=32, num_kv_heads=8, context=131072, steps=128,
                               window=256, band=128, threshold=C3_THRESHOLDS[0.90], rho=0.90, seed=2),
    "C3_rho97": WorkloadConfig("C3_rho97", batch=4, num_q_heads=32, num_kv_heads=8, context=131072, steps=128,
                               window=256, band=128, threshold=C3_THRESHOLDS[0.97], rho=0.97, seed=2),
    "C3_rho99": WorkloadConfig("C3_rho99", batch=4, num_q_heads=32, num_kv_heads=8, context=131072, steps=128,
                               window=256, band=128, threshold=C3_THRESHOLDS[0.99], rho=0.99, seed=2),
    # configs[3]: MQA, run A all misses (threshold 0), run B matched threshold
    "C4_miss": WorkloadConfig("C4_miss", batch=16, num_q_heads=32, num_kv_heads=1, context=65536, steps=128,
                              window=128, band=64, threshold=0.0, rho=0.97, seed=3),
    "C4_hit": WorkloadConfig("C4_hit", batch=16, num_q_heads=32, num_kv_heads=1, context=65536, steps=128,
                             window=128, band=64, threshold=_DEFAULT_T, rho=0.97, seed=3),
    # configs[4]: continuous generation with regime shifts
    "C5": WorkloadConfig("C5", batch=32, num_q_heads=64, num_kv_heads=8, context=8192, steps=16384,
                         window=256, band=64, threshold=_DEFAULT_T, rho=0.98, seed=4,
                         regime_shift_every=2048),
}


def scaled(cfg: WorkloadConfig, **overrides) -> WorkloadConfig:
    """A copy of `cfg` with some fields replaced (used for reduced parity cases)."""
    return dataclasses.replace(cfg, **overrides)


def _rope(x: torch.Tensor, pos: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary embedding, half-split pairing (i, i + d/2), fp32.

    x: [..., d] fp32; pos: broadcastable to x.shape[:-1] (integer positions).
    omega_j = theta^(-2j/d), j = 0..d/2-1.
    """
    d = x.shape[-1]
    half = d // 2
    j = torch.arange(half, device=x.device, dtype=torch.float32)
    omega = torch.exp(-(2.0 * j / d) * math.log(theta))
    ang = pos.to(torch.float32).unsqueeze(-1) * omega
    c, s = torch.cos(ang), torch.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


class Workload:
    """Materialised inputs of one config.

    Attributes
    ----------
    kv_pages : bf16 [num_pages, 2, Hkv, page_size, d]   (index 0 = K post-RoPE, 1 = V)
    block_table : int32 [batch, pages_per_request]       physical page of each logical page
    slot_ids : int32 [batch]                             request -> ring set
    strides : (stride_page, stride_kv, stride_head, stride_tok) in elements
    """

    def __init__(self, cfg: WorkloadConfig, device: str | torch.device = "cpu",
                 kv_chunk_tokens: int = 16384, queries_only: bool = False):
        self.cfg = cfg
        self.device = torch.device(device)
        dev = self.device
        g = torch.Generator(device=dev)          # pages, K, V
        g.manual_seed(cfg.seed)
        gq = torch.Generator(device=dev)         # query process (own stream, so queries_only reproduces it)
        gq.manual_seed(cfg.seed + 7919)
        self._gen = gq
        self._u = None
        if cfg.align != 0.0:
            ga = torch.Generator(device=dev)
            ga.manual_seed(cfg.seed + 104729)
            self._u = torch.randn((cfg.batch, cfg.num_kv_heads, cfg.head_dim), generator=ga, device=dev,
                                  dtype=torch.float32)
        d, ps, hkv = cfg.head_dim, cfg.page_size, cfg.num_kv_heads
        ppr = cfg.pages_per_request
        num_pages = cfg.batch * ppr
        # physical page ids: a seeded random permutation of the pool
        perm = torch.randperm(num_pages, generator=g, device=dev).to(torch.int32)
        self.block_table = perm.view(cfg.batch, ppr).contiguous()
        self.slot_ids = torch.arange(cfg.batch, device=dev, dtype=torch.int32)
        self.strides = (2 * hkv * ps * d, hkv * ps * d, ps * d, d)
        self.kv_pages = None
        if not queries_only:
            self.kv_pages = torch.empty((num_pages, 2, hkv, ps, d), dtype=torch.bfloat16, device=dev)
        # fill K (RoPE at its own position) and V, a bounded number of logical pages at a time
        pages_per_chunk = max(1, kv_chunk_tokens // ps)
        for b in range(cfg.batch if not queries_only else 0):
            for p0 in range(0, ppr, pages_per_chunk):
                p1 = min(ppr, p0 + pages_per_chunk)
                ntok = (p1 - p0) * ps
                kt = torch.randn((ntok, hkv, d), generator=g, device=dev, dtype=torch.float32)
                v = torch.randn((ntok, hkv, d), generator=g, device=dev, dtype=torch.float32)
                if self._u is not None:
                    kt = kt + cfg.align * self._u[b].unsqueeze(0)
                if cfg.use_rope:
                    pos = torch.arange(p0 * ps, p1 * ps, device=dev).view(ntok, 1)
                    kt = _rope(kt, pos, cfg.rope_theta)
                phys = self.block_table[b, p0:p1].long()
                # [ntok, hkv, d] -> [pages, hkv, ps, d]
                kp = kt.view(p1 - p0, ps, hkv, d).permute(0, 2, 1, 3).to(torch.bfloat16)
                vp = v.view(p1 - p0, ps, hkv, d).permute(0, 2, 1, 3).to(torch.bfloat16)
                self.kv_pages[phys, 0] = kp
                self.kv_pages[phys, 1] = vp
        # AR(1) state of the pre-RoPE query process, fp32, never rounded
        self._x = torch.randn((cfg.batch, cfg.num_q_heads, d), generator=gq, device=dev, dtype=torch.float32)
        self._mu = torch.zeros_like(self._x)
        self._step = 0
        if cfg.period > 0:
            pmax = int(cfg.period + 4 * cfg.period_std) + 1
            offs = torch.round(cfg.period_std * torch.randn((cfg.batch, cfg.num_q_heads), generator=gq, device=dev))
            self._period = torch.clamp(cfg.period + offs, 2, pmax).to(torch.int64)           # [batch, Hq]
            self._base = torch.randn((cfg.batch, cfg.num_q_heads, pmax, d), generator=gq, device=dev,
                                     dtype=torch.float32)

    # ------------------------------------------------------------------ queries
    def next_step(self) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        """Inputs of the next decode step: (q_pre bf16 [batch,Hq,d], q_rope bf16 [batch,Hq,d],
        kv_lens int32 [batch]).  kv_len counts the current token, whose K/V are already
        in the cache (all steps' K/V are pre-generated; "append" is kv_len += 1)."""
        cfg = self.cfg
        s = self._step
        if s >= cfg.steps:
            raise StopIteration
        if cfg.period > 0:
            noise = torch.randn(self._x.shape, generator=self._gen, device=self.device, dtype=torch.float32)
            phase = (s % self._period).view(cfg.batch, cfg.num_q_heads, 1, 1).expand(-1, -1, 1, cfg.head_dim)
            x = torch.gather(self._base, 2, phase).squeeze(2) + cfg.query_noise * noise
            if cfg.jump_prob > 0:
                u = torch.rand((cfg.batch, cfg.num_kv_heads), generator=self._gen, device=self.device)
                fresh = torch.randn(self._x.shape, generator=self._gen, device=self.device, dtype=torch.float32)
                jump = (u < cfg.jump_prob).repeat_interleave(cfg.group, dim=1).unsqueeze(-1)
                x = torch.where(jump, fresh, x)
        else:
            if s > 0:
                noise = torch.randn(self._x.shape, generator=self._gen, device=self.device, dtype=torch.float32)
                self._x = cfg.rho * self._x + math.sqrt(1.0 - cfg.rho * cfg.rho) * noise
            if cfg.regime_shift_every > 0 and s % cfg.regime_shift_every == 0:
                self._mu = torch.randn(self._x.shape, generator=self._gen, device=self.device, dtype=torch.float32)
            x = self._x + self._mu if cfg.regime_shift_every > 0 else self._x
        if self._u is not None:
            x = x + cfg.align * self._u.repeat_interleave(cfg.group, dim=1)
        n = cfg.context + s + 1
        kv_lens = torch.full((cfg.batch,), n, device=self.device, dtype=torch.int32)
        if cfg.ragged > 0:
            kv_lens = torch.clamp(kv_lens - cfg.ragged * torch.arange(cfg.batch, device=self.device, dtype=torch.int32), min=1)
        q_pre = x.to(torch.bfloat16)
        if cfg.use_rope:
            pos = (kv_lens - 1).view(cfg.batch, 1).expand(cfg.batch, cfg.num_q_heads)
            q_rope = _rope(x, pos, cfg.rope_theta).to(torch.bfloat16)
        else:
            q_rope = q_pre.clone()
        self._step += 1
        return q_pre, q_rope, kv_lens

    def __iter__(self) -> Iterator[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]]:
        while self._step < self.cfg.steps:
            yield self.next_step()


def bf16_bits(t: torch.Tensor):
    """bf16 tensor -> numpy uint16 array of the same shape holding the raw bit patterns (host copy)."""
    import numpy as np
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
