"""Seeded random geometries through the whole path against the oracle (GPU).  Each case draws heads, group size,
page size, window, band, chunking, ragged lengths, query model, threshold, head dimension and the variants of the match rule from a
seed; decisions must be bit-exact and outputs within the tolerance at every step."""
from __future__ import annotations

import math

import numpy as np
import pytest

from paper_2604_00235_amd.workload import WorkloadConfig

pytestmark = pytest.mark.gpu


def _draw(seed: int):
    rng = np.random.default_rng(1000 + seed)
    group = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 32]))
    hkv = int(rng.choice([1, 2, 3])) if group >= 8 else int(rng.choice([1, 2, 4, 8]))
    window = int(rng.choice([1, 2, 5, 16, 64, 100, 256, 700]))
    band = int(rng.choice([0, 1, 7, 32, 64, 200]))
    batch = int(rng.integers(1, 4))
    context = int(rng.choice([0, 3, 31, 32, 33, 500, 1023, 1500, 2049]))
    steps = int(rng.integers(8, 40)) if window < 200 else int(rng.integers(40, 90))
    recurring = bool(rng.integers(0, 2))
    kw = dict(name=f"fuzz{seed}", batch=batch, num_q_heads=group * hkv, num_kv_heads=hkv, context=context, steps=steps,
              window=window, band=band, page_size=int(rng.choice([16, 32, 64])), seed=seed,
              ragged=int(rng.choice([0, 1, 17])) if context > 60 else 0)
    if recurring:
        period = int(rng.integers(2, max(3, min(window, 30) + 1)))
        kw.update(rho=0.0, period=period, period_std=float(rng.choice([0.0, 1.0])), query_noise=0.1,
                  jump_prob=float(rng.choice([0.0, 0.1])), threshold=0.5 * math.sqrt(128.0))
    else:
        rho = float(rng.choice([0.9, 0.97, 0.99]))
        # near the lag-1 distance sqrt(2 d (1 - rho)), so that hits and misses mix
        kw.update(rho=rho, threshold=float(math.sqrt(2 * 128 * (1 - rho)) * rng.uniform(0.9, 1.1)))
    variant = dict(max_gap=int(rng.choice([0, 0, 1, 3, 20])), group_match=bool(rng.integers(0, 3) == 0))
    chunk = int(rng.choice([0, 32, 64, 96, 256, 1024]))
    fused = bool(rng.integers(0, 4) != 0)
    # largest fresh range the matcher finishes itself: default, never, and values that split the hits of one run
    variant["fused_hit_span"] = int(rng.choice([0, -1, 9, 40, 100, 2048]))
    # head dimension (drawn last, so that the earlier draws of a seed stay what they were); thresholds scale with sqrt(d)
    head_dim = int(rng.choice([128, 128, 64, 96, 32]))
    kw.update(head_dim=head_dim, threshold=kw["threshold"] * math.sqrt(head_dim / 128.0))
    return WorkloadConfig(**kw), variant, chunk, fused


@pytest.mark.parametrize("seed", list(range(20)))
def test_random_geometry(seed):
    from tests.gpu_harness import run_parity
    cfg, variant, chunk, fused = _draw(seed)
    r = run_parity(cfg, chunk_tokens=chunk, check_full=(seed % 2 == 0), check_ring_every=3, fuse_epilogue=fused, **variant)
    assert r["head_steps"] == cfg.steps * cfg.batch * cfg.num_q_heads


def _draw_wide(seed: int):
    """Larger shapes than _draw: up to 70 requests and 2240 heads (the lean build of the per-head matcher), windows up to
    2048 (its 1024-thread build for few heads), bands up to 600, contexts up to 6000, pages up to 256 tokens."""
    rng = np.random.default_rng(50000 + seed)
    group = int(rng.choice([1, 2, 4, 4, 8, 16, 32]))
    hkv = int(rng.choice([1, 2])) if group >= 16 else int(rng.choice([1, 2, 4, 8]))
    hq = group * hkv
    batch = int(rng.choice([1, 2, 5, 17, 40])) if hq >= 32 else int(rng.choice([1, 3, 9, 33, 70]))
    window = int(rng.choice([3, 33, 64, 257, 300, 1024, 2048]))
    band = int(rng.choice([0, 16, 64, 128, 256, 600]))
    context = int(rng.choice([40, 700, 2100, 6000]))
    steps = int(rng.integers(6, 16))
    recurring = bool(rng.integers(0, 2))
    head_dim = int(rng.choice([128, 128, 64, 96, 32]))
    kw = dict(name=f"wide{seed}", batch=batch, num_q_heads=hq, num_kv_heads=hkv, context=context, steps=steps, window=window,
              band=band, page_size=int(rng.choice([16, 64, 256])), seed=seed,
              ragged=int(rng.choice([0, 29])) if context > 100 else 0, head_dim=head_dim)
    if recurring:
        period = int(rng.integers(2, max(3, min(window, steps - 2) + 1)))
        kw.update(rho=0.0, period=period, period_std=float(rng.choice([0.0, 1.0])), query_noise=0.1,
                  jump_prob=float(rng.choice([0.0, 0.1])), threshold=0.5 * math.sqrt(head_dim))
    else:
        rho = float(rng.choice([0.9, 0.97, 0.99]))
        kw.update(rho=rho, threshold=float(math.sqrt(2 * head_dim * (1 - rho)) * rng.uniform(0.9, 1.1)))
    variant = dict(max_gap=int(rng.choice([0, 0, 2, 20])), group_match=bool(rng.integers(0, 4) == 0),
                   fused_hit_span=int(rng.choice([0, -1, 70, 2048])))
    return WorkloadConfig(**kw), variant, int(rng.choice([0, 0, 64, 512])), bool(rng.integers(0, 4) != 0)


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_geometry_wide(seed):
    from tests.gpu_harness import run_parity
    cfg, variant, chunk, fused = _draw_wide(seed)
    r = run_parity(cfg, chunk_tokens=chunk, check_full=(seed % 3 == 0), check_ring_every=4, fuse_epilogue=fused, **variant)
    assert r["head_steps"] == cfg.steps * cfg.batch * cfg.num_q_heads
