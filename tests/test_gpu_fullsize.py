"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (default chunking).

The fp64 oracle runs EVERY (request, head) of these configs on every step of the shortened runs below (a full-length
step of the 128K config costs it a few tenths of a second on the machine's host cores): decisions, matched distances,
outputs, LSE and the counters of all heads are compared at every step, full decode of all heads on every fourth
step, and the appended ring entries on sampled heads.  Only the 16384-step run of the continuous-generation config
samples: two KV groups are followed through every step, and the decisions of all heads are checked on every 64th step
and around every regime shift.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2604_00235_amd.workload import CONFIGS, Workload, WorkloadConfig, bf16_bits, scaled

pytestmark = pytest.mark.gpu


def _group_oracle(cfg: WorkloadConfig, kvp_g: np.ndarray, **variant):
    from oracle.mac_oracle import Oracle
    ps, d = cfg.page_size, cfg.head_dim
    return Oracle(num_q_heads=cfg.group, num_kv_heads=1, head_dim=d, page_size=ps, window=cfg.window,
                  band=cfg.band, threshold=cfg.threshold, strides=(2 * ps * d, ps * d, ps * d, d), max_slots=1, **variant)


def run_fullsize(cfg: WorkloadConfig, steps: int, full_every: int = 4, **variant):
    """`steps` decode steps of `cfg` from empty rings on both sides, all heads compared at every step."""
    import time
    from tests.gpu_harness import DeviceRun, check_rows, say
    from tests.helpers import make_oracle
    say(f"[fullsize] {cfg.name}: batch={cfg.batch} Hq/Hkv={cfg.num_q_heads}/{cfg.num_kv_heads} context={cfg.context} "
        f"steps={steps} W={cfg.window} B={cfg.band} T={cfg.threshold:.4g} ragged={cfg.ragged} {variant}")
    cfg = scaled(cfg, steps=steps)
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl, **variant)            # default chunk_tokens, as bench.py
    kvp = bf16_bits(wl.kv_pages)
    bt = wl.block_table.cpu().numpy()
    slots = wl.slot_ids.cpu().numpy()
    orc = make_oracle(cfg, wl, **variant)
    worst = 0.0
    hits = 0
    t_orc = 0.0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        lens = kv_lens.cpu().numpy()
        qp, qr = bf16_bits(q_pre), bf16_bits(q_rope)
        f_lse = None
        if s % full_every == 0:                      # full decode, every head
            f_out, f_lse = run.full(q_rope, kv_lens)
            t0 = time.time()
            o_out, o_lse = orc.full_decode(lens, qr, kvp, bt)
            t_orc += time.time() - t0
            a, r = check_rows(f_out, o_out, f"{cfg.name} step {s} full_decode")
            worst = max(worst, r)
            assert np.abs(f_lse - o_lse).max() < 1e-3, f"{cfg.name} step {s} full_decode lse"
        g_out, g_lse, g_pos, g_d2 = run.mac_step(q_pre, q_rope, kv_lens)
        t0 = time.time()
        ref = orc.mac_step(slots, lens, qp, qr, kvp, bt)
        t_orc += time.time() - t0
        assert np.array_equal(g_pos, ref["match_pos"]), (
            f"{cfg.name} step {s}: decisions differ at {np.argwhere(g_pos != ref['match_pos'])[:4].tolist()}")
        fin = np.isfinite(ref["d2"])
        assert np.array_equal(np.isfinite(g_d2), fin) and np.allclose(g_d2[fin], ref["d2"][fin], rtol=1e-13, atol=0)
        a, r = check_rows(g_out, ref["out"], f"{cfg.name} step {s} decode_step")
        worst = max(worst, r)
        assert np.abs(g_lse - ref["lse"]).max() < 1e-3, f"{cfg.name} step {s} decode_step lse"
        hits += int((g_pos >= 0).sum())
        if f_lse is not None:                        # on a miss the MAC output is full attention of the same step
            miss = g_pos < 0
            assert np.abs(g_lse[miss] - f_lse[miss]).max(initial=0.0) < 1e-4
        for b in {0, cfg.batch - 1}:                 # the entry this step appended, on sampled heads
            n = int(lens[b])
            for h in {0, cfg.num_q_heads // 2, cfg.num_q_heads - 1}:
                q, o, l, n_p = run.mac.ring_peek(int(slots[b]), (n - 1) % cfg.window, h)
                assert n_p == n and np.array_equal(q, qp[b, h]), f"{cfg.name} step {s}: ring entry tag/query"
                check_rows(o[None], ref["rect_O"][b, h][None], f"{cfg.name} step {s} ring summary b{b} h{h}")
                rl = ref["rect_lse"][b, h]
                assert (l == rl) if np.isinf(rl) else abs(l - rl) < 1e-3
    st = run.mac.stats()
    ost = orc.stats.as_dict()
    for k in ("steps", "head_steps", "hits", "misses", "sum_gap", "kv_tokens_read", "kv_tokens_full"):
        assert st[k] == ost[k], f"stats.{k}: gpu {st[k]} oracle {ost[k]}"
    assert st["steps"] == steps and st["hits"] == hits
    run.mac.close()
    say(f"[fullsize] ok: hits {hits}/{st['head_steps']}, worst rel-L2 {worst:.2e}, "
        f"kv read {st['kv_tokens_read']}/{st['kv_tokens_full']}, oracle {t_orc:.1f} s")
    return hits, st


def test_c2_llama_32k_full_size():
    hits, st = run_fullsize(CONFIGS["C2"], steps=12)
    assert hits == st["head_steps"] - 8 * 32          # every step after the first hits


def test_c2_ragged_lengths_mixed_hits():
    """C2 geometry with request lengths 32768, 29767, ..., 11761 (not multiples of anything) and a threshold near
    the lag-1 distance, so that groups with and without a miss, and slots past the end of short requests, mix."""
    cfg = scaled(CONFIGS["C2"], ragged=3001, threshold=2.8)
    hits, st = run_fullsize(cfg, steps=10)
    assert 0 < hits < st["head_steps"]


@pytest.mark.parametrize("name", ["C3_rho90", "C3_rho97", "C3_rho99"])
def test_c3_long_context_128k_full_size(name):
    hits, st = run_fullsize(CONFIGS[name], steps=10)
    assert 0 < hits < st["head_steps"]


def test_c3_long_context_128k_one_reuse_point_per_group():
    """The headline workload with group-granular matching (the extra leg of bench.py's sweep): a group hits as a
    whole, so about half of the KV reads go away at the threshold that gives 49 % per-head hits."""
    hits, st = run_fullsize(CONFIGS["C3_rho97"], steps=10, group_match=True)
    assert 0 < hits < st["head_steps"] and hits % 4 == 0
    assert st["kv_tokens_read"] < 0.75 * st["kv_tokens_full"]


def test_work_items_at_the_size_cap():
    """128 KV groups of 70000 tokens (4.6 GB of K/V) are more than four work items of the largest size per compute unit:
    the planner then makes more items (in multiples of the compute units) instead of longer ones, and the grid, capped,
    loops.  Step 1 misses everywhere (all groups at full length), step 2 hits."""
    cfg = scaled(CONFIGS["C2"], name="cap", batch=16, context=70000)
    hits, st = run_fullsize(cfg, steps=2, full_every=1)
    assert hits == st["head_steps"] - 16 * 32


@pytest.mark.parametrize("batch,window", [(64, 1024), (32, 2048)])
def test_query_rings_beyond_the_last_level_cache(batch, window):
    """batch x 32 heads x W x 256 B = 537 MB of query rows scanned per step, twice the last-level cache (64 x 32 heads:
    the lean 256-thread build of the matcher; 32 x 32: the plain one).  Short context, a few steps with hits and
    misses, all heads against the oracle."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"bigring{batch}_{window}", batch=batch, num_q_heads=32, num_kv_heads=8, context=150, steps=6,
                         window=window, band=32, threshold=float(np.sqrt(2 * (1 - 0.97) * 128)), rho=0.97, seed=73, ragged=7)
    r = run_parity(cfg, check_full=False, check_ring_every=3)
    assert 0 < r["hits"] < r["head_steps"]


def test_c4_mqa_64k_full_size_all_miss_and_matched():
    hits, st = run_fullsize(CONFIGS["C4_miss"], steps=3, full_every=2)
    assert hits == 0 and st["kv_tokens_read"] == st["kv_tokens_full"]
    hits, st = run_fullsize(CONFIGS["C4_hit"], steps=8)
    assert hits == st["head_steps"] - 16 * 32


def test_c5_continuous_generation_full_batch():
    """C5 geometry and batch as stated (32 x 64/8 heads, prompt 8192); the 16384-step run is cut to 40 steps with
    the regime shift brought forward to every 16 steps so that it is exercised."""
    cfg = scaled(CONFIGS["C5"], regime_shift_every=16)
    hits, st = run_fullsize(cfg, steps=40, full_every=8)
    assert 0 < hits < st["head_steps"]


def test_c5_full_length_16384_steps():
    """BASELINE configs[4] as stated, all 16384 generated steps (context 8192 -> 24576, regime shift every 2048
    steps, the ring of 256 entries wraps 64 times).  Every step runs on the GPU; the oracle follows two sampled KV
    groups through every step (outputs and decisions), and checks the decisions of ALL 2048 heads on every 64th
    step and on the three steps from each regime shift on (its matcher rings are kept up to date at every step)."""
    from oracle.mac_oracle import Oracle
    from tests.gpu_harness import DeviceRun, check_rows, say
    cfg = CONFIGS["C5"]
    say(f"[fullsize] C5 full length: batch={cfg.batch} Hq/Hkv={cfg.num_q_heads}/{cfg.num_kv_heads} steps={cfg.steps}")
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl)
    kvp = bf16_bits(wl.kv_pages)
    bt = wl.block_table.cpu().numpy()
    slots = wl.slot_ids.cpu().numpy()
    G = cfg.group
    morc = Oracle(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, head_dim=cfg.head_dim,
                  page_size=cfg.page_size, window=cfg.window, band=cfg.band, threshold=cfg.threshold,
                  strides=wl.strides, max_slots=cfg.batch)
    groups = [(3, 1), (30, 6)]
    gorc = {}
    for (b, g) in groups:
        kv_g = np.ascontiguousarray(kvp[:, :, g:g + 1])
        gorc[(b, g)] = (_group_oracle(cfg, kv_g), kv_g, bt[b:b + 1].copy())
    hits = checked_all = 0
    worst = 0.0
    miss_steps = set()
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        lens = kv_lens.cpu().numpy()
        qp, qr = bf16_bits(q_pre), bf16_bits(q_rope)
        run.mac.decode_step(run.args(q_pre, q_rope, kv_lens), run.stream)
        torch.cuda.synchronize()
        g_pos = run.pos.cpu().numpy()
        if s % 64 == 0 or s % cfg.regime_shift_every < 3:
            o_pos, _, _ = morc.match(slots, lens, qp)
            assert np.array_equal(g_pos, o_pos), f"step {s}: decisions differ at {np.argwhere(g_pos != o_pos)[:4].tolist()}"
            checked_all += 1
        j = (int(lens[0]) - 1) % cfg.window             # all requests have the same length here
        morc.ring_q[:, j] = qp
        morc.ring_npos[:, j] = lens
        n_hit = int((g_pos >= 0).sum())
        hits += n_hit
        if n_hit < g_pos.size // 2:
            miss_steps.add(s)
        for (b, g), (orc, kv_g, bt_b) in gorc.items():
            hs = slice(g * G, (g + 1) * G)
            ref = orc.mac_step(np.zeros(1, np.int32), lens[b:b + 1], qp[b:b + 1, hs], qr[b:b + 1, hs], kv_g, bt_b)
            assert np.array_equal(ref["match_pos"][0], g_pos[b, hs]), f"step {s} group {(b, g)}"
            a, r = check_rows(run.out[b, hs].cpu().numpy(), ref["out"][0], f"C5 step {s} b{b} g{g}")
            worst = max(worst, r)
        if s % 2048 == 0:
            say(f"[fullsize] C5 step {s}: hits so far {hits}, worst rel-L2 {worst:.2e}")
    st = run.mac.stats()
    assert st["steps"] == cfg.steps and st["hits"] == hits
    # the first step after each regime shift misses everywhere (jump ~ sqrt(2d)); everything else hits
    assert miss_steps == set(range(0, cfg.steps, cfg.regime_shift_every)), sorted(miss_steps)[:12]
    assert hits == (cfg.steps - len(miss_steps)) * cfg.batch * cfg.num_q_heads
    run.mac.close()
    say(f"[fullsize] C5 full length ok: hits {hits}/{st['head_steps']}, all-head decision checks on {checked_all} steps, "
        f"worst rel-L2 {worst:.2e}, KV read {st['kv_tokens_read']}/{st['kv_tokens_full']}")
