#!/usr/bin/env python3
"""Benchmark of the MAC-Attention decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C3_rho97] [--no-cpu-baseline]

A "step" is one pass of the whole hot path (match -> band+tail / full attention -> merge -> ring write-back)
over one batch of synthetic input, all inputs resident in HBM.  Default workload: BASELINE configs[2], the
128K long-context case (batch 4, 32/8 heads, d 128, paged bf16 KV, page 16, W 256, B 128), with the
(rho = 0.97, ~50 % hit rate) pair as the headline and the other two pairs reported alongside.

Prints ONE JSON line: the metric (decode-attention microseconds per step), achieved HBM GB/s of the dominant
kernel against the 8 TB/s roofline, hit rate, KV-bytes-read reduction, speed-up over our own full-attention
decode kernel, and the CPU oracle timed on the host cores on a bounded sample (baseline only).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
KV_BYTES_PER_TOKEN_HEAD = 512   # K row + V row, bf16, d = 128
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attn_kernel_hbm_traffic_ratios.txt")


def traffic_ratios():
    """(config, mode) -> measured HBM traffic / algorithmic bytes of the attention kernel, from the tracked rocprofv3
    --pmc summary (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size; lines `ratio <config> <mode>
    <value>`).  The counters cannot be read from inside this process, so the line reports traffic = ratio x the
    algorithmic bytes of this run, names the file, and reports null for a config that was never profiled."""
    out = {}
    try:
        for ln in open(TRAFFIC_FILE):
            f = ln.split()
            if len(f) == 4 and f[0] == "ratio":
                out[(f[1], f[2])] = float(f[3])
    except OSError:
        pass
    return out


def log(msg: str):
    print(msg, file=sys.stderr, flush=True)


def run_config(name: str, steps: int, warmup: int, torch, mb, wl_mod, keep_kv=None, use_graph=False, group_match=False):
    """Timed MAC steps + timed full-decode steps + per-kernel timing pass for one config.
    Returns (result dict, workload) -- the workload's KV cache is reused by the next config of the sweep."""
    cfg = wl_mod.CONFIGS[name]
    if warmup + 2 * steps > cfg.steps:       # more decode steps asked for than the config states: same workload, run longer
        cfg = wl_mod.scaled(cfg, steps=warmup + 2 * steps)
    t0 = time.time()
    if keep_kv is not None:
        wl = wl_mod.Workload(cfg, device="cuda:0", queries_only=True)
        wl.kv_pages, wl.block_table = keep_kv.kv_pages, keep_kv.block_table
    else:
        wl = wl_mod.Workload(cfg, device="cuda:0")
    torch.cuda.synchronize()
    log(f"[bench] {name}: workload ready in {time.time() - t0:.1f}s "
        f"(KV {wl.kv_pages.numel() * 2 / 1e9:.2f} GB resident in HBM)")
    mac = mb.MacAttention(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, window=cfg.window,
                          band=cfg.band, threshold=cfg.threshold, max_kv_len=cfg.max_kv_len,
                          max_slots=cfg.batch, page_size=cfg.page_size, group_match=group_match)
    B, Hq, d = cfg.batch, cfg.num_q_heads, cfg.head_dim
    out = torch.zeros((B, Hq, d), dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    # all step inputs are generated before the timed regions
    inputs = [wl.next_step() for _ in range(warmup + 2 * steps)]
    args = [mac.make_args(kv_lens=kl, q_rope=qr, kv_pages=wl.kv_pages, strides=wl.strides,
                          block_table=wl.block_table, out=out, slot_ids=wl.slot_ids, q_pre=qp)
            for (qp, qr, kl) in inputs]
    torch.cuda.synchronize()

    # --- warm-up (also fills the rings), then EXACTLY `steps` timed MAC steps
    for a in args[:warmup]:
        mac.decode_step(a, stream)
    torch.cuda.synchronize()
    mac.stats(reset=True)
    t0 = time.perf_counter()
    for a in args[warmup:warmup + steps]:
        mac.decode_step(a, stream)
    torch.cuda.synchronize()
    mac_s = time.perf_counter() - t0
    st = mac.stats(reset=True)

    # --- our own full-attention decode on the same steps' inputs (baseline of the speed-up)
    for a in args[warmup:warmup + 2]:
        mac.full_decode(a, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a in args[warmup:warmup + steps]:
        mac.full_decode(a, stream)
    torch.cuda.synchronize()
    full_s = time.perf_counter() - t0

    # --- per-kernel durations with HIP events on the launch stream: next `steps` MAC steps, then full decode
    mb.mac_attn_set_timing(mac.ctx, True)
    for a in args[warmup + steps:warmup + 2 * steps]:
        mac.decode_step(a, stream)
    k_us, k_n = mb.mac_attn_kernel_us(mac.ctx)
    st2 = mac.stats(reset=True)
    for a in args[warmup + steps:warmup + 2 * steps]:
        mac.full_decode(a, stream)
    f_us, f_n = mb.mac_attn_kernel_us(mac.ctx)
    mb.mac_attn_set_timing(mac.ctx, False)

    # --- the same MAC steps replayed from ONE captured HIP graph.  The graph holds the whole step: three small device
    # kernels that fetch step i's inputs from tensors preloaded with all steps (index_select by a device-side step
    # counter, which the graph also advances) and the library's launches, so a replay needs no host work but
    # hipGraphLaunch.  The eager figure beside it runs exactly the same device work launch by launch.
    graph_us = eager_same_us = None
    if use_graph:
        n_g = warmup + steps
        all_qp = torch.stack([i[0] for i in inputs[:n_g]])
        all_qr = torch.stack([i[1] for i in inputs[:n_g]])
        all_kl = torch.stack([i[2] for i in inputs[:n_g]])
        qp_s, qr_s, kl_s = (t.clone() for t in inputs[0])
        idx = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        g_args = mac.make_args(kv_lens=kl_s, q_rope=qr_s, kv_pages=wl.kv_pages, strides=wl.strides,
                               block_table=wl.block_table, out=out, slot_ids=wl.slot_ids, q_pre=qp_s)

        def one_step(hs):
            torch.index_select(all_qp, 0, idx, out=qp_s.unsqueeze(0))
            torch.index_select(all_qr, 0, idx, out=qr_s.unsqueeze(0))
            torch.index_select(all_kl, 0, idx, out=kl_s.unsqueeze(0))
            mac.decode_step(g_args, hs)
            idx.add_(1)

        side = torch.cuda.Stream()
        for mode in ("eager", "graph"):
            mac.reset()
            idx.zero_()
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                hs = side.cuda_stream
                for _ in range(warmup):
                    one_step(hs)
                side.synchronize()
                if mode == "eager":
                    t0 = time.perf_counter()
                    for _ in range(steps):
                        one_step(hs)
                    side.synchronize()
                    eager_same_us = 1e6 * (time.perf_counter() - t0) / steps
            if mode == "graph":
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    one_step(torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                mac.stats(reset=True)
                t0 = time.perf_counter()
                for _ in range(steps):
                    g.replay()
                torch.cuda.synchronize()
                graph_us = 1e6 * (time.perf_counter() - t0) / steps
                st_g = mac.stats(reset=True)
                assert st_g["steps"] == steps, st_g        # capture ran nothing, every replay ran one step
                del g
        log(f"[bench] {name}: one captured graph per step {graph_us:.1f} us/step; the same device work launched "
            f"eagerly {eager_same_us:.1f} us/step")
    mac.close()

    n_mid = cfg.context + warmup + steps // 2
    full_tokens = B * cfg.num_kv_heads * sum(int(kl[0]) for (_, _, kl) in inputs[warmup + steps:warmup + 2 * steps])
    res = {
        "config": name, "rho": cfg.rho, "threshold": cfg.threshold,
        "us_per_step": 1e6 * mac_s / steps,
        "full_decode_us_per_step": 1e6 * full_s / steps,
        "speedup_vs_full": full_s / mac_s,
        "hit_rate": st["hits"] / max(1, st["head_steps"]),
        "mean_gap": st["sum_gap"] / max(1, st["hits"]),
        "skip_ratio": st["sum_skip_frac"] / max(1, st["head_steps"]),
        "kv_read_reduction_pct": 100.0 * (1.0 - st["kv_tokens_read"] / max(1, st["kv_tokens_full"])),
        "kernel_us": {"match": k_us[0] / k_n, "attention": k_us[1] / k_n, "merge": k_us[2] / k_n,
                      "writeback": k_us[3] / k_n},
        "full_kernel_us": {"attention": f_us[1] / f_n, "merge": f_us[2] / f_n},
        # algorithmic bytes of the split-K attention kernel per launch: K+V rows it streamed (per KV group, from the
        # smallest start among the heads the match kernel did not finish itself), from the library's own counters
        # over the event-timed steps; what the match kernel's hit path read per head is reported beside it
        "attn_bytes_per_launch": KV_BYTES_PER_TOKEN_HEAD * st2["kv_tokens_split"] / k_n,
        "fused_kv_bytes_per_step": KV_BYTES_PER_TOKEN_HEAD * st2["kv_tokens_fused"] / k_n,
        "full_attn_bytes_per_launch": KV_BYTES_PER_TOKEN_HEAD * full_tokens / f_n,
        "kv_len_mid": n_mid,
        "graph_us_per_step": graph_us, "eager_same_work_us_per_step": eager_same_us,
    }
    res["attn_GBps"] = res["attn_bytes_per_launch"] / (res["kernel_us"]["attention"] * 1e-6) / 1e9
    res["full_attn_GBps"] = res["full_attn_bytes_per_launch"] / (res["full_kernel_us"]["attention"] * 1e-6) / 1e9
    res["effective_GBps"] = res["full_attn_bytes_per_launch"] / (res["us_per_step"] * 1e-6) / 1e9
    log(f"[bench] {name}: MAC {res['us_per_step']:.1f} us/step, full {res['full_decode_us_per_step']:.1f} us/step, "
        f"hit {100 * res['hit_rate']:.1f}%, KV-read reduction {res['kv_read_reduction_pct']:.1f}%, "
        f"attention kernel {res['kernel_us']['attention']:.1f} us @ {res['attn_GBps']:.0f} GB/s "
        f"(full: {res['full_kernel_us']['attention']:.1f} us @ {res['full_attn_GBps']:.0f} GB/s)")
    return res, wl


def paper_table(torch, mb, wl_mod, steps: int = 200):
    """Our analogue of the paper's fine-grained latency table (Sec. 5.6: Match / Load-balance / Attention / Overall
    at 32K / 60K / 120K context and KV budgets 1 / 5 / 10 / 20 %, window K = 1024, band r = 256): one request of
    Llama-3.1-8B geometry, recurring queries with a reuse gap of ~400 tokens and some skew inside a KV group, and
    a per-step probability of a whole-group miss chosen to land on the KV budget.  Context, not target: the paper's
    figures are from an H100 with an unstated batch."""
    rows = []
    period, pstd, W, B = 400, 30.0, 1024, 256
    warm = period + int(4 * pstd) + 16
    for ctx in (32768, 61440, 122880):
        kv = None
        for budget in (1, 5, 10, 20):
            # a jump makes its KV group miss at that step and, one period later, once per head of the group
            # (its 4 heads have different periods): 5 full reads per jump
            base = (period + B) / ctx
            f = max(0.0, (budget / 100.0 - base) / (1.0 - base))
            cfg = wl_mod.WorkloadConfig(name=f"T_{ctx}_{budget}", batch=1, num_q_heads=32, num_kv_heads=8, context=ctx,
                                        steps=warm + 2 * steps, window=W, band=B, threshold=0.5 * 128 ** 0.5, rho=0.0,
                                        seed=7, period=period, period_std=pstd, query_noise=0.1, jump_prob=f / 5)
            if kv is None:
                wl = wl_mod.Workload(cfg, device="cuda:0")
                kv = wl
            else:
                wl = wl_mod.Workload(cfg, device="cuda:0", queries_only=True)
                wl.kv_pages, wl.block_table = kv.kv_pages, kv.block_table
            mac = mb.MacAttention(num_q_heads=32, num_kv_heads=8, window=W, band=B, threshold=cfg.threshold,
                                  max_kv_len=cfg.max_kv_len, max_slots=1)
            out = torch.zeros((1, 32, 128), dtype=torch.float32, device="cuda:0")
            stream = torch.cuda.current_stream().cuda_stream
            inputs = [wl.next_step() for _ in range(cfg.steps)]
            args = [mac.make_args(kv_lens=kl, q_rope=qr, kv_pages=wl.kv_pages, strides=wl.strides,
                                  block_table=wl.block_table, out=out, slot_ids=wl.slot_ids, q_pre=qp)
                    for (qp, qr, kl) in inputs]
            for a in args[:warm]:
                mac.decode_step(a, stream)
            torch.cuda.synchronize()
            mac.stats(reset=True)
            t0 = time.perf_counter()
            for a in args[warm:warm + steps]:
                mac.decode_step(a, stream)
            torch.cuda.synchronize()
            mac_us = 1e6 * (time.perf_counter() - t0) / steps
            st = mac.stats(reset=True)
            t0 = time.perf_counter()
            for a in args[warm:warm + steps]:
                mac.full_decode(a, stream)
            torch.cuda.synchronize()
            full_us = 1e6 * (time.perf_counter() - t0) / steps
            mb.mac_attn_set_timing(mac.ctx, True)
            for a in args[warm + steps:warm + 2 * steps]:
                mac.decode_step(a, stream)
            k_us, k_n = mb.mac_attn_kernel_us(mac.ctx)
            mac.close()
            row = {"context": ctx, "kv_budget_pct": budget,
                   "kv_read_pct": round(100.0 * st["kv_tokens_read"] / max(1, st["kv_tokens_full"]), 2),
                   "hit_rate": round(st["hits"] / max(1, st["head_steps"]), 4),
                   "mean_gap": round(st["sum_gap"] / max(1, st["hits"]), 1),
                   "full_us": round(full_us, 1), "match_us": round(k_us[0] / k_n, 1),
                   "attention_us": round(k_us[1] / k_n, 1), "merge_writeback_us": round(k_us[2] / k_n, 1),
                   "overall_us": round(mac_us, 1), "speedup": round(full_us / mac_us, 2)}
            rows.append(row)
            log(f"[table] ctx {ctx:6d} KV {budget:2d}% (read {row['kv_read_pct']:5.2f}%, hit {100 * row['hit_rate']:5.1f}%, "
                f"gap {row['mean_gap']:5.0f}): full {row['full_us']:6.1f} | match {row['match_us']:5.1f} attn "
                f"{row['attention_us']:6.1f} merge+wb {row['merge_writeback_us']:5.1f} | overall {row['overall_us']:6.1f} us "
                f"({row['speedup']:.2f}x)")
        del kv
        torch.cuda.empty_cache()
    return rows


def match_table(torch, mb, wl_mod, timed: int = 40):
    """Our analogue of the paper's kernel micro-benchmark (Sec. 5.7, kernel-breakdown figure, panel a): the Match
    kernel over a window of L queries against the full-attention kernel over L keys, for GQA 8-2, 32-8 and 40-10 and
    L = 512, 1024, 2048.  The paper does not state the batch; batch 1 (latency-bound on this chip) and batch 32 are
    reported.  Threshold 0, so every step misses and attention streams all L keys; the window is full (L steps run
    first from an empty context)."""
    rows = []
    for batch in (1, 32):
        for hq, hkv in ((8, 2), (32, 8), (40, 10)):
            for L in (512, 1024, 2048):
                cfg = wl_mod.WorkloadConfig(name=f"M_{hq}_{hkv}_{L}", batch=batch, num_q_heads=hq, num_kv_heads=hkv,
                                            context=0, steps=L + timed, window=L, band=64, threshold=0.0, rho=0.97, seed=11)
                wl = wl_mod.Workload(cfg, device="cuda:0")
                mac = mb.MacAttention(num_q_heads=hq, num_kv_heads=hkv, window=L, band=64, threshold=0.0,
                                      max_kv_len=cfg.max_kv_len, max_slots=batch)
                out = torch.zeros((batch, hq, 128), dtype=torch.float32, device="cuda:0")
                stream = torch.cuda.current_stream().cuda_stream
                inputs = [wl.next_step() for _ in range(cfg.steps)]
                args = [mac.make_args(kv_lens=kl, q_rope=qr, kv_pages=wl.kv_pages, strides=wl.strides,
                                      block_table=wl.block_table, out=out, slot_ids=wl.slot_ids, q_pre=qp)
                        for (qp, qr, kl) in inputs]
                for a in args[:L]:
                    mac.decode_step(a, stream)
                torch.cuda.synchronize()
                mb.mac_attn_set_timing(mac.ctx, True)
                for a in args[L:]:
                    mac.decode_step(a, stream)
                k_us, k_n = mb.mac_attn_kernel_us(mac.ctx)
                mac.close()
                ring_mb = batch * hq * L * 256 / 1e6
                kv_mb = batch * hkv * (L + timed // 2) * 512 / 1e6
                row = {"batch": batch, "gqa": f"{hq}-{hkv}", "tokens": L, "match_us": round(k_us[0] / k_n, 2),
                       "attention_us": round(k_us[1] / k_n, 2), "match_over_attention": round(k_us[0] / k_us[1], 2),
                       "ring_MB": round(ring_mb, 2), "kv_MB": round(kv_mb, 2)}
                rows.append(row)
                log(f"[match-table] batch {batch:2d} GQA {row['gqa']:>5s} L {L:4d}: match {row['match_us']:6.2f} us "
                    f"({ring_mb:6.1f} MB)  attention {row['attention_us']:6.2f} us ({kv_mb:6.1f} MB)  ratio "
                    f"{row['match_over_attention']:.2f}")
                del wl
    torch.cuda.empty_cache()
    return rows


def balance_table(torch, mb, wl_mod, steps: int = 100):
    """Our analogue of the paper's load-balancing study (Sec. 5.7, kernel-breakdown figure, panel b: contexts 32K / 64K /
    128K x reuse skew 0.1 / 0.2 / 0.3, planner against a naive assignment and a perfect schedule).  Eight requests of
    Llama-3.1-8B geometry (64 KV groups), recurring queries (reuse gap ~400, K = 1024, r = 256); "skew" here is the
    share of KV groups that miss in a step and stream their whole context while the others stream ~650 tokens.  Three
    schedules for the split-K attention kernel on the same steps: work items sized on the device from the step's
    real span (the default), work items of a fixed 2048 tokens dealt to the work-groups in turn (what a host that only
    knows max_kv_len can do), and the time the bytes the step streams would take at the rate the same kernel reaches
    on a uniform full stream of the same cache (measured beside it)."""
    rows = []
    period, pstd, W, B, batch = 400, 30.0, 1024, 256, 8
    warm = period + int(4 * pstd) + 16
    for ctx in (32768, 65536, 131072):
        kv = None
        for skew in (0.1, 0.2, 0.3):
            # a jump makes its KV group miss at that step and, one period later, once per head of the group: 5 per jump
            cfg = wl_mod.WorkloadConfig(name=f"L_{ctx}_{skew}", batch=batch, num_q_heads=32, num_kv_heads=8, context=ctx,
                                        steps=warm + steps, window=W, band=B, threshold=0.5 * 128 ** 0.5, rho=0.0,
                                        seed=17, period=period, period_std=pstd, query_noise=0.1, jump_prob=skew / 5)
            if kv is None:
                wl = wl_mod.Workload(cfg, device="cuda:0")
                kv = wl
            else:
                wl = wl_mod.Workload(cfg, device="cuda:0", queries_only=True)
                wl.kv_pages, wl.block_table = kv.kv_pages, kv.block_table
            inputs = [wl.next_step() for _ in range(cfg.steps)]
            out = torch.zeros((batch, 32, 128), dtype=torch.float32, device="cuda:0")
            stream = torch.cuda.current_stream().cuda_stream
            res = {}
            for label, chunk in (("planner", 0), ("fixed", 2048)):
                mac = mb.MacAttention(num_q_heads=32, num_kv_heads=8, window=W, band=B, threshold=cfg.threshold,
                                      max_kv_len=cfg.max_kv_len, max_slots=batch, chunk_tokens=chunk)
                args = [mac.make_args(kv_lens=kl, q_rope=qr, kv_pages=wl.kv_pages, strides=wl.strides,
                                      block_table=wl.block_table, out=out, slot_ids=wl.slot_ids, q_pre=qp)
                        for (qp, qr, kl) in inputs]
                for a in args[:warm]:
                    mac.decode_step(a, stream)
                torch.cuda.synchronize()
                mac.stats(reset=True)
                mb.mac_attn_set_timing(mac.ctx, True)
                for a in args[warm:]:
                    mac.decode_step(a, stream)
                k_us, k_n = mb.mac_attn_kernel_us(mac.ctx)
                st = mac.stats(reset=True)
                res[label] = (k_us[1] / k_n, st)
                if label == "planner":          # the uniform full stream of the same cache, same kernel
                    for a in args[warm:warm + 20]:
                        mac.full_decode(a, stream)
                    f_us, f_n = mb.mac_attn_kernel_us(mac.ctx)
                    full_us = f_us[1] / f_n
                mb.mac_attn_set_timing(mac.ctx, False)
                mac.close()
            st = res["planner"][1]
            split_tok = st["kv_tokens_split"] / steps
            full_tok = batch * 8 * (ctx + warm + 10)
            perfect_us = full_us * split_tok / full_tok
            planner_us, fixed_us = res["planner"][0], res["fixed"][0]
            row = {"context": ctx, "miss_share": skew, "streamed_MB": round(split_tok * 512 / 1e6, 1),
                   "groups_missing_per_step": round((st["kv_tokens_read"] / steps) / (ctx + warm) , 2),
                   "planner_us": round(planner_us, 1), "fixed_items_us": round(fixed_us, 1),
                   "perfect_us": round(perfect_us, 1), "full_stream_us": round(full_us, 1),
                   "planner_over_perfect": round(planner_us / perfect_us, 3),
                   "excess_recovered": round((fixed_us - planner_us) / max(1e-9, fixed_us - perfect_us), 3)}
            rows.append(row)
            log(f"[balance-table] ctx {ctx:6d} miss share {skew:.1f} ({row['streamed_MB']:7.1f} MB/step, "
                f"~{row['groups_missing_per_step']:.1f} of 64 groups stream everything): planner {planner_us:6.1f} us, "
                f"fixed 2048-token items {fixed_us:6.1f} us, perfect {perfect_us:6.1f} us "
                f"(planner = {row['planner_over_perfect']:.2f} x perfect, recovers {100 * row['excess_recovered']:.0f} % of the excess)")
        del kv
        torch.cuda.empty_cache()
    return rows


def stream_probe(torch, mb, total_bytes: int = 2 << 30):
    """What a kernel that only loads pulls out of HBM on this machine (include/mac_probe.h): 2 GiB read in segments of one
    (page, K|V, head) block of the KV cache (4 KiB) and larger, in address order and in a seeded random order, with the
    non-temporal hint the attention kernel uses and without.  The attention kernel's K/V stream has the random 4 KiB
    pattern; its achieved bandwidth is to be held against that row (the roofline fraction stays against 8 TB/s)."""
    buf = torch.ones(total_bytes // 4, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    gen = torch.Generator(device="cpu")
    gen.manual_seed(1)
    rows = []
    for seg, shuffle, nt, wgs in ((4096, False, True, 512), (4096, True, True, 512), (4096, True, True, 1024),
                                  (4096, True, False, 1024), (2048, True, True, 1024), (16384, True, True, 1024),
                                  (16384, False, True, 256)):
        n = total_bytes // seg
        order = (torch.randperm(n, generator=gen) if shuffle else torch.arange(n)).to(torch.int32).to("cuda:0")
        torch.cuda.synchronize()
        us = mb.mac_probe_stream(buf.data_ptr(), order.data_ptr(), n, seg, nt, wgs, 10, sink.data_ptr(), st)
        rows.append({"segment_bytes": seg, "order": "random" if shuffle else "linear", "non_temporal": nt,
                     "work_groups": wgs, "us_per_2GiB": round(us, 1), "GBps": round(total_bytes / us / 1e3, 0)})
        log(f"[stream-probe] {seg:6d}-byte segments, {rows[-1]['order']:6s} order, "
            f"{'non-temporal' if nt else 'plain       '} loads, {wgs:5d} work-groups: {us:7.1f} us per 2 GiB = "
            f"{total_bytes / us / 1e6:.2f} TB/s")
        del order
    del buf
    torch.cuda.empty_cache()
    return rows


def err_table(torch, mb, wl_mod, align: float = 1.5, context: int = 32768, timed: int = 48):
    """Synthetic analogue of the paper's rectification-error heat-map (Sec. 5.4): the relative error of the MAC output
    against full attention of the same step, Err = |o_MAC - o_full| / |o_full|, averaged over the heads that hit, as a
    function of the reuse gap Delta and the band width r.  One request of Llama-3.1-8B geometry; queries recur with
    period Delta exactly and the window holds Delta + 1 entries, so the entry Delta back is the only near-duplicate
    in the window; keys and queries share a per-KV-head direction
    of weight `align`, which under RoPE makes recent keys carry most of the attention mass.  Both outputs come from
    the library (decode_step and full_decode).  Only the trend is comparable with the paper's figure (trained
    model, real text): error falls quickly as r grows and rises with Delta."""
    rows = []
    kv = None
    for gap in (2, 8, 64, 512):
        W = gap + 1
        for r in (0, 8, 32, 128, 256):
            steps = 2 * gap + timed
            cfg = wl_mod.WorkloadConfig(name=f"E_{gap}_{r}", batch=1, num_q_heads=32, num_kv_heads=8, context=context,
                                        steps=steps, window=W, band=r, threshold=0.5 * 128 ** 0.5, rho=0.0, seed=13,
                                        period=gap, period_std=0.0, query_noise=0.05, align=align)
            if kv is None:
                kv = wl_mod.Workload(wl_mod.scaled(cfg, steps=2 * 512 + timed), device="cuda:0")   # K/V for the longest run
            wl = wl_mod.Workload(cfg, device="cuda:0", queries_only=True)
            wl.kv_pages, wl.block_table = kv.kv_pages, kv.block_table
            mac = mb.MacAttention(num_q_heads=32, num_kv_heads=8, window=W, band=r, threshold=cfg.threshold,
                                  max_kv_len=kv.cfg.max_kv_len, max_slots=1)
            o_mac = torch.zeros((1, 32, 128), dtype=torch.float32, device="cuda:0")
            o_full = torch.zeros_like(o_mac)
            pos = torch.zeros((1, 32), dtype=torch.int32, device="cuda:0")
            stream = torch.cuda.current_stream().cuda_stream
            err_sum = torch.zeros((), dtype=torch.float64, device="cuda:0")
            err_max = torch.zeros((), dtype=torch.float64, device="cuda:0")
            n_hit = torch.zeros((), dtype=torch.int64, device="cuda:0")
            for s, (qp, qr, kl) in enumerate(wl):
                a = mac.make_args(kv_lens=kl, q_rope=qr, kv_pages=wl.kv_pages, strides=kv.strides,
                                  block_table=wl.block_table, out=o_mac, slot_ids=wl.slot_ids, q_pre=qp, match_pos=pos)
                mac.decode_step(a, stream)
                if s == 2 * gap - 1:
                    mac.stats(reset=True)
                if s >= 2 * gap:
                    a.out = o_full.data_ptr()
                    mac.full_decode(a, stream)
                    e = (o_mac - o_full).double().norm(dim=-1) / o_full.double().norm(dim=-1)
                    hit = pos >= 0
                    err_sum += (e * hit).sum()
                    err_max = torch.maximum(err_max, (e * hit).max())
                    n_hit += hit.sum()
            torch.cuda.synchronize()
            st = mac.stats()
            mac.close()
            nh = int(n_hit.item())
            row = {"gap": gap, "band": r, "mean_err": float(err_sum.item()) / max(1, nh), "max_err": float(err_max.item()),
                   "hit_heads": nh, "mean_gap": round(st["sum_gap"] / max(1, st["hits"]), 1)}
            rows.append(row)
            log(f"[err-table] gap {gap:4d} band {r:4d}: mean Err {row['mean_err']:.3e}  max {row['max_err']:.3e}  "
                f"(hits {nh}, measured gap {row['mean_gap']})")
    del kv
    torch.cuda.empty_cache()
    return rows


def cpu_baseline(name: str, torch, wl_mod, sample_steps: int):
    """The fp64 oracle as it stands, timed on the host cores on the first `sample_steps` decode steps of the
    same workload (rings start empty, so the sample is self-consistent)."""
    from oracle.mac_oracle import Oracle, num_threads
    cfg = wl_mod.CONFIGS[name]
    wl = wl_mod.Workload(cfg, device="cuda:0")
    kvp = wl_mod.bf16_bits(wl.kv_pages)
    bt = wl.block_table.cpu().numpy()
    slots = wl.slot_ids.cpu().numpy()
    orc = Oracle(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, head_dim=cfg.head_dim,
                 page_size=cfg.page_size, window=cfg.window, band=cfg.band, threshold=cfg.threshold,
                 strides=wl.strides, max_slots=cfg.batch)
    steps_in = [wl.next_step() for _ in range(sample_steps)]
    host = [(wl_mod.bf16_bits(a), wl_mod.bf16_bits(b), c.cpu().numpy()) for a, b, c in steps_in]
    del wl
    t0 = time.perf_counter()
    for qp, qr, kl in host:
        orc.mac_step(slots, kl, qp, qr, kvp, bt)
    dt = time.perf_counter() - t0
    hit = orc.stats.hits / max(1, orc.stats.head_steps)
    return {"value": 1e6 * dt / sample_steps, "unit": "us/step", "cores": num_threads(), "kind": "oracle",
            "sample": f"first {sample_steps} MAC decode steps of {name} from empty rings (plain C fp64 oracle built with "
                      f"gcc -O2, no -march=native, OpenMP over (request, head)); hit rate in the sample {100 * hit:.0f}%"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="C3_rho97", help="headline config (a C3 pair by default)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the other two (rho, threshold) pairs of C3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=100)
    ap.add_argument("--report", action="store_true",
                    help="also run every BASELINE config (C1, C2, C3 x3, C4 miss/hit, C5 past its first regime) and add "
                         "a per-config summary to the JSON line as 'configs_report'")
    ap.add_argument("--paper-table", action="store_true",
                    help="also run the analogue of the paper's fine-grained latency table (batch 1, 32K/60K/120K x KV "
                         "budgets 1/5/10/20 %%, K 1024, r 256) and add it to the JSON line as 'paper_table'")
    ap.add_argument("--match-table", action="store_true",
                    help="also run the Match-vs-Attention kernel micro-benchmark (GQA 8-2 / 32-8 / 40-10 x 512 / 1024 / "
                         "2048 tokens) and add it to the JSON line as 'match_table'")
    ap.add_argument("--err-table", action="store_true",
                    help="also run the synthetic analogue of the rectification-error heat-map (error of MAC against full "
                         "attention over reuse gap x band width) and add it as 'err_table'")
    ap.add_argument("--balance-table", action="store_true",
                    help="also run the analogue of the paper's load-balancing study (32K / 64K / 128K x share of KV groups "
                         "that miss 0.1 / 0.2 / 0.3: device planner against fixed-size items and a perfect schedule) and "
                         "add it as 'balance_table'")
    ap.add_argument("--graph", action="store_true",
                    help="also time the headline config replayed from one captured HIP graph per step (input refresh, "
                         "the library's launches and the step counter all inside the graph), beside the same device "
                         "work launched eagerly")
    ap.add_argument("--stream-probe", action="store_true",
                    help="also measure what a load-only kernel streams from HBM with the K/V access pattern (random 4 KiB "
                         "blocks) and add it as 'stream_probe': the measured ceiling beside the published peak")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that a rocprofv3 --pmc run of this "
                         "command can scale FETCH_SIZE / WRITE_SIZE")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    from paper_2604_00235_amd import binding as mb
    from paper_2604_00235_amd import workload as wl_mod
    mb.load_library()     # fails loudly if the HIP library is not built

    head, wl = run_config(a.config, a.steps, a.warmup, torch, mb, wl_mod, use_graph=a.graph)
    sweep = {}
    if not a.no_sweep and a.config.startswith("C3_"):
        for other in ("C3_rho90", "C3_rho97", "C3_rho99"):
            if other != a.config:
                sweep[other], _ = run_config(other, a.steps, a.warmup, torch, mb, wl_mod, keep_kv=wl)
        # the same workload with one reuse point per KV group (a variant of the library, not the paper's per-head rule):
        # a group hits as a whole, so the hits of its heads are no longer lost to the group's smallest start
        sweep[a.config + "+group_match"], _ = run_config(a.config, a.steps, a.warmup, torch, mb, wl_mod, keep_kv=wl,
                                                         group_match=True)
    del wl
    torch.cuda.empty_cache()
    if a.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = wl_mod.CONFIGS[a.config]
    ratios = traffic_ratios()
    r_mac, r_full = ratios.get((a.config, "mac")), ratios.get((a.config, "full"))
    traffic_src = (os.path.relpath(TRAFFIC_FILE, ROOT) if r_mac is not None else
                   f"null: {a.config} has no rocprofv3 --pmc record in {os.path.relpath(TRAFFIC_FILE, ROOT)}")
    line = {
        "metric": "decode_attention_us_per_step", "value": round(head["us_per_step"], 2), "unit": "us/step",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(head["us_per_step"] / 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.config}: batch {cfg.batch}, {cfg.num_q_heads}/{cfg.num_kv_heads} heads, d 128, "
                               f"context {cfg.context} (+{a.warmup + a.steps} decoded), paged bf16 KV page {cfg.page_size}, "
                               f"W {cfg.window}, B {cfg.band}, T {cfg.threshold}, AR(1) rho {cfg.rho}",
                   "global_batch": cfg.batch, "seq_len": cfg.context},
        "hit_rate": round(head["hit_rate"], 4),
        "kv_read_reduction_pct": round(head["kv_read_reduction_pct"], 2),
        "full_decode_us_per_step": round(head["full_decode_us_per_step"], 2),
        "speedup_vs_full_decode": round(head["speedup_vs_full"], 3),
        "achieved_hbm_GBps": round(head["attn_GBps"], 1),
        "effective_hbm_GBps": round(head["effective_GBps"], 1),
        "graph_replay_us_per_step": None if head["graph_us_per_step"] is None else round(head["graph_us_per_step"], 2),
        "eager_same_work_us_per_step": (None if head["eager_same_work_us_per_step"] is None
                                        else round(head["eager_same_work_us_per_step"], 2)),
        "kernel_us": {k: round(v, 2) for k, v in head["kernel_us"].items()},
        "roofline": {
            "bound": "hbm", "kernel": "attn_kernel (band+tail / full split-K attention) inside mac_attn_decode_step",
            "achieved": round(head["attn_GBps"], 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(head["attn_GBps"] / HBM_PEAK_GBPS, 4),
            "traffic": None if r_mac is None else round(r_mac * head["attn_bytes_per_launch"]),
            "traffic_over_algorithmic": r_mac, "traffic_source": traffic_src,
            "bytes_per_launch": round(head["attn_bytes_per_launch"]), "us_per_launch": round(head["kernel_us"]["attention"], 2),
        },
        "full_decode_roofline": {
            "achieved": round(head["full_attn_GBps"], 1), "frac": round(head["full_attn_GBps"] / HBM_PEAK_GBPS, 4),
            "traffic": None if r_full is None else round(r_full * head["full_attn_bytes_per_launch"]),
            "traffic_over_algorithmic": r_full,
            "bytes_per_launch": round(head["full_attn_bytes_per_launch"]),
            "us_per_launch": round(head["full_kernel_us"]["attention"], 2),
        },
        "sweep": {k: {"us_per_step": round(v["us_per_step"], 2), "hit_rate": round(v["hit_rate"], 4),
                      "kv_read_reduction_pct": round(v["kv_read_reduction_pct"], 2),
                      "speedup_vs_full_decode": round(v["speedup_vs_full"], 3),
                      "attn_GBps": round(v["attn_GBps"], 1), "threshold": v["threshold"]} for k, v in sweep.items()},
        "paper_context": "paper (H100 SXM5, FlashInfer 0.2.7 baseline, batch unstated): full attention 234.2 us and "
                         "MAC 63.6-104.5 us at 120K; another machine, context not target",
    }
    if a.report:
        plan = [("C1", 10, 4), ("C2", 60, 8), ("C3_rho90", 40, 8), ("C3_rho97", 40, 8), ("C3_rho99", 40, 8),
                ("C4_miss", 30, 4), ("C4_hit", 30, 8), ("C5", 100, 300)]
        rep = []
        for name, st, wu in plan:
            r, w_ = run_config(name, st, wu, torch, mb, wl_mod)
            del w_
            torch.cuda.empty_cache()
            rep.append({"config": name, "us_per_step": round(r["us_per_step"], 1),
                        "full_decode_us_per_step": round(r["full_decode_us_per_step"], 1),
                        "speedup_vs_full_decode": round(r["speedup_vs_full"], 2), "hit_rate": round(r["hit_rate"], 4),
                        "kv_read_reduction_pct": round(r["kv_read_reduction_pct"], 2),
                        "attn_kernel_GBps": round(r["attn_GBps"], 0), "full_attn_kernel_GBps": round(r["full_attn_GBps"], 0),
                        "kernel_us": {k: round(v, 1) for k, v in r["kernel_us"].items()}})
        line["configs_report"] = rep
    if a.paper_table:
        line["paper_table"] = paper_table(torch, mb, wl_mod)
    if a.match_table:
        line["match_table"] = match_table(torch, mb, wl_mod)
    if a.err_table:
        line["err_table"] = err_table(torch, mb, wl_mod)
    if a.balance_table:
        line["balance_table"] = balance_table(torch, mb, wl_mod)
    if a.stream_probe:
        line["stream_probe"] = stream_probe(torch, mb)
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(a.config, torch, wl_mod, a.cpu_steps)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
