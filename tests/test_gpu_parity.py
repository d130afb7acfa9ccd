"""GPU parity: the HIP library (through the C ABI) against the fp64 CPU oracle, element by element, on the
same seeded inputs, at sizes the oracle finishes in seconds that still span several tiles, several split-K
work items and ragged tails.  Needs a real MI355X."""
from __future__ import annotations

import math

import numpy as np
import pytest
import torch

from paper_2604_00235_amd.workload import CONFIGS, Workload, WorkloadConfig, bf16_bits, scaled

pytestmark = pytest.mark.gpu

T_DEFAULT = 0.5 * math.sqrt(128.0)


def test_c1_tiny_config_exact():
    """BASELINE configs[0] as stated: batch 1, 8/2 heads, context 4096, W=32, B=64, 32 steps, seed 0."""
    from tests.gpu_harness import run_parity
    r = run_parity(CONFIGS["C1"])
    assert r["hits"] > 0


@pytest.mark.parametrize("chunk,fused,span", [(0, True, 0), (256, True, -1), (256, False, 0), (256, False, -1),
                                              (128, True, 66)])
def test_llama_shape_reduced_mixed_hits(chunk, fused, span):
    """C2 geometry (32/8 heads) at a reduced, ragged context; threshold near the lag-1 distance so that hits
    and misses mix inside KV groups (per-head start masks, group-level spans)."""
    from tests.gpu_harness import run_parity
    cfg = scaled(CONFIGS["C2"], name="C2r", batch=3, context=2500, steps=24, window=16, band=64,
                 threshold=2.8, ragged=37)
    r = run_parity(cfg, chunk_tokens=chunk, fuse_epilogue=fused, fused_hit_span=span)
    assert 0 < r["hits"] < r["head_steps"]
    if span >= 0:
        assert r["kv_tokens_fused"] > 0           # hits at gap 1: ranges of 65 tokens, finished by the matcher
    if span == 66:
        assert r["kv_tokens_fused"] < r["hits"] * 66      # ... and some longer ones left to the split-K path


def test_mqa_threshold_zero_equals_full_attention():
    """C4 run A (MQA, G=32): threshold 0 => every step misses => output equals full attention."""
    from tests.gpu_harness import run_parity
    cfg = scaled(CONFIGS["C4_miss"], name="C4a", batch=2, context=1500, steps=6, window=8)
    r = run_parity(cfg, chunk_tokens=512)
    assert r["hits"] == 0


@pytest.mark.parametrize("fused,span", [(True, 0), (False, 0), (True, -1)])
def test_mqa_matched_threshold(fused, span):
    """C4 run B (MQA, G=32) at reduced context with the config's threshold: all hits after the first step."""
    from tests.gpu_harness import run_parity
    cfg = scaled(CONFIGS["C4_hit"], name="C4b", batch=2, context=1400, steps=20, window=8, ragged=3)
    r = run_parity(cfg, fuse_epilogue=fused, fused_hit_span=span)
    assert r["hits"] == r["head_steps"] - cfg.batch * cfg.num_q_heads


@pytest.mark.parametrize("fused,span", [(True, 0), (False, 0), (True, -1), (False, 70)])
def test_continuous_generation_regime_shifts_and_ring_wrap(fused, span):
    """C5 geometry (64/8 heads, G=8), regime shift every 8 steps, W=8 so the ring wraps 5 times."""
    from tests.gpu_harness import run_parity
    cfg = scaled(CONFIGS["C5"], name="C5r", batch=2, context=700, steps=40, window=8, band=64,
                 regime_shift_every=8)
    r = run_parity(cfg, chunk_tokens=128, check_ring_every=1, fuse_epilogue=fused, fused_hit_span=span)
    assert 0 < r["hits"] < r["head_steps"]


@pytest.mark.parametrize("kw", [
    dict(context=0, steps=40, band=64, window=4),            # kv_len 1..40: band covers everything, prefix empty
    dict(context=5, steps=12, band=0, window=3),             # B = 0: naive reuse of the whole prefix
    dict(context=100, steps=10, band=7, window=1),           # W = 1: only the previous query is a candidate
    dict(context=31, steps=6, band=16, window=4, threshold=1e30),   # tile edge; everything hits
    dict(context=300, steps=5, band=64, window=4, page_size=64),
    dict(context=300, steps=5, band=300, window=4, page_size=32, ragged=150),
])
def test_edge_cases(kw):
    from tests.gpu_harness import run_parity
    base = dict(name="edge", batch=2, num_q_heads=4, num_kv_heads=2, context=64, steps=8, window=4, band=8,
                threshold=T_DEFAULT, rho=0.97, seed=5)
    base.update(kw)
    for fused, span in ((True, 0), (False, 0), (True, -1)):
        run_parity(WorkloadConfig(**base), chunk_tokens=32, check_ring_every=1, fuse_epilogue=fused, fused_hit_span=span)


def test_strided_kv_layout_and_group_sizes():
    """The cache layout is given by strides: token-major pages [page, 2, tok, head, d]; G = 1, 2, 16."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    for hq, hkv in [(4, 4), (4, 2), (16, 1)]:
        cfg = WorkloadConfig(name="strided", batch=2, num_q_heads=hq, num_kv_heads=hkv, context=333, steps=3,
                             window=4, band=16, threshold=T_DEFAULT, rho=0.97, seed=9)
        wl = Workload(cfg, device="cuda:0")
        nhd = wl.kv_pages.permute(0, 1, 3, 2, 4).contiguous()      # [page, 2, tok, head, d]
        ps, d = cfg.page_size, cfg.head_dim
        strides = (2 * ps * hkv * d, ps * hkv * d, d, hkv * d)
        run = DeviceRun(cfg, wl, chunk_tokens=64, strides=strides, kv_pages=nhd)
        orc = make_oracle(cfg, wl, strides=strides)
        kvp, bt, slots = bf16_bits(nhd), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
        for q_pre, q_rope, kv_lens in wl:
            g_out, _, g_pos, _ = run.mac_step(q_pre, q_rope, kv_lens)
            ref = orc.mac_step(slots, kv_lens.cpu().numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
            assert np.array_equal(g_pos, ref["match_pos"])
            check_rows(g_out, ref["out"], f"strided G={hq // hkv}")
        run.mac.close()


def test_bitwise_determinism_and_reset():
    """Fixed chunking and merge order: two runs give bit-identical outputs and counters; a reset in mid-stream
    forces a miss on the next step (rings start empty)."""
    from tests.gpu_harness import DeviceRun
    cfg = scaled(CONFIGS["C2"], name="det", batch=2, context=900, steps=10, window=8)
    outs = []
    for rep in range(2):
        wl = Workload(cfg, device="cuda:0")
        run = DeviceRun(cfg, wl, chunk_tokens=128)
        seq = []
        for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
            if s == 6:
                run.mac.reset([1])
            o, l, p, d2 = run.mac_step(q_pre, q_rope, kv_lens)
            if s == 6:
                assert np.all(p[1] == -1) and np.all(p[0] >= 0)
            seq.append((o, l, p, d2))
        outs.append((seq, run.mac.stats()))
        run.mac.close()
    for (a, b) in zip(outs[0][0], outs[1][0]):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    assert outs[0][1] == outs[1][1]


def test_error_paths_on_device():
    from paper_2604_00235_amd import binding as mb
    mac = mb.MacAttention(num_q_heads=4, num_kv_heads=2, window=4, band=4, threshold=1.0, max_kv_len=64, max_slots=2)
    t = torch.zeros(16, device="cuda:0", dtype=torch.int32)
    args = mb.mac_attn_step_args()
    with pytest.raises(mb.MacAttnError):
        mb.mac_attn_decode_step(mac.ctx, args)           # batch 0, null pointers
    args.batch = 3
    with pytest.raises(mb.MacAttnError):
        mb.mac_attn_full_decode(mac.ctx, args)           # batch > max_batch
    mac.close()


@pytest.mark.parametrize("span", [0, -1, 100])
@pytest.mark.parametrize("hq,hkv,window,batch", [(32, 8, 1024, 1), (16, 2, 1024, 1), (32, 1, 256, 2), (8, 2, 200, 3),
                                                 (8, 2, 4096, 1)])
def test_recurring_queries_large_window_split_match(hq, hkv, window, batch, span):
    """Second query model (reuse gaps of tens to hundreds of tokens with skew inside a KV group, whole-group misses):
    exercises large windows (the 1024-thread matcher for few heads, several 64-row blocks per wave, a window that is
    not a multiple of the block size, the largest window of 4096 entries), with the fused hit path on, off, and limited to
    ranges of 100 tokens so that heads finished by the matcher and heads left to the split-K path mix inside a group."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"recur{hq}_{hkv}_{window}", batch=batch, num_q_heads=hq, num_kv_heads=hkv, context=1500,
                         steps=150, window=window, band=48, threshold=T_DEFAULT, rho=0.0, seed=21, period=40,
                         period_std=4.0, query_noise=0.1, jump_prob=0.05, ragged=11 if batch > 1 else 0)
    r = run_parity(cfg, chunk_tokens=256, check_full=False, check_ring_every=16, fused_hit_span=span)
    assert 0.3 * r["head_steps"] < r["hits"] < r["head_steps"]
    if span == 100:                                # reuse gaps of 36..44 + band 48: some ranges fit, wrapped ones do not
        assert 0 < r["kv_tokens_fused"]


# ----------------------------------------------------------------------------- variants of the match rule
def _recurring(name, hq, hkv, window, batch=2, steps=150, **kw):
    base = dict(name=name, batch=batch, num_q_heads=hq, num_kv_heads=hkv, context=1500, steps=steps, window=window,
                band=48, threshold=T_DEFAULT, rho=0.0, seed=23, period=40, period_std=4.0, query_noise=0.1,
                jump_prob=0.05, ragged=11 if batch > 1 else 0)
    base.update(kw)
    return WorkloadConfig(**base)


@pytest.mark.parametrize("max_gap", [30, 40, 1000])
def test_distance_cap(max_gap):
    """Accept the nearest candidate only if it is at most max_gap positions back (reuse gaps are ~40 +- 4 here, so
    a cap of 30 removes nearly every hit, 40 about half, 1000 none)."""
    from tests.gpu_harness import run_parity
    cfg = _recurring("cap", 8, 2, 200)
    r = run_parity(cfg, chunk_tokens=256, check_full=False, max_gap=max_gap)
    if max_gap == 30:
        assert r["hits"] < 0.1 * r["head_steps"]
    elif max_gap == 40:
        assert 0.1 * r["head_steps"] < r["hits"] < 0.7 * r["head_steps"]
    else:
        assert r["hits"] > 0.5 * r["head_steps"]


@pytest.mark.parametrize("hq,hkv,window,batch", [(32, 8, 256, 2), (32, 1, 128, 2), (8, 8, 64, 2), (6, 2, 100, 3),
                                                 (10, 2, 1024, 1), (32, 1, 4096, 1)])
def test_group_granular_matching(hq, hkv, window, batch):
    """One reuse point per KV group (ranked by the distance of the group's concatenated queries, threshold G T^2):
    G = 4, 32, 1, 3, 5; windows that are cut into slices, one that is not a multiple of the slice size, and the
    largest window with the largest group."""
    from tests.gpu_harness import run_parity
    steps = 150 if window <= 1024 else 60
    # one period for all heads, so that a group has a common nearest entry (with per-head periods it never hits)
    cfg = _recurring(f"group{hq}_{hkv}_{window}", hq, hkv, window, batch=batch, steps=steps, period_std=0.0)
    r = run_parity(cfg, chunk_tokens=256, check_full=False, check_ring_every=16, group_match=True)
    assert 0.2 * r["head_steps"] < r["hits"] < r["head_steps"]


def test_group_granular_matching_with_cap_ar1_queries():
    """AR(1) queries at C2 geometry, threshold near the lag-1 distance of a whole group, capped at one step back."""
    from tests.gpu_harness import run_parity
    cfg = scaled(CONFIGS["C2"], name="C2g", batch=3, context=2500, steps=24, window=16, band=64, threshold=2.8, ragged=37)
    r = run_parity(cfg, chunk_tokens=256, group_match=True, max_gap=1)
    assert 0 < r["hits"] < r["head_steps"]


def test_bf16_output_is_the_rounded_fp32_output():
    """out_dtype = bf16: the same step on two contexts, one per output type.  The fp32 context is checked against the
    oracle (decisions, decode_step and full_decode outputs); the bf16 result must be that fp32 result rounded to
    nearest even (torch's conversion is the reference rounding)."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = scaled(CONFIGS["C2"], name="bf16out", batch=2, context=700, steps=6, window=8, band=32, threshold=2.8)
    wl = Workload(cfg, device="cuda:0")
    r32 = DeviceRun(cfg, wl, chunk_tokens=128)
    r16 = DeviceRun(cfg, wl, chunk_tokens=128, out_bf16=True)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        lens = kv_lens.cpu().numpy()
        for mode in ("full", "mac"):
            for run in (r32, r16):
                a = run.args(q_pre if mode == "mac" else None, q_rope, kv_lens)
                (run.mac.decode_step if mode == "mac" else run.mac.full_decode)(a, run.stream)
            torch.cuda.synchronize()
            r32.check_guards()
            r16.check_guards()
            if mode == "full":
                ref_out, _ = orc.full_decode(lens, bf16_bits(q_rope), kvp, bt)
            else:
                ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
                ref_out = ref["out"]
                assert np.array_equal(r32.pos.cpu().numpy(), ref["match_pos"])
            check_rows(r32.out.cpu().numpy(), ref_out, f"bf16out step {s} {mode} (fp32 context)")
            assert r16.out.dtype == torch.bfloat16
            assert torch.equal(r16.out, r32.out.to(torch.bfloat16)), mode
        assert torch.equal(r16.pos, r32.pos)
    r32.mac.close()
    r16.mac.close()


@pytest.mark.parametrize("group", [17, 20, 24, 31])
def test_group_sizes_between_17_and_31(group):
    """Two 16-head tiles of which the second is partly filled (the remaining rows carry zero queries and are never
    stored): mixed hits and misses inside the group, ragged lengths, several work items."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"G{group}", batch=2, num_q_heads=group * 2, num_kv_heads=2, context=1200, steps=12,
                         window=8, band=40, threshold=2.8, rho=0.97, seed=31, ragged=19)
    r = run_parity(cfg, chunk_tokens=256, check_ring_every=2)
    assert 0 < r["hits"] < r["head_steps"]


@pytest.mark.parametrize("page_size,context,head_dim", [(16, 1024 + 3, 128), (16, 2048 + 10, 128), (64, 1024 + 9, 128),
                                                        (32, 777, 128), (16, 1024 + 5, 64)])
def test_memory_the_request_does_not_own_may_hold_nan(page_size, context, head_dim):
    """Only the pages a request's block table lists, and of its last page only the rows below kv_len, are the
    request's data.  Here every other byte of the cache is a NaN / Inf pattern: physical page 0 belongs to nobody, and
    in each request's last page the rows past the end are poisoned before every step.  Lengths are chosen so that the
    second 16-token half of the last 32-token tile lies wholly past the end (kv_len mod 32 in 1..16) on some steps."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = WorkloadConfig(name="poison", batch=2, num_q_heads=8, num_kv_heads=2, context=context, steps=6, window=4, band=24,
                         threshold=0.5 * math.sqrt(float(head_dim)), rho=0.97, seed=41, page_size=page_size, ragged=32,
                         head_dim=head_dim)
    wl = Workload(cfg, device="cuda:0")
    pages = torch.cat([torch.zeros_like(wl.kv_pages[:1]), wl.kv_pages]).contiguous()
    bad = torch.tensor([0x7FC0, 0x7F80, 0xFF80, 0xFFFF], dtype=torch.int32).to(torch.int16).to("cuda:0")
    pages[0].view(torch.int16).view(-1, 4)[:] = bad                      # page 0: NaN, +Inf, -Inf, NaN
    wl.block_table = (wl.block_table + 1).contiguous()
    wl.kv_pages = pages
    run = DeviceRun(cfg, wl, chunk_tokens=256)
    orc = make_oracle(cfg, wl)
    bt, slots = wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    hits = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        lens = kv_lens.cpu().numpy()
        clean = pages.clone()
        for b in range(cfg.batch):                                      # rows [n, end of the last page) of request b
            n = int(lens[b])
            if n % page_size:
                pg = int(bt[b, (n - 1) // page_size])
                pages[pg, :, :, n % page_size:] = float("nan")
        kvp = bf16_bits(pages)
        f_out, f_lse = run.full(q_rope, kv_lens)
        o_out, o_lse = orc.full_decode(lens, bf16_bits(q_rope), kvp, bt)
        check_rows(f_out, o_out, f"poison step {s} full_decode")
        g_out, g_lse, g_pos, _ = run.mac_step(q_pre, q_rope, kv_lens)
        ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert np.array_equal(g_pos, ref["match_pos"])
        check_rows(g_out, ref["out"], f"poison step {s} decode_step")
        assert np.abs(g_lse - ref["lse"]).max() < 1e-3
        hits += int((g_pos >= 0).sum())
        pages.copy_(clean)                                              # the poisoned rows are later tokens' data
    assert hits > 0
    run.mac.close()


@pytest.mark.parametrize("window,batch,hq,hkv", [(2, 2, 4, 2), (300, 1, 8, 2), (2, 40, 32, 8)])
def test_candidates_that_tie_to_rounding_are_decided_as_the_index_order_sum_decides(window, batch, hq, hkv):
    """Two window entries whose distances to the query are equal as real numbers (one is a permutation of the other, the
    query is zero) or differ far below the rounding error of a 128-term fp64 sum (one small element nudged).  The
    terms span ~2^60, so the fp64 value depends on the order of summation, and which entry is "nearest" is decided by
    that rounding.  The reference takes the plain left-to-right sum; the library has to come to the same decision and
    the same distance bit for bit (its matcher re-sums such candidates in index order), at every such step.
    Three shapes, one per build of the matcher: 256 threads, 1024 threads (few heads, window above 256) and the lean
    one (more than 1024 heads); the latter two start every triple of steps from empty rings, so that the two entries
    are the whole window."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = WorkloadConfig(name=f"neartie{window}_{batch}", batch=batch, num_q_heads=hq, num_kv_heads=hkv, context=50,
                         steps=30 if batch < 8 else 12, window=window, band=8, threshold=1e30, rho=0.9, seed=51)
    fresh_triples = (window, batch) != (2, 2)
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl, chunk_tokens=32)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    rng = np.random.default_rng(7)

    def seq_sum(row):                                  # the left-to-right fp64 sum of squares, as the reference forms it
        acc = np.float64(0.0)
        for x in row.astype(np.float64):
            acc = acc + x * x
        return acc

    order_matters = decided_by_rounding = 0
    base = None
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        shape = tuple(q_pre.shape)
        if s % 3 == 0:                                 # bf16-exact values (8 significant bits) over 26 binades
            e = rng.integers(-20, 7, size=shape)
            m = rng.integers(0, 128, size=shape)
            sign = rng.choice([-1.0, 1.0], size=shape)
            base = sign * (1.0 + m / 128.0) * np.exp2(e)
            rows = base
        elif s % 3 == 1:                               # the same multiset in another order; every other head: one small element nudged
            rows = np.stack([np.stack([rng.permutation(base[b, h]) for h in range(shape[1])]) for b in range(shape[0])])
            for b in range(shape[0]):
                for h in range(1, shape[1], 2):
                    i = int(np.argmin(np.abs(rows[b, h])))
                    x = rows[b, h, i]
                    ulp = np.exp2(np.floor(np.log2(abs(x))) - 7)            # one step of the 8-bit significand
                    rows[b, h, i] = x + np.sign(x) * ulp
            for b in range(shape[0]):
                for h in range(shape[1]):
                    a, c = seq_sum(base[b, h]), seq_sum(rows[b, h])
                    order_matters += int(a != seq_sum(np.sort(base[b, h])))
                    decided_by_rounding += int(a != c and abs(a - c) <= 2.0 ** -44 * a)
        else:
            rows = np.zeros(shape)
        q_pre = torch.tensor(rows, dtype=torch.float32).to(torch.bfloat16).to("cuda:0")
        assert torch.equal(q_pre.float().cpu(), torch.tensor(rows, dtype=torch.float32)), "not exact in bf16"
        lens = kv_lens.cpu().numpy()
        g_out, g_lse, g_pos, g_d2 = run.mac_step(q_pre, q_rope, kv_lens)
        ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert np.array_equal(g_pos, ref["match_pos"]), f"step {s}: {g_pos.tolist()} vs {ref['match_pos'].tolist()}"
        if s % 3 == 2:
            assert np.array_equal(g_d2, ref["d2"]), f"step {s}: distances differ in the last bits"
            assert (g_pos >= 0).all()
        check_rows(g_out, ref["out"], f"neartie step {s}")
        if s % 3 == 2 and fresh_triples:
            run.mac.reset()
            orc.reset()
    assert order_matters > 0 and decided_by_rounding > 0, (order_matters, decided_by_rounding)
    run.mac.close()


def test_more_work_items_than_work_groups():
    """A caller-fixed item size of 32 tokens on 4 KV groups of ~9000 tokens makes ~1130 work items, more than the
    attention grid's cap (four work-groups per compute unit): work-groups then loop over item, item + grid, ..."""
    cfg = WorkloadConfig(name="many_items", batch=2, num_q_heads=8, num_kv_heads=2, context=9001, steps=5, window=8,
                         band=40, threshold=3.2, rho=0.95, seed=31, ragged=77)
    from tests.gpu_harness import run_parity
    r = run_parity(cfg, chunk_tokens=32, fused_hit_span=-1)
    assert 0 < r["hits"] < 5 * 16


@pytest.mark.parametrize("head_dim,hq,hkv,span,group", [(64, 8, 2, 0, False), (64, 32, 1, 0, False), (32, 6, 2, -1, False),
                                                        (96, 8, 8, 0, False), (64, 8, 2, 0, True), (96, 20, 1, 70, False)])
def test_head_dims_below_128(head_dim, hq, hkv, span, group):
    """d = 32, 64, 96: the caller's queries, outputs and K/V rows have d elements (the library widens rows to 128 inside);
    per-head and per-group matching, the fused hit path on / off / limited, one and two head tiles, ragged requests,
    full decode at every step."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"d{head_dim}_{hq}_{hkv}", batch=3, num_q_heads=hq, num_kv_heads=hkv, context=1300, steps=24,
                         window=16, band=40, threshold=math.sqrt(2 * (1 - 0.97) * head_dim),      # about half of the heads hit
                         rho=0.97, seed=41, ragged=131, head_dim=head_dim)
    r = run_parity(cfg, chunk_tokens=0 if hq != 6 else 96, fused_hit_span=span, group_match=group)
    assert 0 < r["hits"] < r["head_steps"] - 3 * hq


@pytest.mark.parametrize("batch,window,head_dim", [(1, 1024, 64), (40, 64, 64), (40, 300, 128), (36, 16, 96)])
def test_matcher_variants_by_head_count(batch, window, head_dim):
    """The per-head matcher has three builds: 1024 threads for few heads and a large window (batch 1 here), 256 threads, and
    a lean 256-thread one for more heads than four work-groups per compute unit (batch 36 / 40 x 32 heads here).  Each with
    head dimensions below 128 too, windows that are not a multiple of the 32- or 64-row blocks, mixed hits."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"variants{batch}_{window}_{head_dim}", batch=batch, num_q_heads=32, num_kv_heads=8, context=700,
                         steps=20 if batch > 1 else 60, window=window, band=24, threshold=math.sqrt(2 * (1 - 0.97) * head_dim),
                         rho=0.97, seed=43, ragged=13 if batch > 1 else 0, head_dim=head_dim)
    r = run_parity(cfg, check_full=False, check_ring_every=8)
    assert 0 < r["hits"] < r["head_steps"]


@pytest.mark.parametrize("align,head_dim", [(1.5, 128), (3.0, 128), (2.0, 64)])
def test_recency_weighted_logits(align, head_dim):
    """Keys and queries share a per-KV-head direction, so that logits are large for recent keys and decay with
    distance (the input model of the error table): peaked softmax rows with a wide dynamic range of the logits, on the
    hit path, the split-K path and full decode."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"recency{align}_{head_dim}", batch=3, num_q_heads=8, num_kv_heads=2, context=2500, steps=24, window=32,
                         band=48, threshold=math.sqrt(2 * (1 - 0.97) * head_dim) * (1.0 + 0.0), rho=0.97, seed=47, ragged=9,
                         align=align, head_dim=head_dim)
    r = run_parity(cfg, check_full=True, check_ring_every=4)
    assert r["head_steps"] == cfg.steps * cfg.batch * cfg.num_q_heads


@pytest.mark.parametrize("sm_scale", [0.5, 0.01])
def test_softmax_scale_given_by_the_caller(sm_scale):
    """sm_scale other than 1/sqrt(d): 0.5 makes the logits of N(0, 1) rows ~5.7 wide (one key takes most of a row), 0.01
    makes every row nearly uniform.  Both through the hit path, the split-K path and full decode."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"scale{sm_scale}", batch=2, num_q_heads=8, num_kv_heads=2, context=1800, steps=20, window=16,
                         band=40, threshold=math.sqrt(2 * (1 - 0.97) * 128), rho=0.97, seed=53, ragged=5)
    r = run_parity(cfg, check_full=True, check_ring_every=4, sm_scale=sm_scale)
    assert 0 < r["hits"] < r["head_steps"]


def test_requests_join_leave_and_change_places_in_the_batch():
    """Continuous batching: four requests on ring sets 5, 0, 3, 2 of a context with six; every step serves a seeded
    subset of them in a seeded order (2 to 4 requests: rows of kv_lens, queries, block table and slot_ids permuted
    together), so a request's place in the batch changes from step to step and a request that sits out a step finds
    its ring one entry short; at step 14 the request on ring set 3 leaves and a new one takes the set over (reset:
    its first step misses).  Decisions and outputs against the oracle at every step (what the rings hold shows in the
    later steps' decisions and merged outputs)."""
    from paper_2604_00235_amd import binding as mb
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = WorkloadConfig(name="batching", batch=4, num_q_heads=8, num_kv_heads=2, context=900, steps=28, window=8, band=24,
                         threshold=math.sqrt(2 * (1 - 0.97) * 128), rho=0.97, seed=59, ragged=11)
    wl = Workload(cfg, device="cuda:0")
    n_sets = 6
    run = DeviceRun(cfg, wl)
    run.mac.close()
    run.mac = mb.MacAttention(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, window=cfg.window, band=cfg.band,
                              threshold=cfg.threshold, max_kv_len=cfg.max_kv_len, max_slots=n_sets, max_batch=cfg.batch)
    orc = make_oracle(cfg, wl, max_slots=n_sets)
    kvp = bf16_bits(wl.kv_pages)
    set_of = torch.tensor([5, 0, 3, 2], dtype=torch.int32, device="cuda:0")
    rng = np.random.default_rng(61)
    hits = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        if s == 14:
            run.mac.reset([3])
            orc.reset([3])
        k = int(rng.integers(2, 5))
        order = torch.from_numpy(rng.permutation(4)[:k].astype(np.int64)).to("cuda:0")
        qp, qr = q_pre[order].contiguous(), q_rope[order].contiguous()
        kl, bt, sl = kv_lens[order].contiguous(), wl.block_table[order].contiguous(), set_of[order].contiguous()
        a = run.mac.make_args(kv_lens=kl, q_rope=qr, kv_pages=wl.kv_pages, strides=wl.strides, block_table=bt,
                              out=run.out, slot_ids=sl, q_pre=qp, out_lse=run.lse, match_pos=run.pos, match_d2=run.d2)
        run.mac.decode_step(a, run.stream)
        torch.cuda.synchronize()
        run.check_guards()
        ref = orc.mac_step(sl.cpu().numpy(), kl.cpu().numpy(), bf16_bits(qp), bf16_bits(qr), kvp, bt.cpu().numpy())
        pos = run.pos.cpu().numpy()[:k]
        assert np.array_equal(pos, ref["match_pos"]), f"step {s}"
        if s == 14 and 2 in order.tolist():
            assert (pos[order.tolist().index(2)] == -1).all()          # the new request's first step
        check_rows(run.out.cpu().numpy()[:k], ref["out"], f"batching step {s}")
        hits += int((pos >= 0).sum())
    assert hits > 0
    run.mac.close()


def test_optional_outputs_left_out_a_stream_of_the_callers_and_kernel_timing():
    """The same steps on two contexts: one with every optional output (LSE, matched position, distance) on the default
    stream, one with none of them, on a stream of the caller's, with per-kernel timing switched on.  The attention
    outputs must be the same bits; the timing must report one record per call and times that are positive where a
    kernel ran."""
    from paper_2604_00235_amd import binding as mb
    from tests.gpu_harness import DeviceRun
    cfg = WorkloadConfig(name="optional", batch=2, num_q_heads=8, num_kv_heads=2, context=1200, steps=10, window=8, band=32,
                         threshold=math.sqrt(2 * (1 - 0.97) * 128), rho=0.97, seed=67, ragged=3)
    wl = Workload(cfg, device="cuda:0")
    full = DeviceRun(cfg, wl)
    bare = DeviceRun(cfg, wl)
    side = torch.cuda.Stream()
    mb.mac_attn_set_timing(bare.mac.ctx, True)
    calls = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        for mode in ("mac", "full"):
            a = full.args(q_pre if mode == "mac" else None, q_rope, kv_lens)
            (full.mac.decode_step if mode == "mac" else full.mac.full_decode)(a, full.stream)
            b = bare.mac.make_args(kv_lens=kv_lens, q_rope=q_rope, kv_pages=wl.kv_pages, strides=wl.strides,
                                   block_table=wl.block_table, out=bare.out, slot_ids=wl.slot_ids,
                                   q_pre=q_pre if mode == "mac" else None)
            side.wait_stream(torch.cuda.current_stream())
            (bare.mac.decode_step if mode == "mac" else bare.mac.full_decode)(b, side.cuda_stream)
            calls += 1
            torch.cuda.synchronize()
            full.check_guards()
            bare.check_guards()
            assert torch.equal(full.out, bare.out), f"step {s} {mode}"
    us, n = mb.mac_attn_kernel_us(bare.mac.ctx)
    assert n == calls
    assert us[1] > 0 and us[2] > 0 and us[0] > 0          # attention and merge in every call, the matcher in the MAC steps
    assert all(0 <= u < 1e6 for u in us)
    mb.mac_attn_set_timing(bare.mac.ctx, False)
    full.mac.close()
    bare.mac.close()


def test_invalid_step_arguments_are_refused_and_nothing_runs():
    """Each of the step arguments the host can check, broken one at a time on an otherwise valid call: the call returns
    MAC_ATTN_ERR_INVALID_ARG and enqueues nothing (the output keeps its sentinel, the counters do not move)."""
    from paper_2604_00235_amd import binding as mb
    from tests.gpu_harness import DeviceRun
    cfg = WorkloadConfig(name="badargs", batch=2, num_q_heads=4, num_kv_heads=2, context=100, steps=2, window=4, band=8,
                         threshold=1.0, rho=0.9, seed=71)
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl)
    q_pre, q_rope, kv_lens = wl.next_step()
    good = run.args(q_pre, q_rope, kv_lens)
    run.mac.decode_step(good, run.stream)                  # the valid call works
    torch.cuda.synchronize()
    run.mac.stats(reset=True)
    run.out.fill_(-7.0)

    def broken(**kw):
        a = mb.mac_attn_step_args()
        for f, _ in a._fields_:
            setattr(a, f, getattr(good, f))
        for k, v in kw.items():
            setattr(a, k, v)
        return a
    cases = [("kv_lens", broken(kv_lens=None)), ("q_rope", broken(q_rope=None)), ("kv_pages", broken(kv_pages=None)),
             ("block_table", broken(block_table=None)), ("out", broken(out=None)), ("batch 0", broken(batch=0)),
             ("batch 3", broken(batch=3)), ("table stride", broken(block_table_stride=1)),
             ("stride 0", broken(stride_head=0)), ("stride % 8", broken(stride_page=good.stride_page + 4)),
             ("token stride below d", broken(stride_tok=64)), ("q_rope alignment", broken(q_rope=q_rope.data_ptr() + 2)),
             ("kv_pages alignment", broken(kv_pages=wl.kv_pages.data_ptr() + 8))]
    mac_only = [("q_pre", broken(q_pre=None)), ("slot_ids", broken(slot_ids=None)),
                ("q_pre alignment", broken(q_pre=q_pre.data_ptr() + 2))]
    for name, a in cases + mac_only:
        with pytest.raises(mb.MacAttnError) as e:
            mb.mac_attn_decode_step(run.mac.ctx, a, run.stream)
        assert e.value.code == mb.MAC_ATTN_ERR_INVALID_ARG, name
    for name, a in cases:
        with pytest.raises(mb.MacAttnError) as e:
            mb.mac_attn_full_decode(run.mac.ctx, a, run.stream)
        assert e.value.code == mb.MAC_ATTN_ERR_INVALID_ARG, name
    for name, a in mac_only[:2]:
        mb.mac_attn_full_decode(run.mac.ctx, a, run.stream)      # full decode ignores them
        torch.cuda.synchronize()
        run.out.fill_(-7.0)
    torch.cuda.synchronize()
    assert bool((run.out == -7.0).all())
    assert run.mac.stats()["steps"] == 0
    run.check_guards()
    run.mac.close()


@pytest.mark.parametrize("batch,hq,hkv", [(1, 8, 2), (3, 16, 4)])
def test_longest_fresh_ranges_the_matcher_finishes_itself(batch, hq, hkv):
    """Reuse gaps of ~1500 tokens with a band of 256: fresh ranges of ~1760 tokens, finished inside the matcher's
    work-group with fused_hit_span at its maximum of 2048 (several passes over the K and V rows per work-group, the
    logits of a whole range in shared memory), in the 1024-thread build (batch 1) and the 256-thread one."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"longfused{batch}", batch=batch, num_q_heads=hq, num_kv_heads=hkv, context=2600, steps=1590,
                         window=2048, band=256, threshold=T_DEFAULT, rho=0.0, seed=79, period=1500, period_std=12.0,
                         query_noise=0.1, jump_prob=0.0, ragged=5 if batch > 1 else 0)
    r = run_parity(cfg, check_full=False, check_ring_every=200, fused_hit_span=2048)
    assert r["hits"] > 0 and r["kv_tokens_fused"] > 1500 * r["hits"] // 2


@pytest.mark.parametrize("page_size", [128, 1024])
def test_large_pages(page_size):
    """KV pages of 128 and 1024 tokens (a work item then lies inside one or two pages; a request of ~2600 tokens has
    three pages of 1024), per-head matching with the fused hit path, the split-K path and full decode."""
    from tests.gpu_harness import run_parity
    cfg = WorkloadConfig(name=f"page{page_size}", batch=3, num_q_heads=8, num_kv_heads=2, context=2600, steps=16, window=16,
                         band=40, threshold=math.sqrt(2 * (1 - 0.97) * 128), rho=0.97, seed=83, ragged=301, page_size=page_size)
    r = run_parity(cfg, check_full=True, check_ring_every=4)
    assert 0 < r["hits"] < r["head_steps"]


@pytest.mark.parametrize("head_dim", [128, 64])
def test_separate_k_and_v_pools_with_padded_rows(head_dim):
    """Another layout through the same strides: all K pages first, then all V pages ([2, page, head, tok, d + 32]), rows
    padded by 32 elements that hold NaN and must never be read."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = WorkloadConfig(name=f"pools{head_dim}", batch=2, num_q_heads=8, num_kv_heads=2, context=700, steps=8, window=8, band=24,
                         threshold=math.sqrt(2 * (1 - 0.97) * head_dim), rho=0.97, seed=89, ragged=17, head_dim=head_dim)
    wl = Workload(cfg, device="cuda:0")
    ps, d, hkv = cfg.page_size, cfg.head_dim, cfg.num_kv_heads
    pages = wl.kv_pages.shape[0]
    dp = d + 32
    pools = torch.full((2, pages, hkv, ps, dp), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    pools[..., :d] = wl.kv_pages.permute(1, 0, 2, 3, 4)
    strides = (hkv * ps * dp, pages * hkv * ps * dp, ps * dp, dp)
    run = DeviceRun(cfg, wl, strides=strides, kv_pages=pools)
    orc = make_oracle(cfg, wl, strides=strides)
    kvp, bt, slots = bf16_bits(pools), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    hits = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        lens = kv_lens.cpu().numpy()
        g_full, _ = run.full(q_rope, kv_lens)
        o_full, _ = orc.full_decode(lens, bf16_bits(q_rope), kvp, bt)
        check_rows(g_full, o_full, f"pools step {s} full decode")
        g_out, _, g_pos, _ = run.mac_step(q_pre, q_rope, kv_lens)
        ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert np.array_equal(g_pos, ref["match_pos"])
        check_rows(g_out, ref["out"], f"pools step {s}")
        hits += int((g_pos >= 0).sum())
    assert hits > 0
    run.mac.close()


def test_requests_without_tokens_and_lengths_out_of_range():
    """kv_len = 0 (a padding row of a static batch): the output is the empty summary (0, -inf), every head misses and no
    ring entry is written, while the other requests of the batch are served as usual.  Lengths outside [0, max_kv_len]
    are clamped on the device: -5 acts as 0, max_kv_len + 100 as max_kv_len (the oracle is given the clamped values)."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = WorkloadConfig(name="emptyreq", batch=4, num_q_heads=8, num_kv_heads=2, context=300, steps=14, window=8, band=24,
                         threshold=math.sqrt(2 * (1 - 0.97) * 128), rho=0.97, seed=97, ragged=7)
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    hits = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        given = kv_lens.clone()
        given[0] = 0                                   # never has a token
        if s % 3 == 1:
            given[2] = -5                              # sits out every third step
        if s == 9:
            given[3] = cfg.max_kv_len + 100
        lens = np.clip(given.cpu().numpy(), 0, cfg.max_kv_len)
        g_full, g_flse = run.full(q_rope, given)
        o_full, o_flse = orc.full_decode(lens, bf16_bits(q_rope), kvp, bt)
        check_rows(g_full, o_full, f"emptyreq step {s} full decode")
        assert np.array_equal(np.isinf(g_flse), np.isinf(o_flse))
        g_out, g_lse, g_pos, g_d2 = run.mac_step(q_pre, q_rope, given)
        ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert np.array_equal(g_pos, ref["match_pos"]), f"step {s}"
        assert np.array_equal(np.isinf(g_d2), np.isinf(ref["d2"]))
        check_rows(g_out, ref["out"], f"emptyreq step {s}")
        for b in np.where(lens == 0)[0]:
            assert (g_out[b] == 0).all() and (g_lse[b] == -np.inf).all() and (g_pos[b] == -1).all()
            assert (g_full[b] == 0).all() and (g_flse[b] == -np.inf).all()
        hits += int((g_pos >= 0).sum())
    for j in range(cfg.window):                         # the ring set of the request that never had a token is still empty
        for h in (0, cfg.num_q_heads - 1):
            assert run.mac.ring_peek(0, j, h)[3] == 0
    assert hits > 0
    gst, ost = run.mac.stats(), orc.stats.as_dict()
    for k in ("steps", "head_steps", "hits", "misses", "sum_gap", "kv_tokens_read", "kv_tokens_full"):
        assert gst[k] == ost[k], k
    run.mac.close()


def test_a_request_rolls_back_some_tokens():
    """The length of a request goes back by 6 tokens in mid-stream (rejected speculative tokens) and grows again from
    there: its ring then holds entries created at lengths beyond the current one, which are no candidates (Eq. (accept):
    n_p <= n - 1) until the stream overwrites them, entry by entry, with the new ones."""
    from tests.gpu_harness import DeviceRun, check_rows
    from tests.helpers import make_oracle
    cfg = WorkloadConfig(name="rollback", batch=2, num_q_heads=8, num_kv_heads=2, context=200, steps=30, window=16, band=24,
                         threshold=math.sqrt(2 * (1 - 0.97) * 128) * 1.3, rho=0.97, seed=101)
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    hits_after = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        given = kv_lens.clone()
        if s >= 12:
            given[1] -= 6
        lens = given.cpu().numpy()
        g_out, g_lse, g_pos, g_d2 = run.mac_step(q_pre, q_rope, given)
        ref = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert np.array_equal(g_pos, ref["match_pos"]), f"step {s}"
        assert (g_pos[1] < lens[1]).all()
        check_rows(g_out, ref["out"], f"rollback step {s}")
        if s >= 12:
            hits_after += int((g_pos[1] >= 0).sum())
    assert hits_after > 0
    run.mac.close()
