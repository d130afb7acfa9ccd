"""Pins of the CPU oracle against things other than itself (CPU only).

Each test cites what fixes the expected value: a definition of the paper, a closed form,
a library routine on a special case, brute force in exact arithmetic, or an invariant.
"""
from __future__ import annotations

import math

import numpy as np
import pytest
import torch

from oracle.definition import DefinitionMAC, bf16_bits_to_f64, exact_sq_dist, unshifted_summary
from oracle.mac_oracle import Oracle
from paper_2604_00235_amd.workload import Workload, WorkloadConfig, bf16_bits
from tests.helpers import dense_kv, host_inputs, make_oracle, rel_l2


def small_cfg(**kw) -> WorkloadConfig:
    base = dict(name="small", batch=2, num_q_heads=4, num_kv_heads=2, context=37, steps=14, window=4, band=3,
                threshold=3.0, rho=0.9, head_dim=16, page_size=4, seed=11)
    base.update(kw)
    return WorkloadConfig(**base)


# ----------------------------------------------------------------------------- full attention
def test_full_decode_matches_torch_softmax():
    """Sec. 2 "Notation": o = softmax(q.K/sqrt(d)) V; torch.softmax in fp64 is the library routine."""
    cfg = small_cfg(context=53, steps=3, head_dim=32, page_size=8)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, _ = host_inputs(wl)
    for q_pre, q_rope, kv_lens in wl:
        out, lse = orc.full_decode(kv_lens.numpy(), bf16_bits(q_rope), kvp, bt)
        for b in range(cfg.batch):
            n = int(kv_lens[b])
            K, V = dense_kv(wl, b, n)
            for h in range(cfg.num_q_heads):
                g = h // cfg.group
                q = q_rope[b, h].double()
                logits = torch.from_numpy(K[:, g]) @ q * orc.sm_scale
                ref = torch.softmax(logits, 0) @ torch.from_numpy(V[:, g])
                np.testing.assert_allclose(out[b, h], ref.numpy(), rtol=1e-12, atol=1e-14)
                np.testing.assert_allclose(lse[b, h], torch.logsumexp(logits, 0).item(), rtol=1e-13)


def test_full_decode_closed_forms():
    """q = 0 or all keys equal => uniform weights => out = mean of V over [0, n);
    one key with a huge logit => out = that value row."""
    cfg = small_cfg(batch=1, context=29, steps=1, head_dim=16)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, _ = host_inputs(wl)
    q_pre, q_rope, kv_lens = wl.next_step()
    n = int(kv_lens[0])
    K, V = dense_kv(wl, 0, n)
    # q = 0
    out, lse = orc.full_decode(kv_lens.numpy(), np.zeros_like(bf16_bits(q_rope)), kvp, bt)
    for h in range(cfg.num_q_heads):
        np.testing.assert_allclose(out[0, h], V[:, h // cfg.group].mean(0), rtol=1e-13, atol=1e-15)
        assert abs(lse[0, h] - math.log(n)) < 1e-13
    # all keys equal
    wl2 = Workload(cfg)
    wl2.kv_pages[:, 0] = wl2.kv_pages[0, 0, 0, 0]
    out, _ = orc.full_decode(kv_lens.numpy(), bf16_bits(q_rope), bf16_bits(wl2.kv_pages), bt)
    K2, V2 = dense_kv(wl2, 0, n)
    for h in range(cfg.num_q_heads):
        np.testing.assert_allclose(out[0, h], V2[:, h // cfg.group].mean(0), rtol=1e-12, atol=1e-15)
    # one dominant key: key t* = 64 * q direction
    wl3 = Workload(cfg)
    tstar = 17
    page, within = int(wl3.block_table[0, tstar // cfg.page_size]), tstar % cfg.page_size
    qv = q_rope[0, 0].float()
    wl3.kv_pages[page, 0, 0, within] = (qv * 64.0).to(torch.bfloat16)
    out, _ = orc.full_decode(kv_lens.numpy(), bf16_bits(q_rope), bf16_bits(wl3.kv_pages), bt)
    K3, V3 = dense_kv(wl3, 0, n)
    np.testing.assert_allclose(out[0, 0], V3[tstar, 0], atol=1e-9)


def test_shifted_equals_unshifted_definition():
    """The (O, LSE) form equals the unshifted S/Z of Sec. 3.1 on small logits."""
    cfg = small_cfg(batch=1, context=21, steps=1)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, _ = host_inputs(wl)
    _, q_rope, kv_lens = wl.next_step()
    n = int(kv_lens[0])
    K, V = dense_kv(wl, 0, n)
    for h in range(cfg.num_q_heads):
        for lo, hi in [(0, n), (3, 9), (n - 1, n), (5, 5)]:
            O, lse = orc.summary(bf16_bits(q_rope), kvp, bt, 0, h, lo, hi)
            S, Z = unshifted_summary(q_rope[0, h].double().numpy(), K[:, h // cfg.group], V[:, h // cfg.group],
                                     lo, hi, orc.sm_scale)
            if hi > lo:
                np.testing.assert_allclose(O, S / Z, rtol=1e-12, atol=1e-15)
                assert abs(lse - math.log(Z)) < 1e-12
            else:
                assert lse == -np.inf and np.all(O == 0)


# ----------------------------------------------------------------------------- merge
def test_merge_of_arbitrary_partition_equals_unsplit():
    """Sec. 3.1: summaries over disjoint sets merge by addition, at any split point, in any order."""
    cfg = small_cfg(batch=1, context=61, steps=1)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, _ = host_inputs(wl)
    _, q_rope, kv_lens = wl.next_step()
    qb = bf16_bits(q_rope)
    n = int(kv_lens[0])
    rng = np.random.default_rng(5)
    for h in range(cfg.num_q_heads):
        whole, whole_l = orc.summary(qb, kvp, bt, 0, h, 0, n)
        for trial in range(6):
            cuts = np.sort(rng.choice(np.arange(1, n), size=rng.integers(1, 7), replace=False))
            edges = [0, *cuts.tolist(), n]
            parts = [orc.summary(qb, kvp, bt, 0, h, a, b) for a, b in zip(edges[:-1], edges[1:])]
            order = rng.permutation(len(parts))
            O, l = np.zeros(cfg.head_dim), -np.inf       # identity element
            for i in order:
                O, l = Oracle.merge(O, l, parts[i][0], parts[i][1])
            np.testing.assert_allclose(O, whole, rtol=1e-12, atol=1e-15)
            assert abs(l - whole_l) < 1e-12


def test_merge_identity_and_inverse():
    """(0, -inf) is the identity; removing b from merge(a, b) by subtraction of (S, Z) gives back a."""
    rng = np.random.default_rng(0)
    a, b = rng.normal(size=8), rng.normal(size=8)
    la, lb = 0.7, -1.3
    O, l = Oracle.merge(a, la, np.zeros(8), -np.inf)
    np.testing.assert_array_equal(O, a)
    assert l == la
    O, l = Oracle.merge(np.zeros(8), -np.inf, b, lb)
    np.testing.assert_array_equal(O, b)
    O, l = Oracle.merge(np.zeros(8), -np.inf, np.zeros(8), -np.inf)
    assert l == -np.inf and np.all(O == 0)
    O, l = Oracle.merge(a, la, b, lb)
    S, Z = O * math.exp(l), math.exp(l)
    Sa, Za = S - b * math.exp(lb), Z - math.exp(lb)
    np.testing.assert_allclose(Sa / Za, a, rtol=1e-12)
    assert abs(math.log(Za) - la) < 1e-12
    # closed form with two one-element sets: weights e^{la}/(e^{la}+e^{lb})
    wa = 1.0 / (1.0 + math.exp(lb - la))
    np.testing.assert_allclose(O, wa * a + (1 - wa) * b, rtol=1e-13)


# ----------------------------------------------------------------------------- match
def _fill_ring(orc: Oracle, rng, n_now: int, count: int):
    """Put `count` random entries created at lengths n_now-count .. n_now-1 into slot 0."""
    W, Hq, d = orc.W, orc.Hq, orc.d
    for n_p in range(n_now - count, n_now):
        j = (n_p - 1) % W
        vals = torch.from_numpy(rng.normal(size=(Hq, d)).astype(np.float32)).to(torch.bfloat16)
        orc.ring_q[0, j] = bf16_bits(vals)
        orc.ring_npos[0, j] = n_p


def test_match_brute_force_exact_rationals():
    """Eq. (accept) with exact rational arithmetic on the bf16 inputs: exact argmin and decision."""
    rng = np.random.default_rng(3)
    for trial in range(20):
        orc = Oracle(num_q_heads=3, num_kv_heads=1, head_dim=8, page_size=4, window=6, band=2,
                     threshold=float(rng.uniform(2.0, 5.0)), strides=(1, 1, 1, 1), max_slots=1)
        n = 40 + trial
        count = int(rng.integers(0, 7))
        _fill_ring(orc, rng, n, count)
        q = torch.from_numpy(rng.normal(size=(1, 3, 8)).astype(np.float32)).to(torch.bfloat16)
        pos, idx, d2 = orc.match(np.array([0]), np.array([n]), bf16_bits(q))
        qf = bf16_bits_to_f64(bf16_bits(q))[0]
        for h in range(3):
            best, best_np = None, None
            for j in range(orc.W):
                n_p = int(orc.ring_npos[0, j])
                if n_p < 1 or not (n - orc.W <= n_p <= n - 1):
                    continue
                dist = exact_sq_dist(qf[h], bf16_bits_to_f64(orc.ring_q[0, j, h]))
                if best is None or dist < best or (dist == best and n_p > best_np):
                    best, best_np = dist, n_p
            from fractions import Fraction
            hit = best is not None and best < Fraction(orc.T) ** 2
            assert pos[0, h] == (best_np if hit else -1)
            if best is not None:
                assert abs(d2[0, h] - float(best)) <= 1e-14 * float(best)
            else:
                assert d2[0, h] == np.inf


def test_match_window_bounds_and_ties():
    """Candidates are n_p in [n-W, n-1]; stale and empty entries are ignored; equal distances -> most recent;
    T = 0 never hits (strict <), even for an identical query; a huge T always hits once the ring is non-empty."""
    W, Hq, d = 4, 2, 8
    mk = lambda T: Oracle(num_q_heads=Hq, num_kv_heads=1, head_dim=d, page_size=4, window=W, band=1,
                          threshold=T, strides=(1, 1, 1, 1), max_slots=1)
    q = torch.arange(Hq * d, dtype=torch.float32).view(1, Hq, d).to(torch.bfloat16)
    qb = bf16_bits(q)
    n = 100
    # empty ring
    orc = mk(1e6)
    pos, _, d2 = orc.match(np.array([0]), np.array([n]), qb)
    assert np.all(pos == -1) and np.all(np.isinf(d2))
    # duplicates at n_p = 97 and 99 -> picks 99; a stale copy at n_p = 95 (outside [96, 99]) is ignored
    for n_p in (97, 99):
        orc.ring_q[0, (n_p - 1) % W] = qb[0]
        orc.ring_npos[0, (n_p - 1) % W] = n_p
    pos, _, d2 = orc.match(np.array([0]), np.array([n]), qb)
    assert np.all(pos == 99) and np.all(d2 == 0)
    orc0 = mk(0.0)
    orc0.ring_q[:] = orc.ring_q
    orc0.ring_npos[:] = orc.ring_npos
    pos, _, _ = orc0.match(np.array([0]), np.array([n]), qb)
    assert np.all(pos == -1)
    # window edge: entry at n_p = n - W is a candidate, n_p = n - W - 1 is not
    orc = mk(1e6)
    orc.ring_q[0, 0] = qb[0]
    orc.ring_npos[0, 0] = n - W
    assert np.all(orc.match(np.array([0]), np.array([n]), qb)[0] == n - W)
    orc.ring_npos[0, 0] = n - W - 1
    assert np.all(orc.match(np.array([0]), np.array([n]), qb)[0] == -1)
    orc.ring_npos[0, 0] = n          # an entry "from the future" (n_p > n-1) is not a candidate either
    assert np.all(orc.match(np.array([0]), np.array([n]), qb)[0] == -1)


def test_match_rate_follows_chi_square_null():
    """App. B.1: under the isotropic Gaussian null ||q_m - q_p||^2 = 2 chi^2_d, so with one candidate the
    acceptance rate is F_{chi^2_d}(T^2 / 2) = F(d (1 - tau)^2).  Pins '<', the sqrt(2d) scale and that the
    distance (not its square) is compared with T."""
    from scipy.stats import chi2
    d, trials = 32, 4000
    tau = 0.12
    T = math.sqrt(2 * d) * (1 - tau)
    orc = Oracle(num_q_heads=1, num_kv_heads=1, head_dim=d, page_size=4, window=1, band=1,
                 threshold=T, strides=(1, 1, 1, 1), max_slots=1)
    rng = np.random.default_rng(7)
    hits = 0
    for t in range(trials):
        a = rng.normal(size=(1, 1, d)).astype(np.float32)
        b = rng.normal(size=(1, 1, d)).astype(np.float32)
        orc.ring_q[0, 0] = bf16_bits(torch.from_numpy(b[0]).to(torch.bfloat16))
        orc.ring_npos[0, 0] = 9
        pos, _, _ = orc.match(np.array([0]), np.array([10]), bf16_bits(torch.from_numpy(a).to(torch.bfloat16)))
        hits += int(pos[0, 0] == 9)
    p = chi2.cdf(d * (1 - tau) ** 2, d)
    sigma = math.sqrt(p * (1 - p) / trials)
    assert abs(hits / trials - p) < 4 * sigma + 2e-3, (hits / trials, p)


# ----------------------------------------------------------------------------- MAC step
def _run_mac(cfg: WorkloadConfig, wl: Workload, orc: Oracle):
    kvp, bt, slots = host_inputs(wl)
    res = []
    for q_pre, q_rope, kv_lens in wl:
        r = orc.mac_step(slots, kv_lens.numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        full, full_lse = orc.full_decode(kv_lens.numpy(), bf16_bits(q_rope), kvp, bt)
        r["full"], r["full_lse"], r["n"] = full, full_lse, kv_lens.numpy().copy()
        res.append(r)
    return res


def test_threshold_zero_is_exact_full_attention():
    """Sec. 3.2.1: with no match the method falls back to full attention; outputs identical to baseline."""
    cfg = small_cfg(threshold=0.0)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    for r in _run_mac(cfg, wl, orc):
        assert np.all(r["match_pos"] == -1)
        np.testing.assert_allclose(r["out"], r["full"], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(r["lse"], r["full_lse"], rtol=1e-13)
    assert orc.stats.hits == 0 and orc.stats.kv_tokens_read == orc.stats.kv_tokens_full


def test_band_covering_everything_is_exact_full_attention():
    """B >= n: the reused prefix [0, n_p - B) is empty, so even on hits the output is full attention."""
    cfg = small_cfg(threshold=1e6, band=1000)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    res = _run_mac(cfg, wl, orc)
    assert all(np.all(r["match_pos"] >= 0) for r in res[1:])
    for r in res:
        np.testing.assert_allclose(r["out"], r["full"], rtol=1e-12, atol=1e-15)


def test_repeated_identical_query_has_zero_reuse_error():
    """Sec. 3.1: reuse is exact when the logits under Q_m and Q_p agree on the reused prefix.  With RoPE off
    and the same (q_pre, q_rope) at every step, every step after the first hits and equals full attention."""
    cfg = small_cfg(use_rope=False, rho=1.0, threshold=0.5, band=2, window=5, steps=17)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    res = _run_mac(cfg, wl, orc)
    assert np.all(res[0]["match_pos"] == -1)
    for i, r in enumerate(res[1:], 1):
        assert np.all(r["match_pos"] == r["n"][:, None] - 1)          # most recent duplicate
        assert np.all(r["d2"] == 0)
        np.testing.assert_allclose(r["out"], r["full"], rtol=1e-11, atol=1e-14)
    assert orc.stats.hits == (cfg.steps - 1) * cfg.batch * cfg.num_q_heads


def test_zero_keys_give_mean_of_values_whatever_is_reused():
    """All keys zero => every logit is 0 under every query => uniform weights => MAC == full == mean(V) over
    [0, n), hits included (the reused and the fresh parts then carry weights proportional to their sizes).
    Keys that are merely equal would not do: the common logit differs between the cached and the current
    query, which shifts the relative weight of the reused part -- the method's inherent error."""
    cfg = small_cfg(threshold=1e6)
    wl = Workload(cfg)
    wl.kv_pages[:, 0] = 0
    orc = make_oracle(cfg, wl)
    res = _run_mac(cfg, wl, orc)
    assert any(np.any(r["match_pos"] >= 0) for r in res)
    for r in res:
        for b in range(cfg.batch):
            K, V = dense_kv(wl, b, int(r["n"][b]))
            for h in range(cfg.num_q_heads):
                np.testing.assert_allclose(r["out"][b, h], V[:, h // cfg.group].mean(0), rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("band,window,threshold", [(3, 4, 3.0), (0, 3, 4.0), (5, 7, 2.2), (1, 1, 6.0)])
def test_against_literal_definition_with_full_history(band, window, threshold):
    """The C oracle (ring modulo W, shifted (O, LSE), add-only rectification, paged KV) equals the literal
    version (all history filtered by n_p in [n-W, n-1], unshifted (S, Z), rectification by subtraction,
    dense KV, exact rational distances): decisions identical, outputs to rounding.  Runs > 2W steps, so the
    ring wraps several times (Sec. 4.1), and mixes hits and misses."""
    cfg = small_cfg(band=band, window=window, threshold=threshold, steps=max(14, 3 * window), rho=0.93)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = host_inputs(wl)
    Kd = [dense_kv(wl, b, cfg.max_kv_len) for b in range(cfg.batch)]
    lit = [DefinitionMAC(Kd[b][0], Kd[b][1], cfg.num_q_heads, window, band, threshold, orc.sm_scale)
           for b in range(cfg.batch)]
    n_hit = n_miss = 0
    for q_pre, q_rope, kv_lens in wl:
        r = orc.mac_step(slots, kv_lens.numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        for b in range(cfg.batch):
            out, pos = lit[b].step(int(kv_lens[b]), q_pre[b].double().numpy(), q_rope[b].double().numpy())
            np.testing.assert_array_equal(r["match_pos"][b], pos)
            np.testing.assert_allclose(r["out"][b], out, rtol=1e-10, atol=1e-13)
            n_hit += int((pos >= 0).sum())
            n_miss += int((pos < 0).sum())
    assert n_hit > 0 and n_miss > 0, (n_hit, n_miss)


@pytest.mark.parametrize("kw", [dict(max_gap=1), dict(max_gap=2), dict(group_match=True),
                                dict(group_match=True, max_gap=3)])
def test_variants_against_literal_definition(kw):
    """Distance cap (appendix on prefill, recommendation (i)) and one reuse point per KV group, against the literal
    version with exact rational distances on the concatenated group query: decisions identical, outputs to
    rounding; hits and misses both occur."""
    cfg = small_cfg(band=3, window=5, threshold=3.2, steps=24, rho=0.93, num_q_heads=4, num_kv_heads=2)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl, **kw)
    kvp, bt, slots = host_inputs(wl)
    Kd = [dense_kv(wl, b, cfg.max_kv_len) for b in range(cfg.batch)]
    lit = [DefinitionMAC(Kd[b][0], Kd[b][1], cfg.num_q_heads, cfg.window, cfg.band, cfg.threshold, orc.sm_scale, **kw)
           for b in range(cfg.batch)]
    n_hit = n_miss = 0
    for q_pre, q_rope, kv_lens in wl:
        r = orc.mac_step(slots, kv_lens.numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        for b in range(cfg.batch):
            out, pos = lit[b].step(int(kv_lens[b]), q_pre[b].double().numpy(), q_rope[b].double().numpy())
            np.testing.assert_array_equal(r["match_pos"][b], pos)
            np.testing.assert_allclose(r["out"][b], out, rtol=1e-10, atol=1e-13)
            n_hit += int((pos >= 0).sum())
            n_miss += int((pos < 0).sum())
    assert n_hit > 0 and n_miss > 0, (n_hit, n_miss)


def test_distance_cap_only_filters_the_uncapped_decision():
    """The ring of queries does not depend on the decisions (every step inserts its query), so a capped run decides
    exactly like the uncapped run with the hits farther than max_gap turned into misses; a cap of at least W
    changes nothing; max_gap = 0 means no cap."""
    cfg = WorkloadConfig(name="cap", batch=2, num_q_heads=4, num_kv_heads=2, context=60, steps=60, window=16, band=4,
                         threshold=1.6, rho=0.0, head_dim=16, page_size=4, seed=2, period=5, period_std=1.5,
                         query_noise=0.1, jump_prob=0.05)
    runs = {}
    for cap in (0, 3, 16, 1000):
        wl = Workload(cfg)
        orc = make_oracle(cfg, wl, max_gap=cap)
        kvp, bt, slots = host_inputs(wl)
        seq = []
        for q_pre, q_rope, kv_lens in wl:
            r = orc.mac_step(slots, kv_lens.numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
            seq.append((kv_lens.numpy().copy(), r["match_pos"].copy(), r["out"].copy()))
        runs[cap] = seq
    far = 0
    for (n, p0, o0), (_, p3, _), (_, p16, o16), (_, pbig, obig) in zip(runs[0], runs[3], runs[16], runs[1000]):
        gap = n[:, None] - p0
        keep = (p0 >= 0) & (gap <= 3)
        far += int(((p0 >= 0) & (gap > 3)).sum())
        np.testing.assert_array_equal(p3, np.where(keep, p0, -1))
        np.testing.assert_array_equal(p16, p0)
        np.testing.assert_array_equal(pbig, p0)
        np.testing.assert_array_equal(o16, o0)
        np.testing.assert_array_equal(obig, o0)
    assert far > 20          # the cap did remove hits


def test_group_matching_reduces_to_per_head_matching_of_concatenated_queries():
    """One reuse point per KV group == the per-head test applied to the group's queries laid end to end: a pure
    reshape of the query and of the ring ([.., Hq, d] -> [.., Hkv, G*d]) with threshold sqrt(G)*T (G = 4, so that
    (2T)^2 = 4 T^2 exactly).  With G = 1 the two modes are the same function."""
    rng = np.random.default_rng(8)
    Hq, Hkv, d, W = 8, 2, 8, 6
    G = Hq // Hkv
    n_hit = n_miss = 0
    for trial in range(20):
        T = float(np.float32(rng.uniform(2.0, 4.0)))
        grp = Oracle(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=4, window=W, band=2, threshold=T,
                     strides=(1, 1, 1, 1), max_slots=1, group_match=True)
        cat = Oracle(num_q_heads=Hkv, num_kv_heads=Hkv, head_dim=G * d, page_size=4, window=W, band=2, threshold=2 * T,
                     strides=(1, 1, 1, 1), max_slots=1)
        n = 50 + trial
        _fill_ring(grp, rng, n, int(rng.integers(1, 7)))
        if trial % 3 == 0:      # a near-duplicate of a ring entry, so that hits occur
            j = int(np.argmax(grp.ring_npos[0]))
            q = torch.from_numpy(bf16_bits_to_f64(grp.ring_q[0, j])[None] + rng.normal(size=(1, Hq, d)) * 0.3)
        else:
            q = torch.from_numpy(rng.normal(size=(1, Hq, d)))
        qb = bf16_bits(q.float().to(torch.bfloat16))
        cat.ring_q[:] = grp.ring_q.reshape(1, W, Hkv, G * d)
        cat.ring_npos[:] = grp.ring_npos
        pos_g, idx_g, d2_g = grp.match(np.array([0]), np.array([n]), qb)
        pos_c, idx_c, d2_c = cat.match(np.array([0]), np.array([n]), qb.reshape(1, Hkv, G * d))
        np.testing.assert_array_equal(pos_g.reshape(Hkv, G), np.repeat(pos_c.reshape(Hkv, 1), G, axis=1))
        np.testing.assert_array_equal(idx_g.reshape(Hkv, G), np.repeat(idx_c.reshape(Hkv, 1), G, axis=1))
        np.testing.assert_allclose(d2_g.reshape(Hkv, G), np.repeat(d2_c.reshape(Hkv, 1), G, axis=1), rtol=1e-14)
        n_hit += int((pos_g >= 0).sum())
        n_miss += int((pos_g < 0).sum())
    assert n_hit >= 8 and n_miss >= 8, (n_hit, n_miss)
    # G = 1
    a = Oracle(num_q_heads=3, num_kv_heads=3, head_dim=d, page_size=4, window=W, band=2, threshold=3.0,
               strides=(1, 1, 1, 1), max_slots=1, group_match=True)
    b = Oracle(num_q_heads=3, num_kv_heads=3, head_dim=d, page_size=4, window=W, band=2, threshold=3.0,
               strides=(1, 1, 1, 1), max_slots=1)
    _fill_ring(a, rng, 40, 5)
    b.ring_q[:], b.ring_npos[:] = a.ring_q, a.ring_npos
    qb = bf16_bits(torch.from_numpy(rng.normal(size=(1, 3, d)).astype(np.float32)).to(torch.bfloat16))
    for x, y in zip(a.match(np.array([0]), np.array([40]), qb), b.match(np.array([0]), np.array([40]), qb)):
        np.testing.assert_array_equal(x, y)


def test_writeback_holds_rectified_summary_of_this_step():
    """Fig. 1(c) / Sec. 4.2 K3: the entry inserted at length n is prefix (+) fresh[s, n-B) -- checked by
    recomputing it from the pre-step ring and the exported summary/merge; and it sits in slot (n-1) mod W."""
    cfg = small_cfg(threshold=3.5, band=3, window=4, steps=12)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = host_inputs(wl)
    for q_pre, q_rope, kv_lens in wl:
        ring_O, ring_l, ring_n = orc.ring_O.copy(), orc.ring_lse.copy(), orc.ring_npos.copy()
        r = orc.mac_step(slots, kv_lens.numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        for b in range(cfg.batch):
            n = int(kv_lens[b])
            j = (n - 1) % cfg.window
            assert orc.ring_npos[b, j] == n
            np.testing.assert_array_equal(orc.ring_q[b, j], bf16_bits(q_pre)[b])
            for h in range(cfg.num_q_heads):
                n_p = int(r["match_pos"][b, h])
                if n_p >= 0:
                    jj = int(np.where(ring_n[b] == n_p)[0][0])
                    pre, pre_l, s = ring_O[b, jj, h], ring_l[b, jj, h], max(0, n_p - cfg.band)
                else:
                    pre, pre_l, s = np.zeros(cfg.head_dim), -np.inf, 0
                mid, mid_l = orc.summary(bf16_bits(q_rope), kvp, bt, b, h, s, max(s, n - cfg.band))
                exp_O, exp_l = Oracle.merge(pre, pre_l, mid, mid_l)
                np.testing.assert_allclose(orc.ring_O[b, j, h], exp_O, rtol=1e-13, atol=1e-16)
                assert orc.ring_lse[b, j, h] == pytest.approx(exp_l, rel=1e-13) or (exp_l == -np.inf and orc.ring_lse[b, j, h] == -np.inf)


def test_request_without_tokens_changes_nothing_and_gets_the_empty_summary():
    """Sec. 4.1 / Fig. 1(c): ring entries are created at lengths n >= 1 (entry (n - 1) mod W carries the tag n, tag 0 means
    empty).  A request with kv_len = 0 has no key to attend to and no query position to store: its output is the empty
    summary (0, -inf) (Sec. 2: a sum over no keys), every head misses, no ring set changes, and the other requests of
    the batch come out exactly as in a batch without it."""
    cfg = small_cfg(threshold=3.5, band=3, window=4, steps=8)
    wl, wl2 = Workload(cfg), Workload(cfg)
    orc, alone = make_oracle(cfg, wl), make_oracle(cfg, wl2)
    kvp, bt, slots = host_inputs(wl)
    hits = 0
    for q_pre, q_rope, kv_lens in wl:
        lens = kv_lens.numpy().copy()
        lens[0] = 0
        before = [a.copy() for a in (orc.ring_q[0], orc.ring_O[0], orc.ring_lse[0], orc.ring_npos[0])]
        r = orc.mac_step(slots, lens, bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        assert (r["match_pos"][0] == -1).all() and np.isinf(r["d2"][0]).all()
        assert (r["out"][0] == 0).all() and (r["lse"][0] == -np.inf).all()
        for a, b_ in zip(before, (orc.ring_q[0], orc.ring_O[0], orc.ring_lse[0], orc.ring_npos[0])):
            np.testing.assert_array_equal(a, b_)
        assert (orc.ring_npos[0] == 0).all()
        o_full, l_full = orc.full_decode(lens, bf16_bits(q_rope), kvp, bt)
        assert (o_full[0] == 0).all() and (l_full[0] == -np.inf).all()
        # the same step for requests 1.. alone
        r2 = alone.mac_step(slots[1:], lens[1:], bf16_bits(q_pre)[1:], bf16_bits(q_rope)[1:], kvp, bt[1:])
        np.testing.assert_array_equal(r["match_pos"][1:], r2["match_pos"])
        np.testing.assert_array_equal(r["out"][1:], r2["out"])
        hits += int((r2["match_pos"] >= 0).sum())
    assert hits > 0
    st = orc.stats.as_dict()
    assert st["misses"] >= 8 * cfg.num_q_heads and st["kv_tokens_full"] == alone.stats.as_dict()["kv_tokens_full"]


def test_error_falls_as_band_widens():
    """Sec. 5.2 "Insights" (sanity trend, not a pin): with recency-biased logits the error of reuse falls
    as the band grows, and vanishes once the band covers the context."""
    errs = []
    for band in (0, 4, 16, 64, 400):
        cfg = small_cfg(batch=1, num_q_heads=2, num_kv_heads=1, context=200, steps=10, window=8, band=band,
                        threshold=1e6, rho=0.8, head_dim=16, seed=3)
        wl = Workload(cfg)
        # recency bias: scale key t by a factor growing with t so late keys carry most mass
        n_tot = cfg.max_kv_len
        for t in range(n_tot):
            page, within = int(wl.block_table[0, t // cfg.page_size]), t % cfg.page_size
            wl.kv_pages[page, 0, :, within] = (wl.kv_pages[page, 0, :, within].float() * (0.2 + 2.5 * t / n_tot)).to(torch.bfloat16)
        orc = make_oracle(cfg, wl)
        res = _run_mac(cfg, wl, orc)
        errs.append(np.mean([rel_l2(r["out"], r["full"]) for r in res[1:]]))
    assert errs[-1] < 1e-12
    assert errs[0] > errs[2] > errs[-1], errs
    assert errs[1] >= errs[3], errs


def test_stats_definitions():
    """Acceptance rate and skip ratio E[(p - r)_+ / m] with misses as zero (Sec. 5.3), reuse gap, and KV tokens
    streamed per KV group from the smallest start among its heads (Sec. 5.8) -- recomputed in Python."""
    cfg = small_cfg(threshold=3.2, steps=20, window=6)
    wl = Workload(cfg)
    orc = make_oracle(cfg, wl)
    kvp, bt, slots = host_inputs(wl)
    hits = gap = read = full = 0
    skip = 0.0
    for q_pre, q_rope, kv_lens in wl:
        r = orc.mac_step(slots, kv_lens.numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
        for b in range(cfg.batch):
            n = int(kv_lens[b])
            starts = []
            for h in range(cfg.num_q_heads):
                n_p = int(r["match_pos"][b, h])
                s = max(0, n_p - cfg.band) if n_p >= 0 else 0
                starts.append(s)
                if n_p >= 0:
                    hits += 1
                    gap += n - n_p
                    skip += s / n
            for g in range(cfg.num_kv_heads):
                read += n - min(starts[g * cfg.group:(g + 1) * cfg.group])
                full += n
    st = orc.stats
    assert (st.steps, st.head_steps) == (cfg.steps, cfg.steps * cfg.batch * cfg.num_q_heads)
    assert (st.hits, st.misses, st.sum_gap) == (hits, st.head_steps - hits, gap)
    assert (st.kv_tokens_read, st.kv_tokens_full) == (read, full)
    assert st.sum_skip_frac == pytest.approx(skip, rel=1e-12)
    assert 0 < hits < st.head_steps
