"""HIP-graph capture of the decode step (paper App. B.2 "Auxiliary stream and graphs": capture the steady state
to amortise launches).  All per-step values the kernels need (lengths, slot ids, match results, spans) live in
device memory and the step issues no memset, so one captured graph serves every step: the caller only refreshes
the static input buffers.  Every replay is checked against an eager context fed the same inputs, with eager work
and synchronisations between replays, and the first steps also against the oracle."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2604_00235_amd.workload import CONFIGS, Workload, bf16_bits, scaled

pytestmark = pytest.mark.gpu


def test_graph_replay_matches_eager_every_step():
    from paper_2604_00235_amd import binding as mb
    from tests.gpu_harness import check_rows
    from tests.helpers import make_oracle
    cfg = scaled(CONFIGS["C2"], name="graph", batch=3, context=2500, steps=20, window=8, band=64, threshold=2.8,
                 ragged=37)
    wl = Workload(cfg, device="cuda:0")
    dev = wl.device
    B, Hq, d = cfg.batch, cfg.num_q_heads, cfg.head_dim

    def make():
        mac = mb.MacAttention(num_q_heads=Hq, num_kv_heads=cfg.num_kv_heads, window=cfg.window, band=cfg.band,
                              threshold=cfg.threshold, max_kv_len=cfg.max_kv_len, max_slots=B, chunk_tokens=256)
        bufs = dict(out=torch.zeros((B, Hq, d), dtype=torch.float32, device=dev),
                    lse=torch.zeros((B, Hq), dtype=torch.float32, device=dev),
                    pos=torch.zeros((B, Hq), dtype=torch.int32, device=dev))
        return mac, bufs

    q_pre_s = torch.zeros((B, Hq, d), dtype=torch.bfloat16, device=dev)
    q_rope_s = torch.zeros_like(q_pre_s)
    lens_s = torch.ones((B,), dtype=torch.int32, device=dev)
    eager, eb = make()
    graph, gb = make()
    args_of = lambda mac, bf: mac.make_args(kv_lens=lens_s, q_rope=q_rope_s, kv_pages=wl.kv_pages, strides=wl.strides,
                                            block_table=wl.block_table, out=bf["out"], slot_ids=wl.slot_ids,
                                            q_pre=q_pre_s, out_lse=bf["lse"], match_pos=bf["pos"])
    e_args, g_args = args_of(eager, eb), args_of(graph, gb)

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        graph.decode_step(g_args, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert graph.stats()["steps"] == 0                      # capturing runs nothing

    orc = make_oracle(cfg, wl)
    kvp, bt, slots = bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()
    hits = 0
    for s, (q_pre, q_rope, kv_lens) in enumerate(wl):
        q_pre_s.copy_(q_pre); q_rope_s.copy_(q_rope); lens_s.copy_(kv_lens)
        eager.decode_step(e_args, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        junk = (eb["out"] * 2).sum()                        # unrelated eager work between replays
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(gb["pos"], eb["pos"]), f"step {s}: decisions"
        assert torch.equal(gb["out"], eb["out"]) and torch.equal(gb["lse"], eb["lse"]), f"step {s}: replay != eager"
        hits += int((gb["pos"] >= 0).sum())
        if s < 8:
            ref = orc.mac_step(slots, kv_lens.cpu().numpy(), bf16_bits(q_pre), bf16_bits(q_rope), kvp, bt)
            assert np.array_equal(gb["pos"].cpu().numpy(), ref["match_pos"])
            check_rows(gb["out"].cpu().numpy(), ref["out"], f"graph step {s}")
    se, sg = eager.stats(), graph.stats()
    assert se == sg and sg["steps"] == cfg.steps and 0 < hits < sg["head_steps"]
    eager.close(); graph.close()
