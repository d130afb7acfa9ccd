"""The entry point that allocates nothing, mac_attn_full_decode_static (for callers that cannot call hipMalloc),
through the C ABI: its output must equal mac_attn_full_decode's (same kernels, same chunking: bit for bit; and both
within the output tolerance of the oracle), on two calls in a row, the second with a smaller input that reuses the
front of the static buffer while the rest still holds the first call's partials.  Free device memory must not move
across the calls."""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_00235_amd.workload import CONFIGS, Workload, bf16_bits, scaled

pytestmark = pytest.mark.gpu


def _static_call(mb, cfg, wl, q_rope, kv_lens, out, lse, chunk):
    geo = mb.mac_attn_static_geometry(0, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.page_size, 0.0,
                                      cfg.max_kv_len, chunk, 0)
    sp, skv, sh, st = wl.strides
    args = mb.mac_attn_step_args(q_rope.shape[0], None, kv_lens.data_ptr(), None, q_rope.data_ptr(),
                                 wl.kv_pages.data_ptr(), sp, skv, sh, st, wl.block_table.data_ptr(),
                                 int(wl.block_table.stride(0)), out.data_ptr(), lse.data_ptr(), None, None)
    mb.mac_attn_full_decode_static(geo, args, torch.cuda.current_stream().cuda_stream)


def test_static_full_decode_equals_context_full_decode_twice():
    from paper_2604_00235_amd import binding as mb
    from tests.gpu_harness import DeviceRun, check_rows, say
    from tests.helpers import make_oracle
    # first call: 3 requests x 32/8 heads near 5000 tokens (ragged), 20 work items per group; second: 2 requests of a
    # different geometry (MQA-like 16/1 heads, head dimension 64) near 700 tokens
    big = scaled(CONFIGS["C2"], name="static_big", batch=3, context=5000, steps=2, ragged=333)
    small = scaled(CONFIGS["C4_hit"], name="static_small", batch=2, num_q_heads=16, context=700, steps=2, ragged=41, head_dim=64)
    for rep in range(2):                                   # the pair twice: the buffer is dirty from every earlier call
        for cfg, chunk in ((big, 256), (small, 128)):
            say(f"[static] rep {rep} {cfg.name}: batch={cfg.batch} Hq/Hkv={cfg.num_q_heads}/{cfg.num_kv_heads} "
                f"context={cfg.context} chunk={chunk}")
            wl = Workload(cfg, device="cuda:0")
            run = DeviceRun(cfg, wl, chunk_tokens=chunk)
            orc = make_oracle(cfg, wl)
            kvp, bt = bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy()
            out = torch.full((cfg.batch, cfg.num_q_heads, cfg.head_dim), float("nan"), device="cuda:0")
            lse = torch.full((cfg.batch, cfg.num_q_heads), float("nan"), device="cuda:0")
            for q_pre, q_rope, kv_lens in wl:
                ref_out, ref_lse = run.full(q_rope, kv_lens)
                torch.cuda.synchronize()
                free0 = torch.cuda.mem_get_info()[0]
                _static_call(mb, cfg, wl, q_rope, kv_lens, out, lse, chunk)
                torch.cuda.synchronize()
                assert torch.cuda.mem_get_info()[0] == free0, "device memory was allocated or freed by the call"
                assert np.array_equal(out.cpu().numpy(), ref_out) and np.array_equal(lse.cpu().numpy(), ref_lse)
                o_out, o_lse = orc.full_decode(kv_lens.cpu().numpy(), bf16_bits(q_rope), kvp, bt)
                check_rows(out.cpu().numpy(), o_out, f"{cfg.name} static full decode")
                assert np.abs(lse.cpu().numpy() - o_lse).max() < 1e-3
            run.mac.close()


def test_static_full_decode_rejects_what_does_not_fit():
    from paper_2604_00235_amd import binding as mb
    lib = mb.load_library()
    # 128 heads x 4 requests x ceil(131200 / 32) work items x 516 B = 1 GB of partials: beyond the static buffer
    geo = mb.mac_attn_static_geometry(0, 32, 8, 128, 16, 0.0, 131200, 32, 0)
    t = torch.zeros(64, device="cuda:0", dtype=torch.int32)
    q = torch.zeros((4, 32, 128), device="cuda:0", dtype=torch.bfloat16)
    kv = torch.zeros((1, 2, 8, 16, 128), device="cuda:0", dtype=torch.bfloat16)
    bt = torch.zeros((4, 8200), device="cuda:0", dtype=torch.int32)
    out = torch.zeros((4, 32, 128), device="cuda:0")
    args = mb.mac_attn_step_args(4, None, t.data_ptr(), None, q.data_ptr(), kv.data_ptr(), 2 * 8 * 16 * 128, 8 * 16 * 128,
                                 16 * 128, 128, bt.data_ptr(), 8200, out.data_ptr(), None, None, None)
    assert lib.mac_attn_full_decode_static(C.byref(geo), C.byref(args), None) == mb.MAC_ATTN_ERR_TOO_LARGE
    assert b"static" in lib.mac_attn_strerror(mb.MAC_ATTN_ERR_TOO_LARGE)
    geo.head_dim = 256
    assert lib.mac_attn_full_decode_static(C.byref(geo), C.byref(args), None) == mb.MAC_ATTN_ERR_UNSUPPORTED
    assert lib.mac_attn_full_decode_static(None, C.byref(args), None) == mb.MAC_ATTN_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert float(out.abs().sum()) == 0.0                     # nothing was enqueued


def test_static_full_decode_with_the_default_item_size():
    """chunk_tokens = 0 in the geometry: the item size comes from the host rule the header states (a power of two in
    [512, 2048] from batch * Hkv * max_kv_len / 2048, at least 64 G): 512 tokens for 3 x 8 groups of ~5300 tokens.  Same
    bits as a context with that item size fixed."""
    from paper_2604_00235_amd import binding as mb
    from tests.gpu_harness import DeviceRun
    cfg = scaled(CONFIGS["C2"], name="static_default", batch=3, context=5000, steps=2, ragged=333)
    wl = Workload(cfg, device="cuda:0")
    run = DeviceRun(cfg, wl, chunk_tokens=512)
    out = torch.full((cfg.batch, cfg.num_q_heads, cfg.head_dim), float("nan"), device="cuda:0")
    lse = torch.full((cfg.batch, cfg.num_q_heads), float("nan"), device="cuda:0")
    for q_pre, q_rope, kv_lens in wl:
        ref_out, ref_lse = run.full(q_rope, kv_lens)
        _static_call(mb, cfg, wl, q_rope, kv_lens, out, lse, 0)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref_out) and np.array_equal(lse.cpu().numpy(), ref_lse)
    run.mac.close()
