"""The load-only streaming probe (include/mac_probe.h) on the GPU: it runs, and what it reports is a bandwidth."""
from __future__ import annotations

import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("segment,shuffle,non_temporal", [(4096, False, True), (4096, True, True), (2048, True, False), (16384, True, True)])
def test_probe_reports_a_plausible_rate(segment, shuffle, non_temporal):
    import torch
    from paper_2604_00235_amd import binding as mb
    total = 1 << 30                                     # well beyond the 256 MB last-level cache
    buf = torch.ones(total // 4, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    n = total // segment
    gen = torch.Generator(device="cpu")
    gen.manual_seed(3)
    order = (torch.randperm(n, generator=gen) if shuffle else torch.arange(n)).to(torch.int32).to("cuda:0")
    torch.cuda.synchronize()
    us = mb.mac_probe_stream(buf.data_ptr(), order.data_ptr(), n, segment, non_temporal, 512, 5, sink.data_ptr(),
                             torch.cuda.current_stream().cuda_stream)
    tbps = total / us / 1e6
    assert 0.5 < tbps < 8.4, f"{tbps:.2f} TB/s"          # between a tenth of the chip's memory rate and its published peak
    assert int(sink.sum().item()) == 0                     # the xor of the loads never equals the sentinel for this buffer
