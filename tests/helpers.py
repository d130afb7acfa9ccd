"""Small helpers shared by the tests (input plumbing only)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2604_00235_amd.workload import Workload, WorkloadConfig, bf16_bits


def dense_kv(wl: Workload, b: int, ntok: int):
    """Gather request b's K and V rows [ntok, Hkv, d] as float64 from the paged cache."""
    cfg = wl.cfg
    ps = cfg.page_size
    npages = (ntok + ps - 1) // ps
    phys = wl.block_table[b, :npages].long()
    pages = wl.kv_pages[phys]                       # [npages, 2, Hkv, ps, d]
    K = pages[:, 0].permute(0, 2, 1, 3).reshape(npages * ps, cfg.num_kv_heads, cfg.head_dim)[:ntok]
    V = pages[:, 1].permute(0, 2, 1, 3).reshape(npages * ps, cfg.num_kv_heads, cfg.head_dim)[:ntok]
    return K.double().cpu().numpy(), V.double().cpu().numpy()


def make_oracle(cfg: WorkloadConfig, wl: Workload, **over):
    from oracle.mac_oracle import Oracle
    kw = dict(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, head_dim=cfg.head_dim,
              page_size=cfg.page_size, window=cfg.window, band=cfg.band, threshold=cfg.threshold,
              strides=wl.strides, max_slots=cfg.batch)
    kw.update(over)
    return Oracle(**kw)


def host_inputs(wl: Workload):
    return bf16_bits(wl.kv_pages), wl.block_table.cpu().numpy(), wl.slot_ids.cpu().numpy()


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))
