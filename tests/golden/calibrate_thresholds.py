"""Writes tests/golden/c3_thresholds.json: thresholds T for the 128K sweep (BASELINE configs[2]) that give
about 20 / 50 / 90 % per-head hit rates on the seeded AR(1) query streams with rho = 0.90 / 0.97 / 0.99.

Calls only the CPU oracle's matcher (oracle/): for every step and head the squared distance to the nearest
ring entry is recorded (rings start empty; the first step has no candidate), and T is the square root of the
target quantile.  The values are copied by hand into paper_2604_00235_amd/workload.py (C3_THRESHOLDS),
rounded to 3 significant digits; test_workload_thresholds checks they still agree.

    python tests/golden/calibrate_thresholds.py
"""
from __future__ import annotations

import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.mac_oracle import Oracle                                    # noqa: E402
from paper_2604_00235_amd.workload import CONFIGS, Workload, bf16_bits   # noqa: E402

TARGETS = {"C3_rho90": 0.20, "C3_rho97": 0.50, "C3_rho99": 0.90}


def nearest_d2(cfg_name: str) -> np.ndarray:
    cfg = CONFIGS[cfg_name]
    wl = Workload(cfg, queries_only=True)
    orc = Oracle(num_q_heads=cfg.num_q_heads, num_kv_heads=cfg.num_kv_heads, head_dim=cfg.head_dim,
                 page_size=cfg.page_size, window=cfg.window, band=cfg.band, threshold=1e30,
                 strides=wl.strides, max_slots=cfg.batch)
    slots = wl.slot_ids.numpy()
    vals = []
    for q_pre, _, kv_lens in wl:
        lens = kv_lens.numpy()
        qb = bf16_bits(q_pre)
        _, _, d2 = orc.match(slots, lens, qb)
        vals.append(d2[np.isfinite(d2)])
        for b in range(cfg.batch):                 # ring insert (plumbing): slot (n-1) mod W, tag n
            j = (int(lens[b]) - 1) % cfg.window
            orc.ring_q[slots[b], j] = qb[b]
            orc.ring_npos[slots[b], j] = lens[b]
    return np.concatenate(vals)


def main():
    out = {}
    for name, target in TARGETS.items():
        d2 = nearest_d2(name)
        T = float(np.sqrt(np.quantile(d2, target)))
        out[name] = {"rho": CONFIGS[name].rho, "target_hit_rate": target, "threshold": T,
                     "samples": int(d2.size)}
        print(name, out[name])
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "c3_thresholds.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
