"""Literal, tiny-shape version of the method, used to pin oracle/mac_oracle.c.  TEST INFRASTRUCTURE ONLY.

Differences from the C oracle, on purpose, so that the two do not share a mistake:
  * works on dense float64 K, V arrays [tokens, Hkv, d] (no pages, no block table);
  * keeps the *unshifted* sums (S, Z) of Sec. 3.1 -- valid for the small logits of the tests;
  * obtains the stored summary by subtracting the last-B band from the step's total
    (Fig. 1(c): "online subtraction"), not by adding prefix and middle part;
  * keeps the whole history of inserted entries, and selects the window by n_p in [n-W, n-1],
    instead of a ring indexed modulo W (Sec. 4.1);
  * squared distances can be evaluated in exact rational arithmetic;
  * the two matching variants are written from their statement, not from the C code: the distance cap tests the
    gap n - n_p of the nearest candidate after the threshold; group matching concatenates the group's queries
    into one vector of G*d elements and compares its squared distance with G*T^2.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Optional

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 values (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def unshifted_summary(q: np.ndarray, K: np.ndarray, V: np.ndarray, lo: int, hi: int, scale: float):
    """(S, Z) of Sec. 3.1 over keys [lo, hi): S = sum e^{l_t} v_t, Z = sum e^{l_t}, l_t = scale * q.k_t."""
    d = q.shape[0]
    S = np.zeros(d)
    Z = 0.0
    for t in range(lo, hi):
        w = np.exp(scale * float(np.dot(q, K[t])))
        S = S + w * V[t]
        Z = Z + w
    return S, Z


def exact_sq_dist(a: np.ndarray, b: np.ndarray) -> Fraction:
    """sum (a_i - b_i)^2 in exact rational arithmetic (inputs are floats that are exactly representable)."""
    tot = Fraction(0)
    for x, y in zip(a.tolist(), b.tolist()):
        diff = Fraction(x) - Fraction(y)
        tot += diff * diff
    return tot


class DefinitionMAC:
    """One request, all heads; K, V given densely for the whole run."""

    def __init__(self, K: np.ndarray, V: np.ndarray, num_q_heads: int, window: int, band: int,
                 threshold: float, scale: float, exact_match: bool = True, max_gap: int = 0,
                 group_match: bool = False):
        self.K, self.V = K, V                    # [tokens, Hkv, d] float64
        self.Hq = num_q_heads
        self.Hkv = K.shape[1]
        self.G = self.Hq // self.Hkv
        self.W, self.B = window, band
        self.T = float(np.float32(threshold))
        self.scale = float(np.float32(scale))
        self.exact = exact_match
        self.max_gap, self.group_match = max_gap, group_match
        self.history: List[dict] = []            # every inserted entry, never evicted

    def step(self, n: int, q_pre: np.ndarray, q_rope: np.ndarray):
        """q_pre, q_rope: [Hq, d] float64 (exact images of the bf16 inputs).  Returns (out [Hq,d], match_pos [Hq])."""
        Hq, d = q_pre.shape
        out = np.zeros((Hq, d))
        pos = np.full(Hq, -1, np.int64)
        new_entry = {"n_p": n, "q": q_pre.copy(), "S": np.zeros((Hq, d)), "Z": np.zeros(Hq)}
        cands = [e for e in self.history if n - self.W <= e["n_p"] <= n - 1]
        T2 = Fraction(self.T) * Fraction(self.T) if self.exact else self.T * self.T
        for h in range(Hq):
            g = h // self.G
            # the vectors compared: this head's query, or the whole group's queries laid end to end
            hs = slice(g * self.G, (g + 1) * self.G) if self.group_match else slice(h, h + 1)
            nh = self.G if self.group_match else 1
            best = None
            best_d2 = None
            for e in cands:
                a, c = q_pre[hs].reshape(-1), e["q"][hs].reshape(-1)
                if self.exact:
                    d2 = exact_sq_dist(a, c)
                else:
                    d2 = float(np.sum((a - c) ** 2))
                if best is None or d2 < best_d2 or (d2 == best_d2 and e["n_p"] > best["n_p"]):
                    best, best_d2 = e, d2
            hit = best is not None and best_d2 < nh * T2
            if hit and self.max_gap > 0:
                hit = n - best["n_p"] <= self.max_gap
            if hit:
                n_p = best["n_p"]
                s = max(0, n_p - self.B)
                S_pre, Z_pre = best["S"][h], best["Z"][h]
                pos[h] = n_p
            else:
                s = 0
                S_pre, Z_pre = np.zeros(d), 0.0
            Kg, Vg = self.K[:, g, :], self.V[:, g, :]
            # Eq. (rect-recomp): band + tail under the current query; Eq. (rect-merge): add and divide
            S_fresh, Z_fresh = unshifted_summary(q_rope[h], Kg, Vg, s, n, self.scale)
            S_tot, Z_tot = S_pre + S_fresh, Z_pre + Z_fresh
            out[h] = S_tot / Z_tot
            # Fig. 1(c): remove the last-B band (recomputed under this query) from the step's total
            nb = max(s, n - self.B)
            S_band, Z_band = unshifted_summary(q_rope[h], Kg, Vg, nb, n, self.scale)
            new_entry["S"][h] = S_tot - S_band
            new_entry["Z"][h] = Z_tot - Z_band
        self.history.append(new_entry)
        return out, pos
