"""CPU oracle of the speculation-depth controller (test infrastructure only).

Plain statement of the paper's Section 3.5 (Eq. 8-16, Algorithm 4) in its own notation, in Python
floats (IEEE double).  One `DepthController` is the state of one stream of updates: the flow vector
f of length h, the write index, and the smoothed throughput tau_recent.

Readings taken where the passage is silent or at odds with itself:
 * the acceptance gradient uses the mean of f BEFORE f is updated, the flow magnitude the mean of |f|
   AFTER (the order of Algorithm 4's first three lines);
 * Eq. 10 scales by tau_target / max(tau_recent, 1) while Algorithm 4 uses the throughput t that
   comes in with the metrics, and Eq. 15 projects from tau_recent while Algorithm 4 projects from t:
   the algorithm's version is taken (t in both places); tau_recent is the smoothed state of Eq. 16;
 * the integer depth handed to the verify step is not stated: k = floor(d* + 1/2), then limited to
   the largest depth the kernels are built for (`k_cap`).

Pins: tests/test_oracle_depth.py (first-update closed form, saturation of each factor, clipping,
the geometric closed form of the smoothing, a sequence worked by hand).
"""
from __future__ import annotations

import math
from typing import List, Tuple


class DepthController:
    def __init__(self, h: int = 10, d_base: float = 5.0, gamma: float = 5.0, d_min: float = 2.0,
                 d_max: float = 20.0, tau_target: float = 400.0, tau_recent: float = 0.0, k_cap: int = 20):
        assert h >= 1
        self.h, self.d_base, self.gamma, self.d_min, self.d_max = h, d_base, gamma, d_min, d_max
        self.tau_target, self.tau_recent, self.k_cap = tau_target, tau_recent, k_cap
        self.f: List[float] = [0.0] * h
        self.idx = 0

    def update(self, a: float, l: float, t: float) -> Tuple[float, int, float, int]:
        """One adaptation step from the metrics (accept rate a, load l, throughput t).
        Returns (d_star, b_micro, t_proj, k)."""
        delta = a - sum(self.f) / self.h                          # Eq. 8
        self.f[self.idx] = delta
        self.idx = (self.idx + 1) % self.h
        mag = sum(abs(x) for x in self.f) / self.h                # Eq. 9
        scale = max(1.0, self.tau_target / max(t, 1.0))           # Eq. 10 (Algorithm 4's argument)
        adj = 1.0 - min(l, 0.9)                                   # Eq. 11
        d = self.d_base + (a * mag * self.gamma) * adj * scale    # Eq. 12
        d_star = min(max(d, self.d_min), self.d_max)              # Eq. 13
        b_micro = max(1, math.floor(16 * 5 / d_star))             # Eq. 14
        t_proj = t * (1.0 + a * 0.5)                              # Eq. 15 (Algorithm 4's argument)
        self.tau_recent = 0.9 * self.tau_recent + 0.1 * t_proj    # Eq. 16
        k = min(int(math.floor(d_star + 0.5)), self.k_cap)
        return d_star, b_micro, t_proj, k
