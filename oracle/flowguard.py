"""CPU oracle of the metric-aware router's worker selection (test infrastructure only).

Plain statement of the paper's Section 3.2 (Eq. 1-4, Algorithm 2) in Python floats (IEEE double).

Readings taken where the passage is silent or at odds with itself:
 * Eq. 1 takes the memory utilisation M_w in [0,1] while Eq. 3 divides M_w by 100, i.e. reads it in
   per cent: a worker reports one number m in [0,1]; Eq. 1 uses m, Eq. 3 uses (100 m)/100 = m;
 * Eq. 1's normalised queue depth is Q_w = min(depth / Q_max, 1), Eq. 3 uses depth / Q_max unclipped;
 * argmax and argmin take the lowest index among equals; the fallback considers every worker, stale
   or not (Algorithm 2 takes the argmin over all i).

Pins: tests/test_oracle_flowguard.py (scores and thresholds worked by hand, each branch of the algorithm).
"""
from __future__ import annotations

from typing import Sequence, Tuple

ALPHA = (0.4, 0.1, 0.3, 0.2)   # the paper's weights: cache reuse, memory, queue, load
TAU = 0.85                      # overload threshold


def score(cache_hit: float, mem: float, depth: float, load: float, q_max: float,
          alpha: Sequence[float] = ALPHA) -> float:
    q = min(depth / q_max, 1.0)
    return alpha[0] * cache_hit + alpha[1] * (1.0 - mem) + alpha[2] * (1.0 - q) + alpha[3] * (1.0 - load)   # Eq. 1


def overload_score(mem: float, depth: float, q_max: float) -> float:
    return mem + 2.0 * depth / q_max                                                                          # Eq. 3


def select(workers: Sequence[Tuple[float, float, float, float, bool]], q_max: float,
           alpha: Sequence[float] = ALPHA, tau: float = TAU) -> int:
    """workers[i] = (cache_hit, mem, queue depth, load, stale).  Returns the chosen worker's index."""
    best, best_score = -1, 0.0
    for i, (c, m, d, l, stale) in enumerate(workers):
        if stale or overload_score(m, d, q_max) > tau:                                                        # Eq. 2
            continue
        s = score(c, m, d, l, q_max, alpha)
        if best < 0 or s > best_score:
            best, best_score = i, s
    if best >= 0:
        return best
    depths = [w[2] for w in workers]                                                                          # Eq. 4
    return depths.index(min(depths))
