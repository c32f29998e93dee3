"""Pure-Python brute force of Eq. 3 for tiny layers (TEST INFRASTRUCTURE ONLY).

Written with explicit loops over tokens, experts and hidden units and Python
floats, independently of `moe_reference`, so that the two can be checked against
each other.  Only for E <= 6 or so, a handful of tokens and hidden units.
"""
from __future__ import annotations

import itertools
import math


def _route(token_logits, candidates, count):
    """The `count` candidates with the largest logits (ties: lower index) and their Eq. 1 weights."""
    ranked = sorted(candidates, key=lambda e: (-token_logits[e], e))[:count]
    top = max(token_logits[e] for e in ranked)
    ex = {e: math.exp(token_logits[e] - top) for e in ranked}
    den = sum(ex.values())
    return {e: ex[e] / den for e in ranked}


def _mix(weights, Y, t, H):
    return [sum(w * Y[e][t][h] for e, w in weights.items()) for h in range(H)]


def brute_force_enumerate(logits, Y, k, r):
    """loss[i] = sum_t || F'(x_t, C_i) - F(x_t) ||^2 for every r-subset C_i (Sec. 3.2, Eq. 3).

    logits: T lists of E floats; Y: E lists of T lists of H floats.
    Returns (losses, kept_sets) in the order of itertools.combinations.
    """
    E = len(Y)
    T = len(logits)
    H = len(Y[0][0]) if T else 0
    kept_sets = list(itertools.combinations(range(E), r))
    losses = []
    for kept in kept_sets:
        total = 0.0
        for t in range(T):
            row = [float(v) for v in logits[t]]
            full = _mix(_route(row, range(E), min(k, E)), Y, t, H)
            pruned = _mix(_route(row, kept, min(k, r)), Y, t, H)
            total += sum((p - f) ** 2 for p, f in zip(pruned, full))
        losses.append(total)
    return losses, kept_sets
