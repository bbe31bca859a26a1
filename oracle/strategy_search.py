"""Exhaustive search over virtual tensor strategies (test infrastructure; plain Python, tiny graphs).

Sec. 5.2 poses the choice of a points-to graph as maximising the latency saving l(C) over all
conflict-free edge sets C of the opportunity graph, and solves it greedily.  This module is the
plain definition: enumerate every assignment "tensor -> none or one of its bundles", keep the
ones that are points-to graphs (each tensor in at most one bundle, every chain of edges ends at a
physical tensor), evaluate l on each, return the best.  Bundles are given as plain tuples
``(tensor, targets)``; nothing is shared with the product's implementation.
"""
from __future__ import annotations

import itertools


def valid(choice):
    """choice: dict tensor -> targets.  No cycle when following tensor -> targets."""
    state = {}

    def grounded(t):
        if t not in choice:
            return True
        if state.get(t) == "open":
            return False
        if state.get(t) == "done":
            return True
        state[t] = "open"
        ok = all(grounded(x) for x in choice[t])
        state[t] = "done"
        return ok

    return all(grounded(t) for t in choice)


def all_strategies(bundles):
    """bundles: dict tensor -> list of target tuples.  Yields every valid dict tensor -> targets."""
    tensors = sorted(bundles)
    options = [[None] + list(bundles[t]) for t in tensors]
    for pick in itertools.product(*options):
        choice = {t: p for t, p in zip(tensors, pick) if p is not None}
        if valid(choice):
            yield choice


def best_strategy(bundles, saving):
    """saving(choice) -> float.  Returns (best choice, its saving, number of valid strategies)."""
    best, best_s, n = {}, saving({}), 0
    for c in all_strategies(bundles):
        n += 1
        s = saving(c)
        if s > best_s:
            best, best_s = c, s
    return best, best_s, n
