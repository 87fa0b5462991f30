"""Oracle brute-force configuration search (Sec. 5.1, brute-force baseline): evaluate every
configuration for an input and keep the fastest.  Works on any latency source -- a table of
measurements or a generating function -- and is the denominator of "% of exhaustive-best".

TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

import math


def argmin_config(latencies) -> tuple[int, float]:
    """latencies: iterable of (config id, latency); NaN/inf entries are infeasible.
    Returns (best id, best latency); ties keep the first (lowest-position) entry."""
    best = None
    for cid, t in latencies:
        if t is None or math.isnan(t) or math.isinf(t):
            continue
        if best is None or t < best[1]:
            best = (cid, t)
    if best is None:
        raise ValueError("no feasible configuration")
    return best


def search(shapes, configs, latency_fn):
    """For each shape evaluate latency_fn(shape, config) for every config; returns
    [(best config, best latency)] in shape order."""
    return [argmin_config((c, latency_fn(s, c)) for c in configs) for s in shapes]


def fraction_of_best(picked_latency: float, best_latency: float) -> float:
    """Throughput of the pick relative to the exhaustive best (= best time / picked time, <= 1)."""
    return best_latency / picked_latency


def geomean(values) -> float:
    """Geometric mean (the paper's aggregate over shapes, Sec. 5.2)."""
    vals = list(values)
    return math.exp(sum(math.log(v) for v in vals) / len(vals))
