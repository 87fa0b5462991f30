"""Oracle wave-aware piecewise bilinear modelling (Sec. 4.3) and extrapolation (Sec. 4.5).

Input: profiling records <key, micro, G, L, w, mean latency> (Sec. 4.2, profiling output).
Output: a DualTable -- coefficient table <key, w> -> (alpha, beta, gamma, delta) plus one
extrapolation tuple per key, and the anchor micro table <key, w, L> -> micro (plus ext).

"key" is the structural (macro) configuration: every parameter that fixes G, L and the number
of co-resident blocks; "micro" is what is left (Sec. 4.1).

TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

from collections import defaultdict
from dataclasses import dataclass, field
from typing import NamedTuple, Optional

import numpy as np


class Sample(NamedTuple):
    key: int
    micro: int
    G: int
    L: int
    w: int
    us: float
    fam: int = 0     # 0: near-square grid (the paper's sampler); 1, 2, 3: grids of 1, 2, 4 tile rows (extension)


class KeyDesc(NamedTuple):
    bm: int
    bn: int
    bk: int
    nwave: int
    stages: int
    occ: int
    cap: int
    split: int = 1   # S blocks per output tile along K


@dataclass
class Bucket:
    theta: tuple = (0.0, 0.0, 0.0, 0.0)   # alpha, beta, gamma, delta
    status: int = 0                        # 0: no model; else bit0..3 = alpha..delta identified
    anchors: list = field(default_factory=list)   # [(L, micro)] ascending in L


@dataclass
class DualTable:
    W: int
    keys: list            # [KeyDesc]
    local: list           # local[key][w-1] -> Bucket
    ext: list             # ext[key] -> Bucket
    W_row: int = 0        # few-row families (extension): profiled waves, 0 = absent
    row_local: list = field(default_factory=list)   # row_local[fam-1][key][w-1] -> Bucket, fam = 1..row_fams
    row_ext: list = field(default_factory=list)     # row_ext[fam-1][key] -> Bucket
    row_mode: int = 0     # 0: family f holds grids of 1, 2, 4 tile rows and is consulted per key by the shape's tile rows;
                          # 1: family f holds matrices of 16, 32, 64, 128 rows and is consulted by the shape's M for all keys
    # feasibility limits of whatever runs the split-K keys (floats of partial tiles per launch, output
    # tiles per launch); None = unlimited.  Not part of the method: set by the caller (see geometry.split_fits)
    ws_elems: Optional[int] = None
    max_split_tiles: Optional[int] = None

    @property
    def row_fams(self) -> int:
        return len(self.row_local)


def shared_micro(records) -> Optional[tuple[int, list]]:
    """Sec. 4.3: for one <key, w, L> group (or one <key, L> group of the merged ext waves) pick
    the micro with the smallest latency averaged over the group's sampled grid sizes; return
    (micro, [(G, L, us)] of that micro).  A micro lacking a record for any grid size of the
    group is ineligible; ties go to the lowest micro id.  None when no micro is eligible.
    """
    grid = {r.G for r in records}
    by_micro = defaultdict(list)
    for r in records:
        by_micro[r.micro].append(r)
    best = None
    for micro in sorted(by_micro):
        rs = by_micro[micro]
        if {r.G for r in rs} != grid:
            continue
        mean = sum(r.us for r in rs) / len(rs)
        if best is None or mean < best[0]:
            best = (mean, micro, rs)
    if best is None:
        return None
    return best[1], [(r.G, r.L, r.us) for r in best[2]]


def fit_bilinear(rows, relative: bool = False) -> tuple[tuple, int]:
    """Least squares of T ~ alpha*G*L + beta*G + gamma*L + delta (Sec. 4.3, bucket
    model; Sec. 5.1 "least-squares regression").  rows = [(G, L, T)].

    relative = False: ordinary least squares, the sum of (That - T)^2 -- the paper as written.
    relative = True: the sum of ((That - T)/T)^2, i.e. every equation of the system divided by its measured T
    (a reading for loop-anchor sets much wider than the paper's [1024, 5120], where a bucket's latencies span
    two orders of magnitude; needs T > 0).

    Solved in centred, scaled variables u=(G-g0)/sg, v=(L-l0)/sl (on a product grid the columns
    uv, u, v, 1 are mutually orthogonal), then mapped back.  With a single distinct G (or L) the
    terms that cannot be identified are dropped and their coefficients set to 0.
    Returns ((alpha, beta, gamma, delta), status bitmask).
    """
    if not rows:
        return (0.0, 0.0, 0.0, 0.0), 0
    G = np.array([r[0] for r in rows], dtype=np.float64)
    L = np.array([r[1] for r in rows], dtype=np.float64)
    T = np.array([r[2] for r in rows], dtype=np.float64)
    nG, nL = len(set(G.tolist())), len(set(L.tolist()))
    g0, l0 = float(G.mean()), float(L.mean())
    sg = float(np.max(np.abs(G - g0))) or 1.0
    sl = float(np.max(np.abs(L - l0))) or 1.0
    u, v, one = (G - g0) / sg, (L - l0) / sl, np.ones_like(G)
    if relative:
        if not (T > 0).all():
            raise ValueError("relative residuals need positive latencies")
        scale = 1.0 / T      # each equation x.theta = T becomes (x/T).theta = 1
    else:
        scale = np.ones_like(T)

    def solve(columns):
        X = np.stack(columns, axis=1) * scale[:, None]
        return np.linalg.lstsq(X, T * scale, rcond=None)[0]

    a = b = c = 0.0
    if nG >= 2 and nL >= 2:
        sol = solve([u * v, u, v, one])
        a, b, c, d = (float(x) for x in sol)
        status = 0b1111
    elif nG >= 2:
        sol = solve([u, one])
        b, d = float(sol[0]), float(sol[1])
        status = 0b1010
    elif nL >= 2:
        sol = solve([v, one])
        c, d = float(sol[0]), float(sol[1])
        status = 0b1100
    else:
        # the minimiser of sum((d - T)^2) is the mean; of sum(((d - T)/T)^2) it is sum(1/T) / sum(1/T^2)
        d = float(np.sum(1.0 / T) / np.sum(1.0 / T ** 2)) if relative else float(T.mean())
        status = 0b1000
    alpha = a / (sg * sl)
    beta = b / sg - a * l0 / (sg * sl)
    gamma = c / sl - a * g0 / (sg * sl)
    delta = d - b * g0 / sg - c * l0 / sl + a * g0 * l0 / (sg * sl)
    return (alpha, beta, gamma, delta), status


def thin_anchors(anchors: list, limit=None) -> list:
    """Reading for buckets with more loop counts than a table has room for (attention grids: each grid size has its
    own KV lengths): keep the anchors at ranks floor(i*(n-1)/(limit-1)), i = 0..limit-1 -- the smallest, the
    largest and an even spread between them.  The fit still uses every loop count's rows.  limit = None (the
    method as the paper states it) keeps every anchor; a table format's capacity is the caller's to pass in."""
    n = len(anchors)
    if limit is None or n <= limit:
        return list(anchors)
    if limit < 2:
        raise ValueError("limit >= 2")
    return [anchors[(i * (n - 1)) // (limit - 1)] for i in range(limit)]


def _fit_group(records, max_anchors=None, relative: bool = False) -> Bucket:
    """Shared micro per L, then one bilinear fit over the chosen micros' rows."""
    by_L = defaultdict(list)
    for r in records:
        by_L[r.L].append(r)
    rows, anchors = [], []
    for L in sorted(by_L):
        pick = shared_micro(by_L[L])
        if pick is None:
            continue
        anchors.append((L, pick[0]))
        rows.extend(pick[1])
    theta, status = fit_bilinear(rows, relative)
    return Bucket(theta=theta, status=status, anchors=thin_anchors(anchors, max_anchors))


def fit_step(records, cap: int):
    """Ablation "Step" (Sec. 5.4): latency depends on the wave count only, T = w * (a*L + b) with
    w = ceil(G/cap) -- the classical T_wave * ceil(G/N) model (Sec. 3.2) with a per-iteration and a
    fixed cost per wave.  Shared micro per L over all records, then least squares on (w*L, w).
    Returns (a, b, anchors)."""
    by_L = defaultdict(list)
    for r in records:
        by_L[r.L].append(r)
    X, y, anchors = [], [], []
    for L in sorted(by_L):
        pick = shared_micro(by_L[L])
        if pick is None:
            continue
        anchors.append((L, pick[0]))
        for (G, Lr, us) in pick[1]:
            w = -(-G // cap)
            X.append([w * Lr, w])
            y.append(us)
    if not X:
        return 0.0, 0.0, anchors
    X, y = np.array(X, dtype=np.float64), np.array(y, dtype=np.float64)
    if len({row[0] / row[1] for row in X.tolist()}) >= 2:
        scale = np.max(np.abs(X), axis=0)
        sol = np.linalg.lstsq(X / scale, y, rcond=None)[0] / scale
        return float(sol[0]), float(sol[1]), anchors
    return 0.0, float(np.sum(X[:, 1] * y) / np.sum(X[:, 1] ** 2)), anchors


MODEL_WAVE_BILINEAR, MODEL_LINEAR, MODEL_STEP = 0, 1, 2


def fit_tables(samples, keys, W: int, p: int, model: int = MODEL_WAVE_BILINEAR, W_row: int = 0,
               row_fams: int = 1, max_anchors=None, relative: bool = False, row_mode: int = 0) -> DualTable:
    """Build the dual table (Sec. 4.3) with per-key extrapolation entries fitted on the merged
    samples of the last p profiled waves, max(1, W-p+1)..W (Sec. 4.5).  Samples with w > W are
    ignored.  max_anchors: anchor slots per bucket of the table being imitated (see thin_anchors; None = all).
    relative: the objective of every bilinear bucket fit (see fit_bilinear); the Step ablation is always absolute.

    model selects the ablations of Sec. 5.4 expressed in the same table form:
      LINEAR  no wave buckets; one bilinear tuple per key fitted on all waves (stored as the
              extrapolation entry, which every query then uses);
      STEP    T = w*(a*L + b): bucket w holds (0, 0, a*w, b*w); beyond W the step function is
              continued by its linear envelope (a/cap, b/cap, 0, 0).
    """
    samples = [Sample(*s) for s in samples]
    if W_row > 0:
        # every few-row family is a further, independent set of buckets built the same way
        # (wave buckets 1..W_row, extrapolation from the last min(p, W_row) of them)
        t = fit_tables([s for s in samples if s.fam == 0], keys, W, p, model, max_anchors=max_anchors, relative=relative)
        t.W_row = W_row
        t.row_mode = row_mode     # only says how the families are consulted; each is fitted from its records alike
        for f in range(1, row_fams + 1):
            rows_t = fit_tables([s._replace(fam=0) for s in samples if s.fam == f], keys, W_row, min(p, W_row),
                                max_anchors=max_anchors, relative=relative)
            t.row_local.append(rows_t.local)
            t.row_ext.append(rows_t.ext)
        return t
    samples = [s for s in samples if s.fam == 0]
    if model == MODEL_LINEAR:
        t = fit_tables(samples, keys, W, W, MODEL_WAVE_BILINEAR, max_anchors=max_anchors, relative=relative)
        for k in range(len(keys)):
            t.local[k] = [Bucket() for _ in range(W)]
        return t
    if model == MODEL_STEP:
        per_key = defaultdict(list)
        for s in samples:
            s = Sample(*s)
            if 1 <= s.w <= W:
                per_key[s.key].append(s)
        local, ext = [], []
        for k, kd in enumerate(keys):
            a, b, anchors = fit_step(per_key.get(k, []), kd.cap)
            ok = bool(per_key.get(k))
            local.append([Bucket(theta=(0.0, 0.0, a * w, b * w), status=0b1100 if ok else 0, anchors=list(anchors))
                          for w in range(1, W + 1)])
            ext.append(Bucket(theta=(a / kd.cap, b / kd.cap, 0.0, 0.0), status=0b0011 if ok else 0, anchors=list(anchors)))
        return DualTable(W=W, keys=list(keys), local=local, ext=ext)
    per_key_w = defaultdict(list)
    for s in samples:
        s = Sample(*s)
        if 1 <= s.w <= W:
            per_key_w[(s.key, s.w)].append(s)
    local, ext = [], []
    lo = max(1, W - p + 1)
    for k in range(len(keys)):
        local.append([_fit_group(per_key_w.get((k, w), []), max_anchors, relative) for w in range(1, W + 1)])
        merged = [s for w in range(lo, W + 1) for s in per_key_w.get((k, w), [])]
        ext.append(_fit_group(merged, max_anchors, relative))
    return DualTable(W=W, keys=list(keys), local=local, ext=ext)


def r_squared(rows, theta) -> float:
    """Coefficient of determination of a fitted bucket on its own rows (Fig. 5 reports ~0.999)."""
    T = np.array([r[2] for r in rows], dtype=np.float64)
    pred = np.array([theta[0] * r[0] * r[1] + theta[1] * r[0] + theta[2] * r[1] + theta[3] for r in rows])
    ss_tot = float(np.sum((T - T.mean()) ** 2))
    return 1.0 - float(np.sum((T - pred) ** 2)) / ss_tot if ss_tot > 0 else 1.0
