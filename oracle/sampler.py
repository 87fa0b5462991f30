"""Oracle sparse structural sampling (Sec. 4.2).

Wave-aligned regions are cut into I sub-intervals; each contributes the largest grid size that
factors into a nearly square 2D block grid; every grid size is paired with every loop anchor
and turned into a concrete (M, N, K).

TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

import math
from typing import NamedTuple, Optional

from .geometry import ceil_div, wave_region


class GridSample(NamedTuple):
    w: int   # wave index, 1-based
    i: int   # sub-interval index, 1-based
    g: int   # representative grid size (0 when the sub-interval has none)
    m: int   # block-grid rows (m <= n)
    n: int   # block-grid columns


def sub_interval(w: int, i: int, cap: int, I: int) -> tuple[int, int]:
    """[a, b] of the i-th of I parts of R_w (Sec. 4.2).  The paper does not say how to split
    when I does not divide cap; this reading uses floors: offsets floor((i-1)*cap/I)+1 ..
    floor(i*cap/I), which tile R_w exactly and are equal-sized when I | cap."""
    if not (1 <= i <= I):
        raise ValueError("1 <= i <= I")
    lo, _ = wave_region(w, cap)
    a = lo + ((i - 1) * cap) // I
    b = lo - 1 + (i * cap) // I
    return a, b


def most_square(g: int) -> tuple[int, int]:
    """(m, n) with m*n = g, m <= n and m the largest divisor of g not exceeding sqrt(g)."""
    if g < 1:
        raise ValueError("g >= 1")
    m = math.isqrt(g)
    while g % m:
        m -= 1
    return m, g // m


def qualifies(m: int, n: int, tau_num: int, tau_den: int) -> bool:
    """Aspect-ratio constraint n/m <= tau with tau = tau_num/tau_den, compared in integers."""
    return m <= n and n * tau_den <= m * tau_num


def representative(a: int, b: int, tau_num: int, tau_den: int) -> Optional[tuple[int, int, int]]:
    """Largest g in [a, b] with a factorisation g = m*n, m <= n, n/m <= tau (Sec. 4.2).

    A value qualifies iff its most-square factorisation does (that one minimises n/m), so the
    scan tests only that factorisation.  Returns (g, m, n) or None when nothing qualifies.
    """
    for g in range(b, a - 1, -1):
        if g < 1:
            break
        m, n = most_square(g)
        if qualifies(m, n, tau_num, tau_den):
            return g, m, n
    return None


def representative_split(a: int, b: int, S: int, tau_num: int, tau_den: int) -> Optional[tuple[int, int, int]]:
    """Split-K reading of the representative: the task count g of a kernel with S blocks per output
    tile is S times its tile count, so only multiples of S can occur; the largest g in [a, b] whose
    tile grid g/S = m*n is nearly square.  Returns (g, m, n) with m*n = g/S, or None."""
    for g in range(b, a - 1, -1):
        if g < 1:
            break
        if g % S:
            continue
        m, n = most_square(g // S)
        if qualifies(m, n, tau_num, tau_den):
            return g, m, n
    return None


def sample_set(cap: int, W: int, I: int, tau_num: int = 11, tau_den: int = 10, S: int = 1) -> list[GridSample]:
    """The sampling set {g_{w,i}} (Sec. 4.2), w-major then i; empty sub-intervals have g = 0.
    S > 1: see representative_split (m x n is then the tile grid and g = S*m*n)."""
    out = []
    for w in range(1, W + 1):
        for i in range(1, I + 1):
            a, b = sub_interval(w, i, cap, I)
            if b < a:
                r = None
            elif S == 1:
                r = representative(a, b, tau_num, tau_den)
            else:
                r = representative_split(a, b, S, tau_num, tau_den)
            out.append(GridSample(w, i, *(r if r else (0, 0, 0))))
    return out


def row_sample_set(cap: int, W_row: int, I: int, m: int = 1, S: int = 1) -> list[GridSample]:
    """Extension beyond the paper (its sampler keeps to near-square grids and its test shapes have
    M >= 64): grids of m = 1, 2 or 4 tile rows for the serving shapes -- few tile rows, very wide --
    whose B operand streams from HBM with little reuse.  The same wave regions and sub-intervals are
    used (Sec. 4.2); with m rows (and S blocks per tile) a task count must be a multiple of S*m, and
    the representative of a sub-interval is the largest such count in it: g = S*m*n, n = floor(b/(S*m)),
    kept if it is not below a."""
    out = []
    for w in range(1, W_row + 1):
        for i in range(1, I + 1):
            a, b = sub_interval(w, i, cap, I)
            n = b // (S * m)
            g = S * m * n
            out.append(GridSample(w, i, g, m, n) if (b >= a and n >= 1 and g >= a) else GridSample(w, i, 0, 0, 0))
    return out


def row_family(tile_rows: int) -> int:
    """Which sample family serves a shape with ceil(M/T_M) = tile_rows tile rows: the 1-row family for 1,
    the 2-row family for 2..3, the 4-row family for 4..7, the paper's near-square samples (0) otherwise."""
    return 1 if tile_rows <= 1 else 2 if tile_rows <= 3 else 3 if tile_rows <= 7 else 0


ROW_BANDS = (16, 32, 64, 128)


def band_family(M: int, bands=ROW_BANDS) -> int:
    """Row-band families (extension, the second form of the few-row families): which family serves a shape of M rows --
    that of the smallest band holding M, whatever the key's tile height, so that every key is priced from samples of
    the same matrices; 0 (the paper's near-square samples) above the last band."""
    for f, rows in enumerate(bands, start=1):
        if M <= rows:
            return f
    return 0


def band_sample_set(cap: int, W_row: int, I: int, rows: int, BM: int, S: int = 1) -> list[GridSample]:
    """Samples of a row-band family under a key of tile height BM: matrices of exactly `rows` rows, i.e.
    m = ceil(rows/BM) tile rows of which the last may be partial, as wide as the sub-interval allows -- the rule of
    row_sample_set with that m.  The workload has M = rows (not m*BM), N = n*T_N."""
    return row_sample_set(cap, W_row, I, ceil_div(rows, BM), S)


def instantiate(m: int, n: int, L: int, BM: int, BN: int, BK: int, S: int = 1) -> tuple[int, int, int]:
    """Sec. 4.2, workload instantiation: M = m_G*T_M, N = n_G*T_N, K = L*T_K.  With S blocks per tile
    each of them gets exactly L k-tiles: K = L*S*T_K."""
    return m * BM, n * BN, L * S * BK


def loop_anchors(k_anchors, BK: int, S: int = 1) -> list[int]:
    """Loop counts for a list of K anchors under tile depth BK: L_j = ceil(K_j / BK), ascending,
    duplicates removed.  (The paper lists anchors in K -- five spanning [1024, 5120] -- so the
    loop anchors differ per tile depth.)  With S blocks per tile, L_j = ceil(ceil(K_j/BK) / S)."""
    return sorted({-(-(-(-int(k) // BK)) // S) for k in k_anchors})


def profile_budget(n_grid: int, n_loop: int, n_macro: int, n_micro: int) -> int:
    """Sec. 4.2, profiling complexity: N_profile = |G| * |L| * |C_macro| * |C_micro|."""
    return n_grid * n_loop * n_macro * n_micro
