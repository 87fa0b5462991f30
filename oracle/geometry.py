"""Oracle integer geometry: Phi, wave count, capacity (Sec. 3.2, Sec. 3.3, Table 2).

All quantities are Python ints (arbitrary precision), so nothing here can overflow.
TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

import heapq

N_CU = 256            # compute units of one MI355X
LDS_PER_CU = 163840   # bytes of LDS per compute unit (160 KiB)
SIMD_PER_CU = 4
MAX_WAVES_PER_SIMD = 8
VGPR_PER_SIMD_LANE = 512  # unified architectural + accumulation registers per lane


def ceil_div(a: int, b: int) -> int:
    """Smallest integer >= a/b for a >= 0, b > 0."""
    if b <= 0 or a < 0:
        raise ValueError("ceil_div needs a >= 0 and b > 0")
    return -((-a) // b)


def phi_gemm(M: int, N: int, K: int, BM: int, BN: int, BK: int, S: int = 1) -> tuple[int, int]:
    """Table 2, Dense-GEMM row: G = ceil(M/T_M) * ceil(N/T_N) blocks, L = ceil(K/T_K) iterations.

    S > 1 (split-K, a kernel parameter the paper's kernels do not have; reading: Phi counts the
    kernel's own tasks): every output tile is shared by S blocks that divide its ceil(K/T_K)
    k-tiles evenly, the last ones possibly short or empty, so G = S * tiles and each block loops
    L = ceil(ceil(K/T_K) / S) times."""
    if S < 1:
        raise ValueError("S >= 1")
    return S * ceil_div(M, BM) * ceil_div(N, BN), ceil_div(ceil_div(K, BK), S)


def split_fits(M: int, N: int, BM: int, BN: int, S: int, ws_elems=None, max_tiles=None) -> bool:
    """Whether a split-K configuration can run a shape when the S fp32 partial tiles of BM x BN per
    output tile have to fit a workspace of ws_elems floats with one arrival counter for each of at
    most max_tiles output tiles.  The method itself knows no such limit (None = unlimited, the
    default): whoever checks an implementation against this oracle passes that implementation's
    limits in.  Unsplit configurations always fit."""
    if S == 1:
        return True
    tiles = ceil_div(M, BM) * ceil_div(N, BN)
    if max_tiles is not None and tiles > max_tiles:
        return False
    return ws_elems is None or tiles * S * BM * BN <= ws_elems


def phi_grouped(rows, N: int, K: int, BM: int, BN: int, BK: int) -> tuple[int, int]:
    """Table 2, Grouped-GEMM row: G = sum_i ceil(M_i/T_M) * ceil(N/T_N), L = ceil(K/T_K)."""
    return sum(ceil_div(int(m), BM) * ceil_div(N, BN) for m in rows), ceil_div(K, BK)


def uniform_rows(M_total: int, E: int) -> list[int]:
    """Uniform approximation of the routing (Sec. 5.2, grouped-GEMM paragraph): the host does not know the
    per-expert counts, so every one of the E groups is taken to hold ceil(M_total / E) rows."""
    if E < 1:
        raise ValueError("E >= 1")
    return [ceil_div(M_total, E)] * E


def capacity(occ: int, n_cu: int = N_CU) -> int:
    """Blocks that can be resident at once: compute units times resident blocks per unit.

    The paper divides by the SM count alone (Sec. 3.2, step model; Sec. 3.3); with more than one
    block resident per unit a full "wave" holds n_cu * occ blocks, which is what its wave
    quantisation argument (blocks issued in groups bounded by available resources) refers to.
    """
    if occ < 1 or n_cu < 1:
        raise ValueError("occ and n_cu must be >= 1")
    return n_cu * occ


def wave_count(G: int, cap: int) -> int:
    """w = ceil(G / cap): number of waves needed to execute G blocks (Sec. 3.2; Sec. 3.3)."""
    return ceil_div(G, cap)


def last_wave_fill(G: int, cap: int) -> int:
    """Blocks in the final (possibly partial) wave: G - (w-1)*cap, in 1..cap for G >= 1."""
    if G == 0:
        return 0
    return G - (wave_count(G, cap) - 1) * cap


def wave_region(w: int, cap: int) -> tuple[int, int]:
    """Sec. 4.2, wave-aligned regions: R_w = [(w-1)*cap + 1, w*cap] (inclusive)."""
    if w < 1:
        raise ValueError("w >= 1")
    return (w - 1) * cap + 1, w * cap


def occupancy_estimate(lds_bytes: int, vgprs: int, nwave: int, lds_gran: int = 512,
                       block_cap: int = 32) -> int:
    """Resident blocks per compute unit from a block's resource triple.

    Integer model: LDS limit floor(LDS_CU / round_up(lds, gran)); register limit
    floor(512 / round_up(vgprs, 8)) waves per SIMD, capped at 8; a block of nwave wavefronts
    takes nwave of the 4*waves_per_simd slots.  The paper gives no such formula (it ignores
    occupancy); the hardware constants come from AMD's public CDNA documentation and the value
    the HIP runtime reports takes precedence.  parity unpinned beyond hand-worked arithmetic.
    """
    if nwave < 1:
        raise ValueError("nwave >= 1")
    r = ceil_div(max(vgprs, 1), 8) * 8
    wps = min(MAX_WAVES_PER_SIMD, VGPR_PER_SIMD_LANE // r)
    by_wave = (SIMD_PER_CU * wps) // nwave
    if lds_bytes > 0:
        by_lds = LDS_PER_CU // (ceil_div(lds_bytes, lds_gran) * lds_gran)
    else:
        by_lds = block_cap
    return max(0, min(by_wave, by_lds, block_cap))


def greedy_makespan(durations, workers: int) -> float:
    """Discrete-event simulation of greedy dispatch (Sec. 3.2, Fig. 4): each task, in order, goes
    to the worker that becomes free first; returns the time the last worker finishes."""
    if workers < 1:
        raise ValueError("workers >= 1")
    free = [0.0] * workers
    heapq.heapify(free)
    end = 0.0
    for d in durations:
        t = heapq.heappop(free) + float(d)
        end = max(end, t)
        heapq.heappush(free, t)
    return end
