"""Oracle for the attention row of the unified abstraction (Table 2, FlashAttention row; Sec. 4.2,
head-aligned grid sizes and the attention instantiation rule).

  attention()            softmax(scale * Q K^T [+ causal mask]) V per head, in fp64, written as the
                         definition (scores, row maximum, exponentials, row sum, weighted sum of V).
  phi_attn()             (N_h, S_q, S_kv) -> (G, L) for a macro config <T_Q, T_KV>.
  representative_heads() largest multiple of N_h in a sub-interval.
  sample_set_heads()     all representatives for waves 1..W, sub-intervals 1..I.
  instantiate_attn()     (G, L) -> (S_q, S_kv).
  kv_loop_counts()       loop counts induced by scaling the KV length by multipliers of S_q.

TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

from typing import NamedTuple

import numpy as np

from .geometry import ceil_div
from .sampler import sub_interval


def attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float, causal: bool = False) -> np.ndarray:
    """Scaled dot-product attention, one sequence (the operation the FlashAttention kernels of Sec. 5.1 compute).

    Q is [S_q, H_q, D], K and V are [S_kv, H_kv, D] (token-major, heads next, head dimension contiguous); the
    result is [S_q, H_q, D] in fp64.  H_kv divides H_q: query head h reads KV head h // (H_q // H_kv)
    (grouped-query attention; H_kv == H_q is plain multi-head attention).  With causal=True query i sees the
    keys j <= i + (S_kv - S_q): the queries are the last S_q positions of a sequence of S_kv tokens.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S_q, H_q, D = Q.shape
    S_kv, H_kv, Dk = K.shape
    if Dk != D or V.shape != K.shape or H_kv < 1 or H_q % H_kv:
        raise ValueError("shape mismatch")
    if causal and S_kv < S_q:
        raise ValueError("causal attention needs S_kv >= S_q")
    group = H_q // H_kv
    out = np.zeros((S_q, H_q, D), dtype=np.float64)
    if S_kv == 0:
        return out
    shift = S_kv - S_q
    for h in range(H_q):
        kh = h // group
        scores = scale * (Q[:, h, :] @ K[:, kh, :].T)          # [S_q, S_kv]
        if causal:
            i = np.arange(S_q)[:, None]
            j = np.arange(S_kv)[None, :]
            scores = np.where(j <= i + shift, scores, -np.inf)
        m = scores.max(axis=1, keepdims=True)
        e = np.exp(scores - m)
        out[:, h, :] = (e / e.sum(axis=1, keepdims=True)) @ V[:, kh, :]
    return out


def phi_attn(n_heads: int, S_q: int, S_kv: int, T_Q: int, T_KV: int) -> tuple[int, int]:
    """Table 2, FlashAttention row: G = N_h * ceil(S_q / T_Q) blocks, L = ceil(S_kv / T_KV) iterations."""
    if n_heads < 1:
        raise ValueError("n_heads >= 1")
    return n_heads * ceil_div(S_q, T_Q), ceil_div(S_kv, T_KV)


def phi_attn_varlen(n_heads: int, lens_q, lens_kv, T_Q: int, T_KV: int) -> tuple[int, int]:
    """Table 2's FlashAttention row read for a batch of sequences of different lengths (the paper states it for one
    length; Sec. 5.3 runs ragged prefill batches): sequence i contributes ceil(q_i / T_Q) query tiles per head, each
    looping over ceil(kv_i / T_KV) key tiles.  G counts every block; L is the mean loop count over the blocks, rounded
    half up, so that G * L is the launch's number of key-tile iterations to within rounding, as it is exactly for
    equal lengths.  No block at all gives (0, 0)."""
    if n_heads < 1 or len(lens_q) != len(lens_kv):
        raise ValueError("n_heads >= 1, one kv length per query length")
    tiles = [ceil_div(q, T_Q) for q in lens_q]
    loops = [ceil_div(kv, T_KV) for kv in lens_kv]
    t = sum(tiles)
    if t == 0:
        return 0, 0
    iters = sum(a * b for a, b in zip(tiles, loops))
    return n_heads * t, (2 * iters + t) // (2 * t)


def representative_heads(a: int, b: int, n_heads: int) -> int:
    """Sec. 4.2: the sub-interval [a, b] is projected to the head-aligned value floor(b / N_h) * N_h, which
    counts only if it is still >= a; 0 means the sub-interval holds no multiple of N_h."""
    g = (b // n_heads) * n_heads
    return g if g >= max(a, 1) else 0


class HeadSample(NamedTuple):
    w: int        # wave index, 1-based
    i: int        # sub-interval index, 1-based
    g: int        # head-aligned grid size (0: none in this sub-interval)
    q_tiles: int  # query tiles per head, g / N_h


def sample_set_heads(cap: int, W: int, I: int, n_heads: int) -> list[HeadSample]:
    """Eq. 4 with the attention rule for g_{w,i}: W * I entries in (w, i) order."""
    out = []
    for w in range(1, W + 1):
        for i in range(1, I + 1):
            a, b = sub_interval(w, i, cap, I)
            g = representative_heads(a, b, n_heads)
            out.append(HeadSample(w, i, g, g // n_heads))
    return out


def instantiate_attn(g: int, L: int, n_heads: int, T_Q: int, T_KV: int) -> tuple[int, int]:
    """Eq. 6: S_q = (G / N_h) * T_Q, S_kv = L * T_KV."""
    if g % n_heads:
        raise ValueError("G must be a multiple of N_h")
    return (g // n_heads) * T_Q, L * T_KV


def kv_loop_counts(S_q: int, T_KV: int, mult_percent) -> list[int]:
    """Loop anchors of an attention grid point (Sec. 5.1, training-set paragraph: the KV length is the query
    length scaled by multipliers between 1.0 and 3.0).  Reading: the multipliers are given in percent,
    S_kv = floor(S_q * percent / 100) and L = ceil(S_kv / T_KV); equal L are merged, ascending order."""
    return sorted({ceil_div((S_q * int(p)) // 100, T_KV) for p in mult_percent})
