"""Seeded synthetic inputs shared by the HIP path's tests, the CPU oracle's tests and bench.py.

This module only *draws data*: random matrices in their storage encodings, shape lists and
latency surfaces used as stand-ins for measurements.  It holds none of the method's arithmetic
(no GEMM, no tile/wave geometry, no sampling rule, no fit, no lookup) and imports neither the
oracle nor the HIP binding.  Storage encodings are produced with PyTorch's CPU dtype casts, so
neither side under test is used to make its own inputs.

Workload recipe (stand-in for the paper's Dense-GEMM shape sets, which are not public):
values are N(0,1) drawn with numpy's PCG64 from a seed, rounded once to the storage type.
"""
from __future__ import annotations

import math
import zlib

import numpy as np
import torch

E4M3_MAX = 448.0  # largest finite magnitude of OCP FP8 E4M3 (the "fn" flavour)

# (N, K) pairs of the LLM-projection sweep and of the runtime stream.
SWEEP_M = (1, 16, 17, 64, 100, 256, 333, 1024, 4096)
SWEEP_NK = ((4096, 4096), (11008, 4096), (4096, 11008))
STREAM_NK = ((8192, 8192), (28672, 8192), (8192, 28672), (10240, 8192))


def shape_seed(base: int, M: int, N: int, K: int) -> int:
    """Deterministic per-shape sub-seed (CRC32 of the shape mixed with a base seed)."""
    return (base * 1000003 + zlib.crc32(f"{M}x{N}x{K}".encode())) & 0x7FFFFFFF


def normal_f32(rows: int, cols: int, seed: int) -> np.ndarray:
    """rows x cols standard-normal fp32 matrix from a seed."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((rows, cols), dtype=np.float32)


def small_int_f32(rows: int, cols: int, seed: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """Integer-valued fp32 matrix with entries in [lo, hi] (exact in bf16 and in e4m3)."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=(rows, cols)).astype(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 storage bits (uint16), round-to-nearest-even, via torch's CPU cast."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def to_e4m3_bits(x: np.ndarray) -> tuple[np.ndarray, np.float32]:
    """fp32 -> (e4m3 storage bytes, per-tensor fp32 scale s) with s = amax/448, q = rne(x/s).

    x/s is clamped to +-448 before the cast, so the encoding saturates instead of producing NaN.
    An all-zero tensor gets s = 1.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.float32(np.max(np.abs(x))) if x.size else np.float32(0.0)
    s = np.float32(amax / np.float32(E4M3_MAX)) if amax > 0 else np.float32(1.0)
    y = np.clip(x / s, -E4M3_MAX, E4M3_MAX).astype(np.float32)
    q = torch.from_numpy(y).to(torch.float8_e4m3fn)
    return q.view(torch.uint8).numpy().copy(), s


def gemm_operands(M: int, N: int, K: int, seed: int, kind: str = "normal"):
    """fp32 A[M,K] and B[N,K] (both K-contiguous) for one GEMM; kind is 'normal' or 'int'."""
    gen = normal_f32 if kind == "normal" else small_int_f32
    return gen(M, K, seed), gen(N, K, seed + 1)


def sweep_shapes():
    """The 27 LLM-projection shapes (M x (N,K))."""
    return [(m, n, k) for (n, k) in SWEEP_NK for m in SWEEP_M]


def wave_stress_shapes():
    """M=K=4096, N = 128..16384 step 128 (128 shapes)."""
    return [(4096, n, 4096) for n in range(128, 16384 + 1, 128)]


def stream_shapes(count: int = 10000, seed: int = 1005):
    """Runtime stream: M log-uniform in [1,8192], (N,K) uniform over STREAM_NK; duplicates kept."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        u = rng.random()
        m = int(min(8192, max(1, round(math.exp(u * math.log(8192.0))))))
        n, k = STREAM_NK[int(rng.integers(0, len(STREAM_NK)))]
        out.append((m, n, k))
    return out


def paper_range_shapes(count: int = 60, seed: int = 3001):
    """Shapes in the ranges of the paper's Dense-GEMM test set (Sec. 5.1: M in [64, 16384], N in [384, 8192],
    K in [2048, 8192]; the set itself is not public): M log-uniform, N log-uniform rounded to a multiple of 128,
    K a multiple of 256.  `count` distinct shapes, sorted."""
    rng = np.random.default_rng(seed)
    out = set()
    while len(out) < count:
        m = int(round(math.exp(rng.uniform(math.log(64), math.log(16384)))))
        n = int(round(math.exp(rng.uniform(math.log(384), math.log(8192))) / 128)) * 128
        k = int(rng.integers(8, 33)) * 256
        out.add((m, max(n, 384), k))
    return sorted(out)


def short_k_shapes(count: int = 40, seed: int = 3002):
    """Small launches below the paper's lowest loop anchor and around it: M log-uniform in [16, 4096],
    N in {256 .. 4096}, K in {256, 512, 1024, 1536, 2048}, plus the cubes 256, 512 and 1024.  Sorted."""
    rng = np.random.default_rng(seed)
    out = {(256, 256, 256), (1024, 1024, 1024), (512, 512, 512)}
    while len(out) < count:
        m = int(round(math.exp(rng.uniform(math.log(16), math.log(4096)))))
        n = int(rng.choice([256, 512, 1024, 2048, 4096]))
        k = int(rng.choice([256, 512, 1024, 1536, 2048]))
        out.add((m, n, k))
    return sorted(out)


def noise_factors(n: int, seed: int, rel: float) -> np.ndarray:
    """n multiplicative noise factors 1 + rel*N(0,1), clipped to stay positive."""
    rng = np.random.default_rng(seed)
    return np.clip(1.0 + rel * rng.standard_normal(n), 0.05, None)


def random_theta(seed: int, count: int) -> np.ndarray:
    """count random positive coefficient tuples (alpha, beta, gamma, delta) in microseconds.

    Magnitudes follow a GEMM-like surface: alpha ~ 1e-4..1e-3 us per (tile x loop), beta and
    gamma ~ 1e-3..1e-1, delta ~ 1..10.  Used to synthesise latency tables with a known optimum.
    """
    rng = np.random.default_rng(seed)
    a = 10.0 ** rng.uniform(-4.0, -3.0, count)
    b = 10.0 ** rng.uniform(-3.0, -1.0, count)
    g = 10.0 ** rng.uniform(-3.0, -1.0, count)
    d = 10.0 ** rng.uniform(0.0, 1.0, count)
    return np.stack([a, b, g, d], axis=1)


def moe_routing(tokens: int, experts: int, top_k: int, seed: int, skew: float = 1.0) -> np.ndarray:
    """Rows per expert for a synthetic MoE layer: every token picks top_k distinct experts with
    probabilities proportional to 1/rank^skew (skew 0 = uniform), the experts' ranks shuffled by the
    seed.  Returns int64 counts summing to tokens*top_k; some may be 0.  Stands in for a trained
    router's output (no trained weights here)."""
    rng = np.random.default_rng(seed)
    w = 1.0 / np.arange(1, experts + 1, dtype=np.float64) ** skew
    w = rng.permutation(w / w.sum())
    counts = np.zeros(experts, dtype=np.int64)
    for _ in range(tokens):
        counts[rng.choice(experts, size=min(top_k, experts), replace=False, p=w)] += 1
    return counts


def group_offsets(counts) -> np.ndarray:
    """int32 row offsets [0, c0, c0+c1, ...] of back-to-back groups."""
    return np.concatenate([[0], np.cumsum(np.asarray(counts, dtype=np.int64))]).astype(np.int32)


# MoE grouped-GEMM workloads (experts, top_k, N, K): the expert projections of a 128-expert / top-8 /
# hidden 2048 / expert width 768 layer (gate+up fused: N = 1536, K = 2048; down: N = 2048, K = 768) and of
# an 8-expert / top-2 / hidden 4096 / expert width 14336 layer.
MOE_LAYERS = [(128, 8, 1536, 2048), (128, 8, 2048, 768), (8, 2, 28672, 4096), (8, 2, 4096, 14336)]
MOE_TOKENS = [16, 128, 1024, 8192]


# ---- attention workloads (stand-in for the paper's FlashAttention test set: sequence lengths 64..16384,
#      16..128 query heads, 2..16 KV heads, head dimension 128; not public, so drawn from the same ranges) ----
ATTN_HEAD_DIM = 128
ATTN_Q_HEADS = (16, 32, 64, 128)
ATTN_KV_HEADS = (2, 4, 8, 16)


def attn_operands(S_q: int, S_kv: int, H_q: int, H_kv: int, seed: int, q_gain: float = 1.0):
    """(Q [S_q,H_q,128], K [S_kv,H_kv,128], V [S_kv,H_kv,128]) as bf16 storage bits; N(0,1) entries, Q scaled by
    q_gain (a gain above 1 sharpens the softmax)."""
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((S_q, H_q, ATTN_HEAD_DIM), dtype=np.float32) * np.float32(q_gain)
    k = rng.standard_normal((S_kv, H_kv, ATTN_HEAD_DIM), dtype=np.float32)
    v = rng.standard_normal((S_kv, H_kv, ATTN_HEAD_DIM), dtype=np.float32)
    return tuple(to_bf16_bits(x.reshape(-1, ATTN_HEAD_DIM)).reshape(x.shape) for x in (q, k, v))


def attn_shapes(count: int = 64, seed: int = 1006):
    """(S_q, S_kv, H_q, H_kv) draws: log-uniform sequence length in [64, 16384] (prefill: S_kv = S_q), head counts
    from the lists above with H_kv <= H_q."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        s = int(np.clip(round(math.exp(rng.uniform(math.log(64), math.log(16384)))), 64, 16384))
        hq = int(ATTN_Q_HEADS[rng.integers(0, len(ATTN_Q_HEADS))])
        hkv = int(ATTN_KV_HEADS[rng.integers(0, len(ATTN_KV_HEADS))])
        out.append((s, s, hq, min(hkv, hq)))
    return out


def varlen_batches(count: int = 20, seed: int = 4001, lo: int = 512, hi: int = 16384):
    """Ragged prefill batches (the shape of the paper's end-to-end setting, Sec. 5.3): 2, 4 or 8 prompts each, prompt
    lengths log-uniform in [lo, hi].  Returns a list of length lists."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        batch = int(rng.choice([2, 4, 8]))
        out.append([int(round(math.exp(rng.uniform(math.log(lo), math.log(hi))))) for _ in range(batch)])
    return out
