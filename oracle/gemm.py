"""Oracle GEMM: C[i,j] = sum_k A[i,k] * B[j,k] accumulated in fp64 (Sec. 3.2, tiled-GEMM
paragraph; the tiling there does not change the value, so the oracle is the plain definition).

Operands arrive in their storage encoding (bf16 bits, or e4m3 bytes plus a per-tensor fp32
scale) and are decoded here, independently of whatever produced them.  B is supplied
K-contiguous as [N, K], i.e. the product is A times the transpose of the stored B.

TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 storage bits -> fp64.  bf16 is the upper half of an IEEE binary32 word."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def e4m3_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """OCP FP8 E4M3 ("fn": no infinities, one NaN mantissa pattern) bytes -> fp64.

    1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent 0 is subnormal (m/8 * 2^-6);
    exponent 15 with mantissa 7 is NaN, every other code is finite; largest finite = 448.
    """
    b = np.ascontiguousarray(bits, dtype=np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 0xF
    m = (b & 0x7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    sub = (m / 8.0) * 2.0 ** -6
    v = np.where(e == 0, sub, normal)
    v = np.where((e == 15) & ((b & 0x7) == 7), np.nan, v)
    return sign * v


def decode(bits: np.ndarray, in_type: str, scale: float = 1.0) -> np.ndarray:
    """Storage encoding -> the real values the GEMM is defined on (fp64)."""
    if in_type == "bf16":
        return bf16_bits_to_f64(bits)
    if in_type == "e4m3":
        return e4m3_bits_to_f64(bits) * float(np.float32(scale))
    raise ValueError(in_type)


def gemm_loops(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Triple loop in Python floats (IEEE binary64); tiny inputs only."""
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2
    c = np.zeros((M, N), dtype=np.float64)
    for i in range(M):
        for j in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(a[i, k]) * float(b[j, k])
            c[i, j] = acc
    return c


def gemm_f64(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """fp64 product through numpy's matmul (a library primitive standing for the sum above)."""
    return np.asarray(a, dtype=np.float64) @ np.asarray(b, dtype=np.float64).T


def rows_f64(a: np.ndarray, b: np.ndarray, rows) -> np.ndarray:
    """Selected complete rows of the product: C[rows, :]."""
    return np.asarray(a, dtype=np.float64)[list(rows)] @ np.asarray(b, dtype=np.float64).T


def cols_f64(a: np.ndarray, b: np.ndarray, cols) -> np.ndarray:
    """Selected complete columns of the product: C[:, cols]."""
    return np.asarray(a, dtype=np.float64) @ np.asarray(b, dtype=np.float64)[list(cols)].T


# ---- C triple loop (oracle/gemm_ref.c), for shapes Python loops cannot finish ----------------
_lib = None


def _load_c():
    global _lib
    if _lib is None:
        path = os.path.join(_HERE, "libgemm_ref.so")
        if not os.path.exists(path):
            raise RuntimeError("oracle/libgemm_ref.so not built; run __graft_entry__.build()")
        lib = ctypes.CDLL(path)
        lib.oracle_gemm_bf16.restype = ctypes.c_int
        lib.oracle_gemm_bf16.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_void_p] * 3 + [ctypes.c_int]
        lib.oracle_gemm_e4m3.restype = ctypes.c_int
        lib.oracle_gemm_e4m3.argtypes = ([ctypes.c_int64] * 3 + [ctypes.c_void_p] * 2
                                         + [ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_int])
        lib.oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def c_threads() -> int:
    """Number of threads the C loop uses by default (OpenMP's maximum)."""
    return int(_load_c().oracle_threads())


def gemm_c(a_bits: np.ndarray, b_bits: np.ndarray, in_type: str = "bf16",
           scale_a: float = 1.0, scale_b: float = 1.0, threads: int = 0) -> np.ndarray:
    """fp64 triple loop in C on storage-encoded operands; returns C as fp64 [M, N]."""
    lib = _load_c()
    M, K = a_bits.shape
    N, K2 = b_bits.shape
    assert K == K2
    c = np.empty((M, N), dtype=np.float64)
    if in_type == "bf16":
        a = np.ascontiguousarray(a_bits, dtype=np.uint16)
        b = np.ascontiguousarray(b_bits, dtype=np.uint16)
        rc = lib.oracle_gemm_bf16(M, N, K, a.ctypes.data, b.ctypes.data, c.ctypes.data, threads)
    elif in_type == "e4m3":
        a = np.ascontiguousarray(a_bits, dtype=np.uint8)
        b = np.ascontiguousarray(b_bits, dtype=np.uint8)
        rc = lib.oracle_gemm_e4m3(M, N, K, a.ctypes.data, b.ctypes.data,
                                  float(np.float32(scale_a)), float(np.float32(scale_b)),
                                  c.ctypes.data, threads)
    else:
        raise ValueError(in_type)
    if rc != 0:
        raise RuntimeError(f"oracle gemm_ref failed rc={rc}")
    return c


def grouped_gemm_c(a_bits: np.ndarray, b_bits: np.ndarray, offsets, in_type: str = "bf16",
                   scale_a: float = 1.0, scale_b: float = 1.0) -> np.ndarray:
    """Grouped GEMM by its definition (Table 2, grouped-GEMM row; MoE: the rows routed to expert e are
    multiplied by expert e's weights): for every group e, C[r0:r1] = A[r0:r1] * B[e]^T with
    r0, r1 = offsets[e], offsets[e+1].  a_bits [M_total, K], b_bits [E, N, K]; one plain dense product
    per group, rows outside every group stay NaN so that a test notices if they are touched."""
    E, N, K = b_bits.shape
    assert len(offsets) == E + 1 and a_bits.shape[1] == K
    c = np.full((a_bits.shape[0], N), np.nan, dtype=np.float64)
    for e in range(E):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 > r0:
            c[r0:r1] = gemm_c(a_bits[r0:r1], b_bits[e], in_type, scale_a, scale_b)
    return c


# ---- comparison metrics used by the parity tests ---------------------------------------------
def rel_frobenius(c: np.ndarray, c_ref: np.ndarray) -> float:
    """||C - C_ref||_F / ||C_ref||_F (0 when both are all-zero)."""
    c = np.asarray(c, dtype=np.float64)
    den = float(np.linalg.norm(c_ref))
    num = float(np.linalg.norm(c - c_ref))
    return num / den if den > 0 else num


def max_scaled_err(c: np.ndarray, c_ref: np.ndarray) -> float:
    """max_ij |C - C_ref| / max(|C_ref|_ij, rms(C_ref)): per-element error for bf16 outputs.

    A pure relative error is undefined where C_ref passes through zero, so each element is
    scaled by the larger of its own magnitude and the matrix's RMS value.
    """
    c = np.asarray(c, dtype=np.float64)
    rms = float(np.sqrt(np.mean(np.square(c_ref)))) if c_ref.size else 0.0
    den = np.maximum(np.abs(c_ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(c - c_ref) / den)) if c_ref.size else 0.0
