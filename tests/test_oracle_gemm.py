"""Pins for oracle/gemm.py: decoders against the formats' definitions and a third-party decoder,
the product against exact integer arithmetic, hand-worked values and its transposition."""
import numpy as np
import pytest
import torch

import wt_synth
from oracle import gemm as og


def test_bf16_known_codes():
    codes = np.array([0x3F80, 0xC000, 0x4049, 0x0000, 0x3E80, 0x7F80], dtype=np.uint16)
    want = [1.0, -2.0, 3.140625, 0.0, 0.25, np.inf]
    assert og.bf16_bits_to_f64(codes).tolist() == want


def test_bf16_all_codes_match_torch():
    codes = np.arange(65536, dtype=np.uint16)
    mine = og.bf16_bits_to_f64(codes)
    ref = torch.from_numpy(codes.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    both_nan = np.isnan(mine) & np.isnan(ref)
    assert np.all((mine == ref) | both_nan)


def test_e4m3_known_codes():
    # 0x38: e=7,m=0 -> 1; 0x7E: e=15,m=6 -> 1.75*2^8 = 448; 0x01: smallest subnormal 2^-9;
    # 0x08: smallest normal 2^-6; 0xC0: -(2^1) = -2; 0x3C: 1.5
    codes = np.array([0x38, 0x7E, 0x01, 0x08, 0xC0, 0x3C, 0x00], dtype=np.uint8)
    want = [1.0, 448.0, 2.0 ** -9, 2.0 ** -6, -2.0, 1.5, 0.0]
    assert og.e4m3_bits_to_f64(codes).tolist() == want
    assert np.isnan(og.e4m3_bits_to_f64(np.array([0x7F, 0xFF], dtype=np.uint8))).all()


def test_e4m3_all_codes_match_torch():
    codes = np.arange(256, dtype=np.uint8)
    mine = og.e4m3_bits_to_f64(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    both_nan = np.isnan(mine) & np.isnan(ref)
    assert np.all((mine == ref) | both_nan)
    assert np.nanmax(mine) == 448.0 and np.isnan(mine).sum() == 2


def test_hand_worked_product_and_transposition():
    # A is [M,K]; B is stored [N,K]; C[i,j] = sum_k A[i,k] B[j,k].  A transposed-operand bug
    # (using B as [K,N]) cannot even be formed here (K=2, N=3) and a swapped i/j gives C^T.
    a = np.array([[1, 2], [3, 4]], dtype=np.float64)
    b = np.array([[5, 6], [7, 8], [9, 10]], dtype=np.float64)
    want = np.array([[17, 23, 29], [39, 53, 67]], dtype=np.float64)
    assert np.array_equal(og.gemm_loops(a, b), want)
    assert np.array_equal(og.gemm_f64(a, b), want)
    ab = wt_synth.to_bf16_bits(a.astype(np.float32))
    bb = wt_synth.to_bf16_bits(b.astype(np.float32))
    assert np.array_equal(og.gemm_c(ab, bb), want)
    assert np.array_equal(og.rows_f64(a, b, [1]), want[1:2])
    assert np.array_equal(og.cols_f64(a, b, [2, 0]), want[:, [2, 0]])


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (17, 33, 40), (64, 48, 129)])
def test_integer_matrices_exact(M, N, K):
    # integer entries in [-8,8]: every partial sum is an integer far below 2^53, so the fp64
    # product must equal the int64 product exactly, whatever the summation order.
    a32, b32 = wt_synth.gemm_operands(M, N, K, seed=7 + M, kind="int")
    want = a32.astype(np.int64) @ b32.astype(np.int64).T
    ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)
    a, b = og.decode(ab, "bf16"), og.decode(bb, "bf16")
    assert np.array_equal(a, a32) and np.array_equal(b, b32)
    assert np.array_equal(og.gemm_f64(a, b), want)
    assert np.array_equal(og.gemm_c(ab, bb), want)
    if M * N * K <= 30000:
        assert np.array_equal(og.gemm_loops(a, b), want)


def test_identity_b_returns_a():
    a32 = wt_synth.normal_f32(9, 16, 3)
    ab = wt_synth.to_bf16_bits(a32)
    eye = wt_synth.to_bf16_bits(np.eye(16, dtype=np.float32))
    assert np.array_equal(og.gemm_c(ab, eye), og.decode(ab, "bf16"))
    perm = np.eye(16, dtype=np.float32)[::-1].copy()     # B[j,k]=1 iff k=15-j -> C[i,j]=A[i,15-j]
    assert np.array_equal(og.gemm_c(ab, wt_synth.to_bf16_bits(perm)), og.decode(ab, "bf16")[:, ::-1])


def test_normal_inputs_three_routes_agree():
    a32, b32 = wt_synth.gemm_operands(20, 24, 300, seed=11)
    ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)
    a, b = og.decode(ab, "bf16"), og.decode(bb, "bf16")
    c_loops, c_np, c_c = og.gemm_loops(a, b), og.gemm_f64(a, b), og.gemm_c(ab, bb)
    assert np.array_equal(c_loops, c_c)                     # same order of summation
    assert og.rel_frobenius(c_np, c_loops) < 1e-14          # BLAS may reorder the sum
    # bf16 rounding of N(0,1) inputs moves the product by ~2^-9 relative, not more
    c_unrounded = a32.astype(np.float64) @ b32.astype(np.float64).T
    assert 1e-4 < og.rel_frobenius(c_loops, c_unrounded) < 1e-2


def test_e4m3_scaled_product():
    a32, b32 = wt_synth.gemm_operands(6, 5, 64, seed=5)
    aq, sa = wt_synth.to_e4m3_bits(a32)
    bq, sb = wt_synth.to_e4m3_bits(b32)
    a, b = og.decode(aq, "e4m3", sa), og.decode(bq, "e4m3", sb)
    # the quantised operands are within half an e4m3 step (2^-4 relative) of the inputs, or
    # within half a subnormal step in absolute terms
    assert np.all(np.abs(a - a32) <= np.maximum(np.abs(a32) * 2.0 ** -4, float(sa) * 2.0 ** -10))
    assert float(np.max(np.abs(og.e4m3_bits_to_f64(aq)))) == 448.0   # amax maps to the top code
    c = og.gemm_c(aq, bq, "e4m3", sa, sb)
    raw = og.e4m3_bits_to_f64(aq) @ og.e4m3_bits_to_f64(bq).T
    assert og.rel_frobenius(c, raw * float(sa) * float(sb)) < 1e-14
    assert og.rel_frobenius(c, og.gemm_loops(a, b)) < 1e-15


def test_e4m3_integer_exact():
    a32, b32 = wt_synth.gemm_operands(5, 7, 48, seed=9, kind="int")
    aq = torch.from_numpy(a32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    bq = torch.from_numpy(b32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    want = a32.astype(np.int64) @ b32.astype(np.int64).T
    assert np.array_equal(og.gemm_c(aq, bq, "e4m3", 1.0, 1.0), want)


def test_metrics():
    ref = np.array([[3.0, 4.0]])
    assert og.rel_frobenius(ref, ref) == 0.0
    assert abs(og.rel_frobenius(np.array([[3.0, 4.5]]), ref) - 0.1) < 1e-15
    # rms(ref)=sqrt(12.5)~3.54: element 0 is scaled by 3.54, element 1 by 4
    e = og.max_scaled_err(np.array([[3.1, 4.0]]), ref)
    assert abs(e - 0.1 / np.sqrt(12.5)) < 1e-12
