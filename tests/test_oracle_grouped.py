"""Pins for the oracle's grouped-GEMM pieces: Table 2's grouped row against closed forms, the uniform
approximation, and the grouped product against an independent dense formulation."""
import numpy as np
import pytest

import wt_synth
from oracle import gemm as og
from oracle import geometry as geo


def test_grouped_phi_reduces_to_dense_and_adds_up():
    # one group is the dense row of Table 2; equal groups multiply it; empty groups add nothing
    assert geo.phi_grouped([300], 500, 1000, 128, 64, 32) == geo.phi_gemm(300, 500, 1000, 128, 64, 32)
    G1, L = geo.phi_gemm(300, 500, 1000, 128, 64, 32)
    assert geo.phi_grouped([300] * 7 + [0, 0], 500, 1000, 128, 64, 32) == (7 * G1, L)
    # ragged groups: every group pays its own partial tile (3 + 1 + 1 + 0 row tiles x 8 column tiles)
    assert geo.phi_grouped([257, 1, 128, 0], 500, 64, 128, 64, 64) == ((3 + 1 + 1 + 0) * 8, 1)
    # splitting rows over more groups never needs fewer tiles than the dense problem
    rng = np.random.default_rng(3)
    for _ in range(50):
        rows = rng.integers(0, 400, size=rng.integers(1, 9)).tolist()
        G, _ = geo.phi_grouped(rows, 777, 512, 64, 128, 64)
        Gd, _ = geo.phi_gemm(sum(rows), 777, 512, 64, 128, 64)
        assert Gd <= G <= Gd + len(rows) * geo.ceil_div(777, 128)


def test_uniform_rows():
    assert geo.uniform_rows(1000, 8) == [125] * 8
    assert geo.uniform_rows(1001, 8) == [126] * 8
    assert geo.uniform_rows(0, 4) == [0] * 4
    with pytest.raises(ValueError):
        geo.uniform_rows(5, 0)


def test_grouped_product_equals_block_diagonal_dense_product():
    """Stack the groups' weights side by side: the dense product of A with [B_0; B_1; ...] contains, for a
    row of group e, the grouped result in column block e (numpy matmul in fp64 as the second opinion)."""
    counts = [5, 0, 17, 1, 9]
    off = wt_synth.group_offsets(counts)
    E, N, K = len(counts), 12, 40
    rng = np.random.default_rng(11)
    a32 = rng.standard_normal((int(off[-1]), K)).astype(np.float32)
    b32 = rng.standard_normal((E, N, K)).astype(np.float32)
    ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32.reshape(E * N, K)).reshape(E, N, K)
    got = og.grouped_gemm_c(ab, bb, off)
    a, b = og.decode(ab, "bf16"), og.decode(bb.reshape(E * N, K), "bf16")
    dense = a @ b.T                                        # [M_total, E*N]
    for e in range(E):
        r0, r1 = int(off[e]), int(off[e + 1])
        np.testing.assert_allclose(got[r0:r1], dense[r0:r1, e * N:(e + 1) * N], rtol=1e-12, atol=1e-12)
    assert not np.isnan(got).any()
    # rows past the last offset belong to no group and stay untouched
    got2 = og.grouped_gemm_c(np.concatenate([ab, ab[:3]]), bb, off)
    assert np.isnan(got2[-3:]).all() and np.array_equal(got2[:-3], got)


def test_moe_routing_generator():
    c = wt_synth.moe_routing(1000, 16, 2, seed=5)
    assert c.sum() == 2000 and len(c) == 16 and c.min() >= 0
    assert np.array_equal(c, wt_synth.moe_routing(1000, 16, 2, seed=5))
    assert wt_synth.group_offsets([3, 0, 2]).tolist() == [0, 3, 3, 5]
