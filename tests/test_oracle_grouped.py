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


# ---- the grouped selector ----------------------------------------------------------------------
from oracle import fit as ofit        # noqa: E402
from oracle import select as osel     # noqa: E402


def _bucket(theta, anchors):
    return ofit.Bucket(theta=theta, status=15, anchors=anchors)


def test_select_grouped_hand_worked_two_keys_and_a_split_key():
    """E = 3 groups, 100 rows in all, N = 128, K = 256; the host sees only (E, M_total), so every group is taken
    to hold ceil(100/3) = 34 rows (Sec. 5.2, grouped-GEMM paragraph) and G follows Table 2's grouped row.
      key 0 <128, 64, 64>:  per group ceil(34/128) = 1 row tile x ceil(128/64) = 2 -> G = 3*2 = 6,  L = 4
                            T = 1.0*6 + 0.5*4 + 2 = 10
      key 1 <32, 64, 64>:   per group ceil(34/32) = 2 x 2 -> G = 12, L = 4;  T = 0.5*12 + 0.5*4 + 1 = 9   <- wins
      key 2 = key 0 split in two along K: a split key runs no grouped launch and is skipped although its plane
                            (T = 0.1) would win.
    Had the dense row of Table 2 been used instead (G = ceil(100/128)*2 = 2 and ceil(100/32)*2 = 8), key 0 would
    win with 1.0*2 + 2 + 2 = 6 against 0.5*8 + 2 + 1 = 7 -- so the case tells the two mappings apart.
    Stage II: key 1's anchors are L = 2 -> micro 1 and L = 8 -> micro 2; L = 4 is nearer to 2."""
    keys = [ofit.KeyDesc(128, 64, 64, 4, 2, 1, 256), ofit.KeyDesc(32, 64, 64, 4, 2, 1, 256),
            ofit.KeyDesc(128, 64, 64, 4, 2, 1, 256, 2)]
    local = [[_bucket((0.0, 1.0, 0.5, 2.0), [(4, 0)])], [_bucket((0.0, 0.5, 0.5, 1.0), [(2, 1), (8, 2)])],
             [_bucket((0.0, 0.0, 0.0, 0.1), [(2, 0)])]]
    ext = [_bucket((0.0, 0.0, 0.0, 1e6), [(4, 0)]) for _ in keys]
    table = ofit.DualTable(W=1, keys=keys, local=local, ext=ext)
    k, micro, t = osel.select_grouped(table, 3, 100, 128, 256)
    assert (k, micro) == (1, 1) and t == 9.0
    # the dense selector on the same table: the split key wins, and among unsplit keys the dense mapping picks key 0
    assert osel.select(table, 100, 128, 256)[0] == 2
    table.local[2][0].status = 0
    table.ext[2].status = 0
    k, micro, t = osel.select(table, 100, 128, 256)
    assert (k, micro) == (0, 0) and t == 6.0
    # a single group is the dense problem
    assert osel.select_grouped(table, 1, 100, 128, 256) == (0, 0, 6.0)
    # beyond the profiled waves the extrapolation tuples decide (Sec. 4.5): 3 groups of 16384 rows
    table.ext[0].theta = (0.0, 0.0, 0.0, 7.0)
    assert osel.select_grouped(table, 3, 3 * 16384, 128, 256) == (0, 0, 7.0)


def test_select_grouped_prices_the_family_of_one_groups_rows():
    """With the few-row sample families present, the family consulted for a key is that of ONE group's tile rows
    (the kernel runs E independent row bands), not of the total.  E = 3, M_total = 100 -> 34 rows per group:
      key 1 (bm = 32): 2 tile rows per group -> family 2 (2..3 rows); ceil(100/32) = 4 would be family 3.
      key 0 (bm = 128): 1 tile row either way -> family 1.
    Family buckets: key 0 / family 1 -> T = 20; key 1 / family 2 -> T = 5, family 3 -> T = 50.
    Reading one group's rows: key 1 wins at 5.  Reading the total: key 0 would win at 20."""
    keys = [ofit.KeyDesc(128, 64, 64, 4, 2, 1, 256), ofit.KeyDesc(32, 64, 64, 4, 2, 1, 256)]
    near = [[_bucket((0.0, 0.0, 0.0, 100.0), [(4, 0)])] for _ in keys]
    ext = [_bucket((0.0, 0.0, 0.0, 1e6), [(4, 0)]) for _ in keys]
    const = lambda t, micro: _bucket((0.0, 0.0, 0.0, t), [(4, micro)])
    none = lambda: ofit.Bucket()
    row_local = [[[const(20.0, 1)], [none()]],           # family 1: key 0, key 1
                 [[none()], [const(5.0, 2)]],            # family 2
                 [[none()], [const(50.0, 0)]]]           # family 3
    row_ext = [[none(), none()] for _ in range(3)]
    table = ofit.DualTable(W=1, keys=keys, local=near, ext=ext, W_row=1, row_local=row_local, row_ext=row_ext)
    assert osel.select_grouped(table, 3, 100, 128, 256) == (1, 2, 5.0)
    # the dense selector sees 4 tile rows for key 1 -> family 3 (T = 50) and picks key 0 / family 1
    assert osel.select(table, 100, 128, 256) == (0, 1, 20.0)
    # without the families both fall back to the near-square buckets: a tie at 100, lowest key id
    table.W_row = 0
    assert osel.select_grouped(table, 3, 100, 128, 256) == (0, 0, 100.0)


def test_select_grouped_with_one_group_is_the_dense_selector_on_unsplit_keys():
    """E = 1: Table 2's grouped row is its dense row and the uniform approximation is exact, so the grouped selector
    must agree with the dense one on any table without split keys -- here a table fitted from a random surface."""
    keys = [ofit.KeyDesc(256, 256, 64, 4, 2, 1, 256), ofit.KeyDesc(128, 128, 64, 4, 2, 2, 256),
            ofit.KeyDesc(64, 64, 64, 4, 2, 5, 256), ofit.KeyDesc(16, 64, 128, 1, 2, 8, 256)]
    W = 4
    local = [[_bucket(tuple(wt_synth.random_theta(300 + 11 * k, W)[w]), [(8, (k + w) % 3), (40, (k + w + 1) % 3)])
              for w in range(W)] for k in range(len(keys))]
    ext = [_bucket(tuple(wt_synth.random_theta(500 + k, 1)[0]), [(16, k % 3)]) for k in range(len(keys))]
    table = ofit.DualTable(W=W, keys=keys, local=local, ext=ext)
    rng = np.random.default_rng(5)
    seen = set()
    for _ in range(300):
        M, N, K = int(rng.integers(1, 3000)), int(rng.integers(1, 3000)), 8 * int(rng.integers(1, 700))
        got = osel.select_grouped(table, 1, M, N, K)
        assert got == osel.select(table, M, N, K)
        seen.add(got[0])
    assert len(seen) >= 2       # the case is not degenerate: more than one key gets picked


def test_select_grouped_rows_hand_worked_real_counts_flip_the_choice():
    """The table of the hand-worked case above (split key left out), N = 128, K = 256 (L = 4), 100 rows in 3 groups.
      rows (100, 0, 0): key 0 <128, 64, 64>: (1 + 0 + 0) row tiles x 2 -> G = 2, T = 1.0*2 + 0.5*4 + 2 = 6   <- wins
                        key 1 <32, 64, 64>:  (4 + 0 + 0) x 2 -> G = 8, T = 0.5*8 + 0.5*4 + 1 = 7
      (an empty group adds no tile; the uniform reading of the same launch, 34 rows each, picks key 1 at 9 against 10)
      rows (33, 33, 34): key 0: 3 x 2 -> G = 6, T = 10; key 1: (2 + 2 + 2) x 2 -> G = 12, T = 9 <- wins, as uniform.
      rows (90, 5, 5):   key 0: 3 x 2 -> 10;  key 1: (3 + 1 + 1) x 2 = 10 -> T = 5 + 2 + 1 = 8 <- wins."""
    keys = [ofit.KeyDesc(128, 64, 64, 4, 2, 1, 256), ofit.KeyDesc(32, 64, 64, 4, 2, 1, 256),
            ofit.KeyDesc(128, 64, 64, 4, 2, 1, 256, 2)]
    local = [[_bucket((0.0, 1.0, 0.5, 2.0), [(4, 0)])], [_bucket((0.0, 0.5, 0.5, 1.0), [(2, 1), (8, 2)])],
             [_bucket((0.0, 0.0, 0.0, 0.1), [(2, 0)])]]          # the split key's plane would win if it were priced
    ext = [_bucket((0.0, 0.0, 0.0, 1e6), [(4, 0)]) for _ in keys]
    table = ofit.DualTable(W=1, keys=keys, local=local, ext=ext)
    assert osel.select_grouped_rows(table, [100, 0, 0], 128, 256) == (0, 0, 6.0)
    assert osel.select_grouped(table, 3, 100, 128, 256) == (1, 1, 9.0)
    assert osel.select_grouped_rows(table, [33, 33, 34], 128, 256) == (1, 1, 9.0)
    assert osel.select_grouped_rows(table, [90, 5, 5], 128, 256) == (1, 1, 8.0)
    # one group: the dense problem on the unsplit keys
    assert osel.select_grouped_rows(table, [100], 128, 256) == (0, 0, 6.0)
    with pytest.raises(ValueError):
        osel.select_grouped_rows(table, [], 128, 256)


def test_select_grouped_rows_family_of_the_mean_group_and_uniform_equivalence():
    """Few-row families: the family consulted is that of the mean group, ceil(sum / E) rows.  rows (100, 0, 0) -> 34:
    key 1 (bm = 32) has 2 tile rows -> family 2 (T = 5), key 0 family 1 (T = 20): key 1 at 5, whatever the split of
    the 100 rows.  And on equal groups the function is select_grouped: same G, same family, same stages."""
    keys = [ofit.KeyDesc(128, 64, 64, 4, 2, 1, 256), ofit.KeyDesc(32, 64, 64, 4, 2, 1, 256)]
    near = [[_bucket((0.0, 0.0, 0.0, 100.0), [(4, 0)])] for _ in keys]
    ext = [_bucket((0.0, 0.0, 0.0, 1e6), [(4, 0)]) for _ in keys]
    const = lambda t, micro: _bucket((0.0, 0.0, 0.0, t), [(4, micro)])
    none = lambda: ofit.Bucket()
    row_local = [[[const(20.0, 1)], [none()]], [[none()], [const(5.0, 2)]], [[none()], [const(50.0, 0)]]]
    row_ext = [[none(), none()] for _ in range(3)]
    table = ofit.DualTable(W=1, keys=keys, local=near, ext=ext, W_row=1, row_local=row_local, row_ext=row_ext)
    assert osel.select_grouped_rows(table, [100, 0, 0], 128, 256) == (1, 2, 5.0)
    assert osel.select_grouped_rows(table, [40, 30, 30], 128, 256) == (1, 2, 5.0)

    keys = [ofit.KeyDesc(256, 256, 64, 4, 2, 1, 256), ofit.KeyDesc(128, 128, 64, 4, 2, 2, 256),
            ofit.KeyDesc(64, 64, 64, 4, 2, 5, 256), ofit.KeyDesc(16, 64, 128, 1, 2, 8, 256)]
    W = 4
    local = [[_bucket(tuple(wt_synth.random_theta(300 + 11 * k, W)[w]), [(8, (k + w) % 3), (40, (k + w + 1) % 3)])
              for w in range(W)] for k in range(len(keys))]
    ext = [_bucket(tuple(wt_synth.random_theta(500 + k, 1)[0]), [(16, k % 3)]) for k in range(len(keys))]
    table = ofit.DualTable(W=W, keys=keys, local=local, ext=ext)
    rng = np.random.default_rng(6)
    seen = set()
    for _ in range(300):
        E, M = int(rng.integers(1, 40)), int(rng.integers(0, 6000))
        N, K = int(rng.integers(1, 3000)), 8 * int(rng.integers(1, 700))
        got = osel.select_grouped_rows(table, geo.uniform_rows(M, E), N, K)
        assert got == osel.select_grouped(table, E, M, N, K)
        seen.add(got[0])
    assert len(seen) >= 2
