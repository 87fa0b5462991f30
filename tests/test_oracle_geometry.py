"""Pins for oracle/geometry.py and oracle/sampler.py: the paper's printed examples, closed
forms, an independent greedy-dispatch simulation, and brute force on tiny capacities."""
import math
from fractions import Fraction

import pytest

from _pins import load_pins
from oracle import geometry as geo
from oracle import sampler as smp

P = load_pins()


def test_ceil_div_against_exact_rationals():
    for a in range(0, 70):
        for b in range(1, 13):
            assert geo.ceil_div(a, b) == math.ceil(Fraction(a, b))
    with pytest.raises(ValueError):
        geo.ceil_div(3, 0)


def test_fig2_wave_quantisation_example():
    G, n = P["fig2_blocks"], P["fig2_sms"]
    assert geo.wave_count(G, geo.capacity(1, n)) == P["fig2_waves"]
    assert G // n == P["fig2_full_waves"]
    assert n - geo.last_wave_fill(G, n) == P["fig2_idle_in_last"]


def test_fig3_tile_example():
    bm, bn, bk = P["fig3_tile"]
    G, L = geo.phi_gemm(4096, 4096, P["fig3_K"], bm, bn, bk)
    assert (G, L) == (32 * 64, 64)
    assert geo.wave_count(G, P["fig3_sms"]) == 16          # 2048/132 = 15.5...


def test_region_boundaries():
    for cap in (4, 132, 256, 512, 1280):
        for w in (1, 2, 7, 40):
            lo, hi = geo.wave_region(w, cap)
            assert geo.wave_count(lo, cap) == w == geo.wave_count(hi, cap)
            assert geo.wave_count(hi + 1, cap) == w + 1
            if lo > 1:
                assert geo.wave_count(lo - 1, cap) == w - 1
    assert geo.wave_count(132, 132) == 1 and geo.wave_count(133, 132) == 2


def test_wave_count_equals_zero_variance_simulation():
    # Zero-variance greedy dispatch gives perfect steps T = mu * ceil(G / N)   (Sec. 3.2, Fig. 4)
    n, mu = P["fig4_workers"], float(P["fig4_mu"])
    for G in list(range(1, 3 * n + 3)) + [10 * n, 10 * n + 1]:
        assert geo.greedy_makespan([mu] * G, n) == mu * geo.wave_count(G, n)
    # with unequal tasks greedy dispatch beats lock-step waves
    assert geo.greedy_makespan([3, 1, 1, 1], 2) == 3.0


def test_mi355x_worked_cases():
    # 256x256 tiles, one block per CU: 16384 x 8192 -> 64*32 = 2048 tiles = exactly 8 waves
    G, L = geo.phi_gemm(16384, 8192, 8192, 256, 256, 64)
    assert (G, L, geo.wave_count(G, geo.capacity(1))) == (2048, 128, 8)
    # 4096 x 11008 -> 16*43 = 688 tiles -> 3 waves, the last one 176/256 full
    G, _ = geo.phi_gemm(4096, 11008, 4096, 256, 256, 64)
    assert (G, geo.wave_count(G, 256), geo.last_wave_fill(G, 256)) == (688, 3, 176)
    # 128x128 tiles, two blocks per CU (capacity 512): 4096 x N has 32*N/128 tiles; the wave
    # count steps up at N = 2048*k + 128
    cap = geo.capacity(2)
    assert cap == 512
    for k in (1, 2, 5):
        assert geo.wave_count(geo.phi_gemm(4096, 2048 * k, 4096, 128, 128, 64)[0], cap) == k
        assert geo.wave_count(geo.phi_gemm(4096, 2048 * k + 128, 4096, 128, 128, 64)[0], cap) == k + 1
    # skinny: M=1, N=4096, BN=64 -> 64 tiles, one wave; ragged M counts partial tiles whole
    assert geo.phi_gemm(1, 4096, 4096, 16, 64, 64) == (64, 64)
    assert geo.phi_gemm(17, 4096, 4095, 16, 64, 64) == (2 * 64, 64)
    assert geo.phi_gemm(333, 11008, 4096, 128, 128, 32) == (3 * 86, 128)


def test_phi_round_trip():
    # Sec. 4.2 instantiation followed by Table 2's mapping returns the sampled point
    for (bm, bn, bk) in [(16, 32, 128), (128, 64, 64), (256, 256, 32)]:
        for (m, n, L) in [(1, 1, 1), (5, 5, 16), (11, 12, 80), (101, 101, 160)]:
            M, N, K = smp.instantiate(m, n, L, bm, bn, bk)
            assert geo.phi_gemm(M, N, K, bm, bn, bk) == (m * n, L)


def test_occupancy_hand_cases():
    # 64 KiB LDS, 128 registers, 4 wavefronts: LDS allows 2, registers allow 4 waves/SIMD -> 4
    assert geo.occupancy_estimate(65536, 128, 4) == 2
    # 16 KiB LDS, 64 registers, 4 wavefronts: waves/SIMD min(8, 512/64)=8 -> 8 blocks; LDS 10
    assert geo.occupancy_estimate(16384, 64, 4) == 8
    # 512 registers: one wave per SIMD -> one 4-wave block, and no 8-wave block at all
    assert geo.occupancy_estimate(32768, 512, 4) == 1
    assert geo.occupancy_estimate(32768, 512, 8) == 0
    # a single-wave block with 256 registers: 2 waves per SIMD, 8 slots
    assert geo.occupancy_estimate(8192, 256, 1) == 8
    assert geo.occupancy_estimate(163840, 64, 4) == 1 and geo.occupancy_estimate(163841, 64, 4) == 0


# ---- sampler ----------------------------------------------------------------------------------
def _brute_representative(a, b, tnum, tden):
    best = None
    for m in range(1, b + 1):
        for n in range(m, b // m + 1):
            g = m * n
            if a <= g <= b and n * tden <= m * tnum and (best is None or g > best):
                best = g
    return best


def test_sub_intervals_tile_the_region():
    for cap in (4, 12, 132, 256, 250, 1280):
        for I in (1, 2, 3, 4, 7):
            for w in (1, 3):
                lo, hi = geo.wave_region(w, cap)
                ivs = [smp.sub_interval(w, i, cap, I) for i in range(1, I + 1)]
                assert ivs[0][0] == lo and ivs[-1][1] == hi
                for (a0, b0), (a1, b1) in zip(ivs, ivs[1:]):
                    assert a1 == b0 + 1
                if cap % I == 0:
                    assert all(b - a + 1 == cap // I for a, b in ivs)


def test_hand_example_132_sms():
    # N_SM = 132, I = 4, first wave: sub-intervals [1,33] [34,66] [67,99] [100,132].
    # 33=3x11, 32=4x8, 31, 30=5x6 (1.2), 29, 28=4x7, 27=3x9, 26=2x13 fail; 25=5x5 passes.
    # 66=6x11, 65=5x13 fail; 64=8x8.  99=9x11 (1.22) .. 82 fail (90=9x10 is 1.11); 81=9x9.
    # 132=11x12 (1.0909) passes.
    got = [s for s in smp.sample_set(132, 1, 4)]
    assert [(s.g, s.m, s.n) for s in got] == [(25, 5, 5), (64, 8, 8), (81, 9, 9), (132, 11, 12)]
    assert [smp.sub_interval(1, i, 132, 4) for i in (1, 2, 3, 4)] == [(1, 33), (34, 66), (67, 99), (100, 132)]


def test_tau_boundary_is_inclusive_and_integer():
    assert smp.qualifies(10, 11, 11, 10)          # ratio exactly 1.1
    assert not smp.qualifies(9, 10, 11, 10)       # 1.111...
    assert not smp.qualifies(11, 10, 11, 10)      # m <= n required
    assert smp.representative(110, 110, 11, 10) == (110, 10, 11)
    assert smp.representative(90, 90, 11, 10) is None


def test_most_square():
    assert smp.most_square(1) == (1, 1) and smp.most_square(97) == (1, 97)
    assert smp.most_square(36) == (6, 6) and smp.most_square(132) == (11, 12)
    for g in range(1, 400):
        m, n = smp.most_square(g)
        assert m * n == g and m <= n
        assert all(g % d for d in range(m + 1, math.isqrt(g) + 1))


@pytest.mark.parametrize("cap,I", [(4, 1), (4, 4), (12, 4), (132, 4), (132, 3), (60, 4)])
def test_sampler_matches_brute_force(cap, I):
    for s in smp.sample_set(cap, 6, I):
        a, b = smp.sub_interval(s.w, s.i, cap, I)
        want = _brute_representative(a, b, 11, 10)
        assert (s.g or None) == want


def test_sample_set_has_W_times_I_sub_intervals_152_non_empty_at_capacity_256():
    """Sec. 5.1 quotes 160 grid points for W = 40, I = 4: that is the nominal W*I, one slot per sub-interval.  The
    list below always has W*I entries; at capacity 256 eight of those sub-intervals hold no value with a near-square
    factorisation (g = 0 entries), so 152 real samples exist; at larger capacities every sub-interval has one."""
    W, I = P["train_W"], P["train_I"]
    for occ in (1, 2, 3, 5, 8):
        cap = geo.capacity(occ)
        S = smp.sample_set(cap, W, I, P["tau_num"], P["tau_den"])
        assert len(S) == P["train_grid_points"] == W * I
        for s in S:
            a, b = smp.sub_interval(s.w, s.i, cap, I)
            if s.g == 0:
                # a 64-wide sub-interval near g ~ 5000..10000 can hold no nearly-square product
                # (e.g. [5185, 5248] lies between 72*72 and 72*73); brute force must agree
                assert occ == 1 and _brute_representative(a, b, 11, 10) is None
                continue
            assert a <= s.g <= b and s.m * s.n == s.g and s.m <= s.n and 10 * s.n <= 11 * s.m
            assert geo.wave_count(s.g, cap) == s.w
    assert sum(s.g == 0 for s in smp.sample_set(256, W, I)) == 8
    assert sum(s.g > 0 for s in smp.sample_set(256, W, I)) == 152
    for occ in (2, 3, 5, 8):
        assert all(s.g > 0 for s in smp.sample_set(geo.capacity(occ), W, I))
    # attention's counting rule: I=3 and W in [20,35] gives 60..105 points
    assert P["attn_I"] * P["attn_W_lo"] == P["attn_points_lo"]
    assert P["attn_I"] * P["attn_W_hi"] == P["attn_points_hi"]
    # budget identity (Sec. 4.2): |G| * |L| * |macro| * |micro|
    assert smp.profile_budget(160, P["train_k_anchor_count"], 1, 1) == 800


def test_loop_anchors_per_tile_depth():
    ks = (1024, 2048, 3072, 4096, 5120)
    assert smp.loop_anchors(ks, 64) == [16, 32, 48, 64, 80]
    assert smp.loop_anchors(ks, 128) == [8, 16, 24, 32, 40]
    assert smp.loop_anchors((100, 64, 65), 64) == [1, 2]


def test_single_row_sample_set():
    # extension: 1 x g grids, g = top of each sub-interval, same regions as the paper's sampler
    S = smp.row_sample_set(256, 2, 4)
    assert [(s.w, s.i, s.g, s.m, s.n) for s in S] == [
        (1, 1, 64, 1, 64), (1, 2, 128, 1, 128), (1, 3, 192, 1, 192), (1, 4, 256, 1, 256),
        (2, 1, 320, 1, 320), (2, 2, 384, 1, 384), (2, 3, 448, 1, 448), (2, 4, 512, 1, 512)]
    for s in smp.row_sample_set(132, 5, 3):
        a, b = smp.sub_interval(s.w, s.i, 132, 3)
        assert s.g == b and geo.wave_count(s.g, 132) == s.w
        assert geo.phi_gemm(*smp.instantiate(s.m, s.n, 7, 16, 64, 128), 16, 64, 128) == (s.g, 7)


def test_few_row_sample_sets_brute_force():
    """m-row grids: the representative is the largest multiple of S*m in the sub-interval (none if the
    interval holds no multiple), found here by scanning every count."""
    for cap, m, S in ((256, 2, 1), (256, 4, 1), (256, 4, 2), (132, 4, 1), (12, 4, 1), (64, 2, 8)):
        for s in smp.row_sample_set(cap, 5, 3, m, S):
            a, b = smp.sub_interval(s.w, s.i, cap, 3)
            ok = [g for g in range(a, b + 1) if g % (S * m) == 0]
            assert s.g == (max(ok) if ok else 0)
            if s.g:
                assert (s.m, s.n) == (m, s.g // (S * m)) and geo.wave_count(s.g, cap) == s.w
    assert smp.row_sample_set(256, 3, 4, 1, 1) == smp.row_sample_set(256, 3, 4)


# ---- split-K reading of Phi and of the sampler ------------------------------------------------------
def test_split_phi_partitions_the_k_tiles():
    """S blocks per tile, each with L = ceil(ceil(K/BK)/S) k-tiles: the ranges [s*L, (s+1)*L) clipped to
    the tile's ceil(K/BK) k-tiles cover each of them exactly once, L is the longest range, and the
    nested ceiling equals ceil(K/(S*BK)).  S = 1 is Table 2's row unchanged."""
    for K in (8, 64, 100, 1000, 1024, 4096, 4104, 11008, 28672):
        for BK in (32, 64, 128, 256):
            Lt = math.ceil(Fraction(K, BK))
            assert geo.phi_gemm(300, 500, K, 128, 64, BK) == (3 * 8, Lt) == geo.phi_gemm(300, 500, K, 128, 64, BK, 1)
            for S in (2, 4, 8):
                G, L = geo.phi_gemm(300, 500, K, 128, 64, BK, S)
                assert G == S * 3 * 8
                assert L == math.ceil(Fraction(K, S * BK))
                ranges = [range(s * L, min(Lt, (s + 1) * L)) for s in range(S)]
                assert sorted(t for r in ranges for t in r) == list(range(Lt))
                assert max(len(r) for r in ranges) == L


def test_split_workspace_rule():
    lim = dict(ws_elems=1 << 26, max_tiles=1 << 16)
    assert geo.split_fits(10**6, 10**6, 256, 256, 1, **lim)
    # 2^26 floats hold 1024 tiles of 128x128 split in 4, and not one more
    assert geo.split_fits(128 * 32, 128 * 32, 128, 128, 4, **lim)
    assert not geo.split_fits(128 * 32 + 1, 128 * 32, 128, 128, 4, **lim)
    assert geo.split_fits(16 * 256, 16 * 256, 16, 16, 2, **lim) and not geo.split_fits(16 * 256 + 1, 16 * 256, 16, 16, 2, **lim)  # 2^16 tiles
    # the limits are the caller's: without them every split fits, and each works alone
    assert geo.split_fits(128 * 32 + 1, 128 * 32, 128, 128, 4) and geo.split_fits(10**5, 10**5, 16, 16, 8)
    assert not geo.split_fits(64, 64, 16, 16, 2, ws_elems=16 * 16 * 2 * 16 - 1) and geo.split_fits(64, 64, 16, 16, 2, ws_elems=16 * 16 * 2 * 16)
    assert not geo.split_fits(64, 64, 16, 16, 2, max_tiles=15) and geo.split_fits(64, 64, 16, 16, 2, max_tiles=16)


@pytest.mark.parametrize("cap,S", [(8, 2), (12, 4), (64, 2), (64, 8), (132, 4), (256, 8)])
def test_split_sampler_brute_force(cap, S):
    """Every split-K representative is the largest multiple of S in its sub-interval whose tile count
    has any factorisation with 1 <= n/m <= tau, found here by trying all (m, n)."""
    I, W = 4, 6
    for smp_ in smp.sample_set(cap, W, I, S=S):
        a, b = smp.sub_interval(smp_.w, smp_.i, cap, I)
        ok = [S * m * n for m in range(1, b + 1) for n in range(m, b // m + 1)
              if a <= S * m * n <= b and 10 * n <= 11 * m]
        assert smp_.g == (max(ok) if ok else 0)
        if smp_.g:
            assert smp_.g == S * smp_.m * smp_.n and smp_.m <= smp_.n and 10 * smp_.n <= 11 * smp_.m
            assert geo.wave_count(smp_.g, cap) == smp_.w
    assert smp.sample_set(cap, W, I, S=1) == smp.sample_set(cap, W, I)
    assert smp.loop_anchors((1024, 2048, 3072), 64, S) == sorted({math.ceil(Fraction(k, 64 * S)) for k in (1024, 2048, 3072)})
    assert smp.instantiate(3, 4, 5, 128, 64, 32, S) == (384, 256, 5 * 32 * S)
