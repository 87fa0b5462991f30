"""Pins for oracle/attention.py: the attention definition against closed forms, brute force and a library
routine; the attention row of Table 2, the head-aligned representative of Sec. 4.2 and Eq. 6 against hand
values, brute force and the grid-point counts the paper states (60-105 for I = 3, W = 20..35)."""
import math

import numpy as np
import pytest
import torch

from _pins import load_pins
from oracle import attention as att
from oracle.sampler import sub_interval


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_zero_queries_give_the_mean_of_v():
    K, V = _rand((37, 2, 8), 1), _rand((37, 2, 8), 2)
    out = att.attention(np.zeros((5, 4, 8)), K, V, 0.3)
    for h in range(4):
        np.testing.assert_allclose(out[:, h], np.broadcast_to(V[:, h // 2].mean(0), (5, 8)), rtol=0, atol=1e-14)


def test_zero_queries_causal_give_prefix_means_aligned_to_the_end():
    V = _rand((9, 1, 4), 3)
    out = att.attention(np.zeros((4, 1, 4)), _rand((9, 1, 4), 4), V, 1.0, causal=True)
    for i in range(4):  # query i is token 5 + i of 9 and sees keys 0 .. 5 + i
        np.testing.assert_allclose(out[i, 0], V[: 6 + i, 0].mean(0), rtol=0, atol=1e-14)


def test_single_key_returns_its_value():
    V = _rand((1, 3, 16), 5)
    out = att.attention(_rand((7, 3, 16), 6), _rand((1, 3, 16), 7), V, 0.7)
    np.testing.assert_allclose(out, np.broadcast_to(V, (7, 3, 16)), rtol=0, atol=1e-15)


def test_two_keys_closed_form_is_a_logistic_mixture():
    q, k0, k1, v0, v1, s = 0.8, 1.5, -0.25, 2.0, -3.0, 0.37
    out = att.attention(np.full((1, 1, 1), q), np.array([[[k0]], [[k1]]]), np.array([[[v0]], [[v1]]]), s)
    p0 = 1.0 / (1.0 + math.exp(-s * q * (k0 - k1)))
    assert out[0, 0, 0] == pytest.approx(p0 * v0 + (1 - p0) * v1, abs=1e-15)


def test_a_dominant_key_selects_its_value_row():
    D = 8
    K = 50.0 * np.eye(D)[:, None, :]           # 8 keys, one head, orthogonal
    V = _rand((D, 1, D), 8)
    Q = np.eye(D)[[3, 0, 6], None, :]          # queries aligned with keys 3, 0, 6
    out = att.attention(Q, K, V, 1.0)
    np.testing.assert_allclose(out[:, 0], V[[3, 0, 6], 0], rtol=0, atol=1e-12)


def test_adding_one_vector_to_every_key_changes_nothing():
    Q, K, V = _rand((6, 2, 8), 9), _rand((11, 2, 8), 10), _rand((11, 2, 8), 11)
    c = _rand((1, 2, 8), 12)
    np.testing.assert_allclose(att.attention(Q, K + c, V, 0.35), att.attention(Q, K, V, 0.35), rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal,S_q,S_kv", [(False, 5, 13), (True, 4, 4), (True, 3, 10)])
def test_against_explicit_loops(causal, S_q, S_kv):
    H_q, H_kv, D, scale = 4, 2, 3, 0.41
    Q, K, V = _rand((S_q, H_q, D), 13), _rand((S_kv, H_kv, D), 14), _rand((S_kv, H_kv, D), 15)
    got = att.attention(Q, K, V, scale, causal)
    for i in range(S_q):
        for h in range(H_q):
            kh = h // (H_q // H_kv)
            vis = [j for j in range(S_kv) if not causal or j <= i + S_kv - S_q]
            wts = [math.exp(scale * sum(Q[i, h, d] * K[j, kh, d] for d in range(D))) for j in vis]
            for d in range(D):
                ref = sum(w * V[j, kh, d] for w, j in zip(wts, vis)) / sum(wts)
                assert got[i, h, d] == pytest.approx(ref, abs=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_against_the_library_routine_in_fp64(causal):
    S, H_q, H_kv, D = 33, 6, 2, 16
    Q, K, V = _rand((S, H_q, D), 16), _rand((S, H_kv, D), 17), _rand((S, H_kv, D), 18)
    tq = torch.from_numpy(Q).permute(1, 0, 2)
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(H_q // H_kv, dim=0)
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(H_q // H_kv, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=0.2)
    np.testing.assert_allclose(att.attention(Q, K, V, 0.2, causal), ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)


def test_rejects_mismatched_heads_and_short_causal_context():
    with pytest.raises(ValueError):
        att.attention(np.zeros((2, 3, 4)), np.zeros((2, 2, 4)), np.zeros((2, 2, 4)), 1.0)
    with pytest.raises(ValueError):
        att.attention(np.zeros((5, 1, 4)), np.zeros((2, 1, 4)), np.zeros((2, 1, 4)), 1.0, causal=True)


# ---- Table 2 (FlashAttention row), Sec. 4.2 head alignment, Eq. 6 -----------------------------------

def test_phi_attn_hand_values():
    assert att.phi_attn(32, 1000, 1000, 128, 64) == (32 * 8, 16)
    assert att.phi_attn(16, 128, 129, 128, 128) == (16, 2)
    assert att.phi_attn(128, 1, 1, 256, 32) == (128, 1)
    assert att.phi_attn(8, 0, 64, 64, 64) == (0, 1)


def test_phi_attn_varlen_hand_values_block_enumeration_and_equal_lengths():
    """Two sequences of 100 and 300 tokens (queries = keys), T_Q = 128, T_KV = 64, 2 heads: 1 and 3 query tiles per
    head, looping 2 and 5 times -> 4 tiles, 2 + 15 = 17 iterations per head, mean 4.25 -> L = 4, G = 8.  A mean of
    exactly 2.5 (one tile looping twice, one three times) rounds up to 3."""
    from fractions import Fraction

    assert att.phi_attn_varlen(2, [100, 300], [100, 300], 128, 64) == (8, 4)
    assert att.phi_attn_varlen(1, [10, 10], [100, 150], 64, 64) == (2, 3)
    assert att.phi_attn_varlen(4, [0, 0], [64, 64], 64, 64) == (0, 0)
    assert att.phi_attn_varlen(4, [], [], 64, 64) == (0, 0)
    assert att.phi_attn_varlen(3, [5, 0, 70], [0, 900, 70], 64, 32) == (9, 2)      # tiles 1, 0, 2; loops 0, 29, 3
    with pytest.raises(ValueError):
        att.phi_attn_varlen(2, [1, 2], [1], 64, 64)
    # every block listed one by one: G is their number, L the mean of their loop counts rounded half up
    rng = np.random.default_rng(12)
    for _ in range(200):
        b, H = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        T_Q, T_KV = int(rng.choice([64, 128, 256])), int(rng.choice([32, 64, 128]))
        lq = [int(x) for x in rng.integers(0, 3000, size=b)]
        lkv = [int(x) for x in rng.integers(0, 5000, size=b)]
        blocks = [-(-kv // T_KV) for q, kv in zip(lq, lkv) for _h in range(H) for _t in range(-(-q // T_Q))]
        G, L = att.phi_attn_varlen(H, lq, lkv, T_Q, T_KV)
        assert G == len(blocks)
        if blocks:
            assert L == math.floor(Fraction(sum(blocks), len(blocks)) + Fraction(1, 2))
            assert abs(G * L - sum(blocks)) * 2 <= G
    # equal lengths: Table 2's row with the batch folded into the head count
    for (b, H, S_q, S_kv, T_Q, T_KV) in [(1, 8, 300, 1000, 64, 32), (4, 32, 1024, 2048, 256, 128), (7, 5, 1, 1, 128, 64)]:
        assert att.phi_attn_varlen(H, [S_q] * b, [S_kv] * b, T_Q, T_KV) == att.phi_attn(b * H, S_q, S_kv, T_Q, T_KV)


@pytest.mark.parametrize("n_heads", [1, 7, 16, 40, 128])
def test_representative_heads_is_the_largest_multiple_in_the_interval(n_heads):
    rng = np.random.default_rng(n_heads)
    for _ in range(200):
        a = int(rng.integers(1, 3000))
        b = a + int(rng.integers(0, 300))
        brute = max((g for g in range(a, b + 1) if g % n_heads == 0), default=0)
        assert att.representative_heads(a, b, n_heads) == brute


def test_grid_point_counts_match_the_paper_s_range():
    # Sec. 5.1 (values in tests/golden/paper_pins.txt): I = 3 and W from 20 to 35 give 60 to 105 grid points per
    # KV-length anchor -- the sampler must produce exactly that many when every sub-interval holds a head multiple
    P = load_pins()
    I, W_lo, W_hi = P["attn_I"], P["attn_W_lo"], P["attn_W_hi"]
    for W, n_heads in ((W_lo, 16), (W_hi, 128)):
        pts = att.sample_set_heads(256 * 2, W, I, n_heads)  # capacity 512: every third holds a multiple of 128
        assert len(pts) == I * W and all(p.g > 0 for p in pts)
    assert sum(p.g > 0 for p in att.sample_set_heads(256, W_lo, I, 16)) == P["attn_points_lo"]
    assert sum(p.g > 0 for p in att.sample_set_heads(256, W_hi, I, 64)) == P["attn_points_hi"]


def test_sample_set_heads_layout_and_alignment():
    pts = att.sample_set_heads(256, 4, 3, 128)
    assert [(p.w, p.i) for p in pts] == [(w, i) for w in range(1, 5) for i in range(1, 4)]
    # [1,85] holds no multiple of 128; [86,170] -> 128; [171,256] -> 256
    assert [p.g for p in pts[:3]] == [0, 128, 256]
    for p in pts:
        a, b = sub_interval(p.w, p.i, 256, 3)
        assert p.g == 0 or (a <= p.g <= b and p.g % 128 == 0 and p.q_tiles * 128 == p.g)


def test_instantiate_attn_round_trips_through_phi():
    for n_heads, T_Q, T_KV in ((16, 64, 32), (32, 128, 64), (128, 256, 128)):
        for p in att.sample_set_heads(256, 6, 3, n_heads):
            if p.g == 0:
                continue
            for L in (1, 7, 40):
                S_q, S_kv = att.instantiate_attn(p.g, L, n_heads, T_Q, T_KV)
                assert (S_q, S_kv) == (p.q_tiles * T_Q, L * T_KV)
                assert att.phi_attn(n_heads, S_q, S_kv, T_Q, T_KV) == (p.g, L)
    with pytest.raises(ValueError):
        att.instantiate_attn(33, 1, 32, 64, 64)


def test_kv_loop_counts_hand_values():
    # S_q = 1024, T_KV = 64: multipliers 1.0, 1.5, 2.0, 2.5, 3.0 -> S_kv 1024 .. 3072 -> L = 16, 24, 32, 40, 48
    assert att.kv_loop_counts(1024, 64, (100, 150, 200, 250, 300)) == [16, 24, 32, 40, 48]
    # S_q = 64, T_KV = 128: 64, 96, 128, 160, 192 tokens -> 1, 1, 1, 2, 2 iterations, merged
    assert att.kv_loop_counts(64, 128, (100, 150, 200, 250, 300)) == [1, 2]
