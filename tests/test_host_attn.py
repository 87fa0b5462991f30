"""Host-side parity of the attention context (no GPU): Phi, head-aligned sampler, sampling plan, fit and
selection of libwt against the oracle."""
import os

import numpy as np
import pytest

import paper_2604_10187_amd as wt
import wt_synth
from oracle import attention as oa
from oracle import fit as ofit
from oracle import select as osel
from _pins import lib_limits, split_limits

SPLIT_LIMITS = split_limits()                 # the library's split-K workspace limits, from include/wt.h
MAX_ANCHORS = lib_limits()["max_anchors"]     # anchor slots per bucket of its table format
from oracle.geometry import ceil_div

MULT = (100, 150, 200, 250, 300)
TABLE = os.path.join(os.path.dirname(wt.LIB_PATH), "tables", "mi355x_attn.wt")


@pytest.fixture(scope="module")
def ctx():
    c = wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    yield c
    wt.wt_destroy(c)


def _keys(ctx):
    out = []
    for k in range(wt.wt_key_count(ctx)):
        c, r = wt.wt_config_get(ctx, 3 * k)
        assert r.key_id == k and c.bn == 1 and c.split == 1 and c.stages == 1
        out.append(c)
    return out


def test_attention_context_rules():
    with pytest.raises(wt.WtError):
        wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_F32)       # bf16 output only
    c = wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    try:
        assert wt.wt_config_count(c) == 3 * wt.wt_key_count(c) >= 24
        with pytest.raises(wt.WtError):
            wt.wt_set_persistent(c, True)
        with pytest.raises(wt.WtError):                          # n_heads missing
            wt.wt_sample_plan(c, wt.make_grid(W=2, I=3, k_anchors=MULT))
        # launches on a context without a device are refused with a status, batched and variable-length ones too
        cfg, _ = wt.wt_config_get(c, 0)
        for call in (lambda: wt.wt_attn(c, 4, 2, 64, 64, None, None, None, None, 0.1, 0, cfg),
                     lambda: wt.wt_attn_batched(c, 3, 4, 2, 64, 64, None, None, None, None, 0.1, 0, cfg),
                     lambda: wt.wt_attn_varlen(c, 3, 4, 2, 64, 64, None, None, None, None, None, None, 0.1, 0, cfg)):
            with pytest.raises(wt.WtError) as e:
                call()
            assert e.value.status == wt.WT_ERR_NO_DEVICE
        for call in (lambda: wt.wt_attn_batched(c, -1, 4, 2, 64, 64, None, None, None, None, 0.1, 0, cfg),
                     lambda: wt.wt_attn_batched(c, 1 << 20, 4, 2, 64, 64, None, None, None, None, 0.1, 0, cfg),
                     lambda: wt.wt_attn_varlen(c, 1025, 4, 2, 64, 64, None, None, None, None, None, None, 0.1, 0, cfg)):
            with pytest.raises(wt.WtError) as e:
                call()
            assert e.value.status == wt.WT_ERR_INVALID_ARG
    finally:
        wt.wt_destroy(c)


def test_phi_matches_table_2(ctx):
    rng = np.random.default_rng(7)
    for c in _keys(ctx):
        for _ in range(50):
            S_q, S_kv, H = int(rng.integers(1, 20000)), int(rng.integers(1, 50000)), int(rng.integers(1, 129))
            G, L = oa.phi_attn(H, S_q, S_kv, c.bm, c.bk)
            assert wt.wt_wave_count(ctx, S_q, H, S_kv, c) == (G, L, ceil_div(G, 256))


@pytest.mark.parametrize("cap,W,I,heads", [(256, 10, 3, 32), (256, 20, 3, 16), (256, 6, 3, 128), (512, 7, 4, 40),
                                           (256, 35, 3, 64), (100, 9, 5, 7)])
def test_head_aligned_sampler_bit_exact(cap, W, I, heads):
    g, q = wt.wt_sample_grid_heads(cap, W, I, heads)
    want = oa.sample_set_heads(cap, W, I, heads)
    assert [(int(a), int(b)) for a, b in zip(g, q)] == [(s.g, s.q_tiles) for s in want]


def _plan(keys, W, I, heads):
    """(key, g, w, L) of every workload, from the oracle's rules (capacity 256)."""
    out = []
    for k, c in enumerate(keys):
        for s in oa.sample_set_heads(256, W, I, heads):
            if s.g == 0:
                continue
            S_q, _ = oa.instantiate_attn(s.g, 1, heads, c.bm, c.bk)
            for L in oa.kv_loop_counts(S_q, c.bk, MULT):
                out.append((k, s.g, s.w, L))
    return out


@pytest.mark.parametrize("heads", [16, 32, 128])
def test_sampling_plan_counts_and_buffers(ctx, heads):
    keys = _keys(ctx)
    W, I = 6, 3
    plan = _plan(keys, W, I, heads)
    n, bQ, bKV, bO = wt.wt_sample_plan(ctx, wt.make_grid(W=W, I=I, k_anchors=MULT, n_heads=heads))
    assert n == 3 * len(plan)
    sq = max(oa.instantiate_attn(g, L, heads, keys[k].bm, keys[k].bk)[0] for k, g, w, L in plan)
    skv = max(oa.instantiate_attn(g, L, heads, keys[k].bm, keys[k].bk)[1] for k, g, w, L in plan)
    assert (bQ, bKV, bO) == (sq * heads * 128 * 2, skv * heads * 128 * 4, sq * heads * 128 * 2)


def test_fit_and_select_parity_on_a_synthetic_surface(ctx, tmp_path):
    keys = _keys(ctx)
    W, I, p, heads = 8, 3, 4, 32
    recs = []
    for (k, g, w, L) in _plan(keys, W, I, heads):
        th = wt_synth.random_theta(900 + k, W)[w - 1]
        scale = keys[k].bm * keys[k].bk / (128.0 * 64)
        for micro in range(3):
            t = scale * (th[0] * g * L + th[1] * g) + th[2] * L + th[3]
            recs.append((k, micro, g, L, w, 0, t * (1.0 + 0.04 * ((micro + L // 5 + k) % 3))))
    samples = np.array(recs, dtype=wt.SAMPLE_DTYPE)
    wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=p, k_anchors=MULT, n_heads=heads), samples)
    path = str(tmp_path / "attn.wt")
    wt.wt_save(ctx, path)
    table, _ = osel.read_table(path, **SPLIT_LIMITS)
    kds = table.keys
    assert [(kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, kd.cap, kd.split) for kd in kds] == \
        [(c.bm, 1, c.bk, c.nwave, 1, 256, 1) for c in keys]
    want = ofit.fit_tables([tuple(r)[:5] + (float(r["mean_us"]),) for r in samples], kds, W, p, max_anchors=MAX_ANCHORS)
    for k in range(len(keys)):
        for gb, wb in list(zip(table.local[k], want.local[k])) + [(table.ext[k], want.ext[k])]:
            assert gb.status == wb.status and gb.anchors == wb.anchors
    for (S_q, S_kv, H_q, _) in wt_synth.attn_shapes(400, 11):
        key, micro, t = osel.select_attn(table, H_q, S_q, S_kv)
        c = wt.wt_select(ctx, S_q, H_q, S_kv)
        assert (c.bm, c.bk, c.nwave, c.swizzle) == (keys[key].bm, keys[key].bk, keys[key].nwave, micro)
        assert wt.wt_predict_us(ctx, S_q, H_q, S_kv, c) == t
    _varlen_selection_matches(ctx, table, keys, seed=21)


def _varlen_selection_matches(ctx, table, keys, seed):
    """wt_select_attn_varlen against the oracle's select_attn_varlen on ragged batches (prefill: keys = queries; decode
    and chunked prefill: keys > queries; some empty sequences), and its reduction to wt_select on equal lengths."""
    rng = np.random.default_rng(seed)
    batches = wt_synth.varlen_batches(60, seed) + wt_synth.varlen_batches(40, seed + 1, lo=1, hi=700)
    differs = 0
    for i, lens in enumerate(batches):
        H_q = int(wt_synth.ATTN_Q_HEADS[i % 4])
        lq = list(lens)
        lkv = list(lens) if i % 3 else [s + int(rng.integers(0, 4000)) for s in lens]
        if i % 7 == 0:
            lq[0] = 0
        key, micro, _ = osel.select_attn_varlen(table, H_q, lq, lkv)
        c = wt.wt_select_attn_varlen(ctx, lq, lkv, H_q)
        assert (c.bm, c.bk, c.nwave, c.swizzle) == (keys[key].bm, keys[key].bk, keys[key].nwave, micro), (lq, lkv, H_q)
        mean_q, mean_kv = -(-sum(lq) // len(lq)), -(-sum(lkv) // len(lkv))
        differs += wt.wt_select(ctx, mean_q, len(lq) * H_q, mean_kv).id != c.id
    assert differs >= 3          # pricing the real lengths is not pricing the mean length
    for (S_q, S_kv, H_q, _) in wt_synth.attn_shapes(40, seed + 2):
        for b in (1, 3):
            assert wt.wt_select_attn_varlen(ctx, [S_q] * b, [S_kv] * b, H_q).id == wt.wt_select(ctx, S_q, b * H_q, S_kv).id


def test_varlen_selector_argument_checks(ctx):
    INV = wt.WT_ERR_INVALID_ARG
    for (lq, lkv, H) in [([], [], 8), ([1] * 1025, [1] * 1025, 8), ([5, -1], [5, 5], 8), ([5, 5], [5, -2], 8),
                         ([5], [5], 0), ([5], [5], 65537), ([2**30] * 3, [1] * 3, 8), ([1] * 3, [2**30] * 3, 8),
                         ([2**30], [2**30], 65536)]:
        with pytest.raises(wt.WtError) as e:
            wt.wt_select_attn_varlen(ctx, lq, lkv, H)
        assert e.value.status == INV, (len(lq), H)
    with pytest.raises(ValueError):
        wt.wt_select_attn_varlen(ctx, [1, 2], [1], 8)
    fresh = wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    gemm = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_BF16)
    try:
        with pytest.raises(wt.WtError) as e:
            wt.wt_select_attn_varlen(fresh, [5], [5], 8)
        assert e.value.status == wt.WT_ERR_NOT_FITTED
        with pytest.raises(wt.WtError) as e:
            wt.wt_select_attn_varlen(gemm, [5], [5], 8)
        assert e.value.status == INV
        with pytest.raises(wt.WtError) as e:
            wt.wt_select_grouped_rows(fresh, [5], 8, 8)
        assert e.value.status == INV
    finally:
        wt.wt_destroy(fresh)
        wt.wt_destroy(gemm)


def test_shipped_attention_table_selects_like_the_oracle():
    c = wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    try:
        wt.wt_load(c, TABLE)
        table, meta = osel.read_table(TABLE, **SPLIT_LIMITS)
        keys = _keys(c)
        assert len(table.keys) == len(keys)
        for (S_q, S_kv, H_q, _) in wt_synth.attn_shapes(300, 12):
            key, micro, t = osel.select_attn(table, H_q, S_q, S_kv)
            got = wt.wt_select(c, S_q, H_q, S_kv)
            assert (got.bm, got.bk, got.nwave, got.swizzle) == (keys[key].bm, keys[key].bk, keys[key].nwave, micro)
            assert wt.wt_predict_us(c, S_q, H_q, S_kv, got) == t
        _varlen_selection_matches(c, table, keys, seed=31)
    finally:
        wt.wt_destroy(c)
