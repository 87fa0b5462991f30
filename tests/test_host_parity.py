"""CPU-side parity of libwt's host half against the oracle (no GPU): the library loads and
exports every declared symbol; Phi / wave counts, the sampler and table lookups are bit-exact;
fitted coefficients agree to 1e-9."""
import os
import re

import numpy as np
import pytest

import paper_2604_10187_amd as wt
import wt_synth
from oracle import fit as ofit
from oracle import geometry as geo
from oracle import sampler as smp
from oracle import select as osel
from _pins import lib_limits, split_limits

SPLIT_LIMITS = split_limits()                 # the library's split-K workspace limits, from include/wt.h
MAX_ANCHORS = lib_limits()["max_anchors"]     # anchor slots per bucket of its table format

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
K_ANCHORS = (1024, 2048, 3072, 4096, 5120)
W_SPLIT = 6        # waves for which the synthetic split-K keys have records


@pytest.fixture(scope="module")
def ctx():
    c = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
    yield c
    wt.wt_destroy(c)


def _keys(ctx, occ_aware=False):
    """Structural keys as the oracle sees them; capacity = 256 CUs (default mode) or 256 x occupancy."""
    out = []
    for i in range(0, wt.wt_config_count(ctx), 3):
        c, r = wt.wt_config_get(ctx, i)
        out.append(ofit.KeyDesc(c.bm, c.bn, c.bk, c.nwave, c.stages, r.occ, geo.capacity(r.occ if occ_aware else 1), c.split))
    return out


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wt.h")).read()
    declared = set(re.findall(r"\b(wt_[a-z_0-9]+)\s*\(", header))
    assert declared == set(wt.EXPORTS)
    L = wt.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_persistent_modes_are_checked():
    """Launch policy: 0 one block per task, 1 fixed stride, 2 device-side queue (needs a device context)."""
    c = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_BF16)
    try:
        wt.wt_set_persistent(c, 1)
        wt.wt_set_persistent(c, 0)
        with pytest.raises(wt.WtError) as e:
            wt.wt_set_persistent(c, 2)
        assert e.value.status == wt.WT_ERR_NO_DEVICE
        for bad in (-1, 3):
            with pytest.raises(wt.WtError) as e:
                wt.wt_set_persistent(c, bad)
            assert e.value.status == wt.WT_ERR_INVALID_ARG
    finally:
        wt.wt_destroy(c)


def test_binding_states_the_headers_limits():
    lim = lib_limits()
    assert (wt.WT_SPLITK_WS_FLOATS, wt.WT_SPLITK_MAX_TILES, wt.WT_MAX_ANCHORS) == (lim["ws_elems"], lim["max_split_tiles"], lim["max_anchors"])


def test_oversized_grids_and_foreign_tables_are_refused(tmp_path):
    """No exception crosses the ABI and nothing that can be fitted and saved fails to load: W and I beyond 4096
    are invalid arguments for wt_fit / wt_sample_grid / wt_sample_plan, and a table written for another output
    type or another compute-unit count is refused by wt_load."""
    c = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_BF16)
    other = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
    try:
        one = np.zeros(1, dtype=wt.SAMPLE_DTYPE)
        one["w"], one["G"], one["L"], one["mean_us"] = 1, 10, 4, 1.0
        for bad in (dict(W=4097), dict(W=2**31 - 1), dict(I=0), dict(W=0)):
            with pytest.raises(wt.WtError) as e:
                wt.wt_fit(c, wt.make_grid(**{**dict(W=4, I=2, p=2), **bad}), one)
            assert e.value.status == wt.WT_ERR_INVALID_ARG
        import ctypes
        got = ctypes.c_size_t()      # straight through the ABI (the binding would size host arrays from W * I)
        assert wt.lib().wt_sample_grid(256, 2**31 - 1, 4, 11, 10, 1, None, None, None, 0, ctypes.byref(got)) == wt.WT_ERR_INVALID_ARG
        assert wt.lib().wt_sample_grid_heads(256, 4, 2**31 - 1, 8, None, None, 0, ctypes.byref(got)) == wt.WT_ERR_INVALID_ARG
        with pytest.raises(wt.WtError) as e:
            wt.wt_sample_plan(c, wt.make_grid(W=2**31 - 1, I=4))
        assert e.value.status == wt.WT_ERR_INVALID_ARG
        wt.wt_fit(c, wt.make_grid(W=4096, I=1, p=1), one)       # the largest W is accepted ...
        path = str(tmp_path / "big.wt")
        wt.wt_save(c, path)
        wt.wt_load(c, path)                                      # ... and loads again
        with pytest.raises(wt.WtError) as e:                     # bf16-out table into an f32-out context
            wt.wt_load(other, path)
        assert e.value.status == wt.WT_ERR_INVALID_ARG
        raw = bytearray(open(path, "rb").read())
        raw[32:36] = (132).to_bytes(4, "little")                 # header word 8: compute units
        p2 = tmp_path / "cu.wt"
        p2.write_bytes(bytes(raw))
        with pytest.raises(wt.WtError) as e:
            wt.wt_load(c, str(p2))
        assert e.value.status == wt.WT_ERR_INVALID_ARG
    finally:
        wt.wt_destroy(c)
        wt.wt_destroy(other)


def test_registry_shape(ctx):
    n = wt.wt_config_count(ctx)
    assert n == 3 * wt.wt_key_count(ctx) and n >= 100
    seen = set()
    for i in range(n):
        c, r = wt.wt_config_get(ctx, i)
        assert c.id == i and r.key_id == i // 3 and r.micro_id == c.swizzle == i % 3
        assert r.lds_bytes == (c.bm + c.bn) * c.bk * 2 * c.stages <= 160 * 1024
        assert wt.wt_config_find(ctx, *c.astuple()) == i
        assert c.split in (1, 2, 4, 8)
        seen.add(c.astuple())
    assert len(seen) == n
    # split-K keys come after every unsplit key and reuse an unsplit key's kernel
    splits = [wt.wt_config_get(ctx, i)[0].split for i in range(0, n, 3)]
    first = next(i for i, sp in enumerate(splits) if sp > 1)
    assert all(sp == 1 for sp in splits[:first]) and all(sp > 1 for sp in splits[first:]) and first >= 50
    for i in range(3 * first, n, 3):
        c, _ = wt.wt_config_get(ctx, i)
        assert wt.wt_config_find(ctx, c.bm, c.bn, c.bk, c.nwave, c.stages, 0, 1) < 3 * first
    with pytest.raises(wt.WtError):
        wt.wt_config_find(ctx, 48, 48, 64, 4, 2, 0)
    with pytest.raises(wt.WtError):
        wt.wt_config_find(ctx, 128, 128, 64, 4, 3, 0, 3)


def test_device_calls_refused_on_host_context(ctx):
    c, _ = wt.wt_config_get(ctx, 0)
    a = np.zeros(64, dtype=np.uint16)
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx, 1, 1, 8, a, a, a, c)
    assert e.value.status == wt.WT_ERR_NO_DEVICE


def test_wave_counts_bit_exact(ctx):
    shapes = wt_synth.sweep_shapes() + wt_synth.wave_stress_shapes()[::7] + wt_synth.stream_shapes(200)
    shapes += [(16384, 8192, 8192), (1, 1, 8), (0, 5, 8)]
    for i in range(0, wt.wt_config_count(ctx), 3):
        c, r = wt.wt_config_get(ctx, i)
        cap = geo.capacity(1)
        for (M, N, K) in shapes:
            G, L = geo.phi_gemm(M, N, K, c.bm, c.bn, c.bk, c.split)
            assert wt.wt_wave_count(ctx, M, N, K, c) == (G, L, geo.wave_count(G, cap))
    # in the occupancy-aware mode an occupancy override moves the wave boundaries
    c, r = wt.wt_config_get(ctx, 0)
    assert wt.wt_wave_count(ctx, 256 * 20, 256 * 40, 64, c)[2] == geo.wave_count(800, 256) == 4
    wt.wt_set_capacity_mode(ctx, wt.WT_CAP_CU_TIMES_OCC)
    wt.wt_key_set_occ(ctx, 0, 3)
    assert wt.wt_wave_count(ctx, 256 * 20, 256 * 40, 64, c)[2] == geo.wave_count(800, 768) == 2
    wt.wt_key_set_occ(ctx, 0, r.occ)
    wt.wt_set_capacity_mode(ctx, wt.WT_CAP_CU_ONLY)


@pytest.mark.parametrize("cap", [4, 12, 132, 256, 512, 768, 1280, 2048, 250])
@pytest.mark.parametrize("I", [1, 3, 4])
def test_sampler_bit_exact(cap, I):
    W = 40 if cap >= 132 else 9
    g, m, n = wt.wt_sample_grid(cap, W, I)
    want = smp.sample_set(cap, W, I)
    assert len(g) == len(want) == W * I
    assert [(int(a), int(b), int(c)) for a, b, c in zip(g, m, n)] == [(s.g, s.m, s.n) for s in want]


@pytest.mark.parametrize("cap", [256, 512, 768, 250, 12])
@pytest.mark.parametrize("S", [2, 4, 8])
@pytest.mark.parametrize("I", [1, 3, 4])
def test_sampler_split_bit_exact(cap, S, I):
    """Split-K keys: task counts are multiples of S; the library derives the tile-count interval and
    searches it, the oracle scans task counts downwards -- same samples."""
    W = 12
    g, m, n = wt.wt_sample_grid(cap, W, I, split=S)
    want = smp.sample_set(cap, W, I, S=S)
    assert [(int(a), int(b), int(c)) for a, b, c in zip(g, m, n)] == [(s.g, s.m, s.n) for s in want]
    assert all(int(a) == S * int(b) * int(c) for a, b, c in zip(g, m, n))


def test_sampler_other_tau():
    for tnum, tden in ((3, 2), (1, 1), (2, 1)):
        g, m, n = wt.wt_sample_grid(132, 5, 4, tnum, tden)
        want = smp.sample_set(132, 5, 4, tnum, tden)
        assert [(int(a), int(b), int(c)) for a, b, c in zip(g, m, n)] == [(s.g, s.m, s.n) for s in want]


# ---- fit + select on a synthetic latency surface --------------------------------------------------
def _synthetic_samples(keys, W, I, noise_seed=None):
    recs = []
    for k, kd in enumerate(keys):
        th = wt_synth.random_theta(300 + k, W)
        scale = (kd.bm * kd.bn * kd.bk) / (128.0 * 128 * 64)      # bigger tiles cost more per (tile x loop)
        # split-K keys are profiled for the first waves only and cost a little extra per task
        Wk = W if kd.split == 1 else min(W, W_SPLIT)
        for s in smp.sample_set(kd.cap, Wk, I, S=kd.split):
            if s.g == 0 or not geo.split_fits(s.m * kd.bm, s.n * kd.bn, kd.bm, kd.bn, kd.split, SPLIT_LIMITS["ws_elems"], SPLIT_LIMITS["max_split_tiles"]):
                continue                              # no such grid, or it cannot run: never profiled
            for L in smp.loop_anchors(K_ANCHORS, kd.bk, kd.split):
                for micro in range(3):
                    a, b, c, d = th[s.w - 1]
                    t = scale * (a * s.g * L + b * s.g * (1.0 + 0.05 * (kd.split > 1))) + c * L + d
                    t *= 1.0 + 0.03 * ((micro + L // 8 + k) % 3)     # micro preference varies with L
                    recs.append((k, micro, s.g, L, s.w, 0, t))
    arr = np.array(recs, dtype=wt.SAMPLE_DTYPE)
    if noise_seed is not None:
        arr["mean_us"] *= wt_synth.noise_factors(len(arr), noise_seed, 0.02)
    return arr


@pytest.mark.parametrize("noise_seed,weighting", [(None, 0), (5, 0), (None, 1), (5, 1), (6, 1)])
def test_fit_and_select_parity(ctx, tmp_path, noise_seed, weighting):
    """weighting 0: ordinary least squares per bucket; 1: relative residuals (every record weighs 1/T^2)."""
    W, I, p = 12, 4, 5
    keys = _keys(ctx)
    samples = _synthetic_samples(keys, W, I, noise_seed)
    grid = wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, weighting=weighting)
    wt.wt_fit(ctx, grid, samples)
    path = str(tmp_path / "table.wt")
    wt.wt_save(ctx, path)
    table, meta = osel.read_table(path, **SPLIT_LIMITS)
    assert meta["I"] == I and meta["p"] == p and table.W == W and len(table.keys) == len(keys)
    assert meta["weighting"] == weighting
    assert table.keys == keys
    # (1) coefficients and anchors against the oracle's own fit of the same records
    want = ofit.fit_tables([tuple(r)[:5] + (float(r["mean_us"]),) for r in samples], keys, W, p, max_anchors=MAX_ANCHORS,
                           relative=bool(weighting))
    if weighting and noise_seed is not None:
        # the two objectives are different fits: on noisy records the relative table is not the absolute one
        other = ofit.fit_tables([tuple(r)[:5] + (float(r["mean_us"]),) for r in samples], keys, W, p, max_anchors=MAX_ANCHORS)
        assert any(not np.allclose(a.theta, b.theta, rtol=1e-6, atol=0.0)
                   for k in range(len(keys)) for a, b in zip(want.local[k], other.local[k]) if a.status == 0b1111)
    for k in range(len(keys)):
        for got_b, want_b in list(zip(table.local[k], want.local[k])) + [(table.ext[k], want.ext[k])]:
            assert got_b.status == want_b.status and got_b.anchors == want_b.anchors
            scale = max(abs(x) for x in want_b.theta) or 1.0
            # compare through predictions at the bucket's scale (coefficients cancel heavily)
            assert np.allclose(got_b.theta, want_b.theta, rtol=1e-9, atol=1e-9 * scale) or \
                _pred_close(got_b.theta, want_b.theta, keys[k])
    # (2) lookups bit-exact: the oracle's selector on the very table the library wrote
    shapes = wt_synth.sweep_shapes() + wt_synth.stream_shapes(3000) + wt_synth.wave_stress_shapes()[::5]
    for (M, N, K) in shapes:
        key, micro, t = osel.select(table, M, N, K)
        c = wt.wt_select(ctx, M, N, K)
        kd = keys[key]
        assert (c.bm, c.bn, c.bk, c.nwave, c.stages, c.swizzle, c.split) == (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, micro, kd.split)
        assert wt.wt_predict_us(ctx, M, N, K, c) == t        # same bits, not merely close
    # (3) load round trip gives the same decisions
    ctx2 = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
    try:
        with pytest.raises(wt.WtError) as e:
            wt.wt_select(ctx2, 64, 64, 64)
        assert e.value.status == wt.WT_ERR_NOT_FITTED
        wt.wt_load(ctx2, path)
        for (M, N, K) in shapes[:300]:
            assert wt.wt_select(ctx2, M, N, K).id == wt.wt_select(ctx, M, N, K).id
    finally:
        wt.wt_destroy(ctx2)


def test_split_keys_in_selection(ctx, tmp_path):
    """Split-K keys take part in Stage I with G = S*tiles and L = ceil(K/(S*bk)); outside their profiled
    waves (no bucket, no extrapolation tuple) and where their partial tiles exceed the workspace they are
    not candidates.  Decisions and predictions equal the oracle's bit for bit."""
    W, I, p = 12, 4, 5
    keys = _keys(ctx)
    samples = _synthetic_samples(keys, W, I, noise_seed=21)
    grid = wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_split=W_SPLIT)
    wt.wt_fit(ctx, grid, samples)
    path = str(tmp_path / "split.wt")
    wt.wt_save(ctx, path)
    table, _ = osel.read_table(path, **SPLIT_LIMITS)
    assert table.keys == keys
    # the plan holds exactly the records the oracle's sampler enumerates (3 micros each)
    n_plan, *_ = wt.wt_sample_plan(ctx, grid)
    assert n_plan == len(samples)
    picked_split = 0
    shapes = wt_synth.sweep_shapes() + wt_synth.stream_shapes(1500) + [(256, 256, 8192), (64, 512, 16384), (8, 1024, 4096)]
    for (M, N, K) in shapes:
        key, micro, t = osel.select(table, M, N, K)
        c = wt.wt_select(ctx, M, N, K)
        assert c.id == 3 * key + micro and wt.wt_predict_us(ctx, M, N, K, c) == t
        picked_split += keys[key].split > 1
    assert picked_split >= 10
    for k, kd in enumerate(keys):
        if kd.split == 1:
            continue
        cfg, _ = wt.wt_config_get(ctx, 3 * k)
        assert not table.ext[k].status                       # nothing profiled in the last p waves
        M = N = 16 * 1024                                     # far beyond the profiled waves
        G, L = geo.phi_gemm(M, N, 4096, kd.bm, kd.bn, kd.bk, kd.split)
        assert geo.wave_count(G, kd.cap) > W_SPLIT
        with pytest.raises(wt.WtError) as e:
            wt.wt_predict_us(ctx, M, N, 4096, cfg)
        fits = geo.split_fits(M, N, kd.bm, kd.bn, kd.split, SPLIT_LIMITS["ws_elems"], SPLIT_LIMITS["max_split_tiles"])
        assert e.value.status == (wt.WT_ERR_NOT_FITTED if fits else wt.WT_ERR_INFEASIBLE)


def test_grouped_geometry_and_selection(ctx):
    """Grouped GEMM: exact Phi for known per-group rows (Table 2, grouped row) and the uniform-approximation
    selection on the dense table, both bit-exact against the oracle."""
    W, I, p = 12, 4, 5
    keys = _keys(ctx)
    wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_split=W_SPLIT), _synthetic_samples(keys, W, I, 31))
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        wt.wt_save(ctx, d + "/g.wt")
        table, _ = osel.read_table(d + "/g.wt", **SPLIT_LIMITS)
    differs = 0
    for (E, top_k, N, K) in wt_synth.MOE_LAYERS:
        for tokens in wt_synth.MOE_TOKENS:
            rows = wt_synth.moe_routing(tokens, E, top_k, seed=tokens + E)
            for i in range(0, wt.wt_config_count(ctx), 3 * 7):
                c, _ = wt.wt_config_get(ctx, i)
                if c.split != 1:
                    with pytest.raises(wt.WtError):
                        wt.wt_wave_count_grouped(ctx, rows, N, K, c)
                    continue
                G, L = geo.phi_grouped(rows.tolist(), N, K, c.bm, c.bn, c.bk)
                assert wt.wt_wave_count_grouped(ctx, rows, N, K, c) == (G, L, geo.wave_count(G, geo.capacity(1)))
            key, micro, t = osel.select_grouped(table, E, tokens * top_k, N, K)
            c = wt.wt_select_grouped(ctx, E, tokens * top_k, N, K)
            assert c.id == 3 * key + micro and c.split == 1
            routings = [wt_synth.moe_routing(tokens, E, top_k, seed=tokens + E, skew=skew) for skew in (1.0, 0.25)]
            routings.append(np.array([tokens * top_k] + [0] * (E - 1)))        # every row in one group
            for rows in routings:           # the real counts (Table 2's grouped row as it stands)
                key_r, micro_r, _ = osel.select_grouped_rows(table, rows.tolist(), N, K)
                c = wt.wt_select_grouped_rows(ctx, rows, N, K)
                assert c.id == 3 * key_r + micro_r and c.split == 1
                differs += (key_r, micro_r) != (key, micro)
    assert differs >= 3         # the real counts do change picks, so the comparison above tells the two calls apart
    # one group is the dense problem
    for (M, N, K) in wt_synth.sweep_shapes():
        key, micro, _ = osel.select_grouped(table, 1, M, N, K)
        assert wt.wt_select_grouped(ctx, 1, M, N, K).id == 3 * key + micro
        assert wt.wt_select_grouped_rows(ctx, [M], N, K).id == 3 * key + micro
    # argument checks of the real-counts call: no group, too many, a negative count, a sum beyond int32, G*L beyond int64
    for bad in ([], [1] * 1025, [5, -1], [2**30, 2**30, 2**30]):
        with pytest.raises(wt.WtError) as e:
            wt.wt_select_grouped_rows(ctx, bad, 128, 128)
        assert e.value.status == wt.WT_ERR_INVALID_ARG
    with pytest.raises(wt.WtError) as e:
        wt.wt_select_grouped_rows(ctx, [2**30], 2**20, 2**20)
    assert e.value.status == wt.WT_ERR_INVALID_ARG
    fresh = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_BF16)
    try:
        with pytest.raises(wt.WtError) as e:
            wt.wt_select_grouped_rows(fresh, [5, 5], 128, 128)
        assert e.value.status == wt.WT_ERR_NOT_FITTED
    finally:
        wt.wt_destroy(fresh)


def _pred_close(th_a, th_b, kd):
    pts = [(g, L) for g in (kd.cap // 2 + 1, kd.cap) for L in (8, 80)]
    for g, L in pts:
        a, b = osel.predict(th_a, g, L), osel.predict(th_b, g, L)
        if abs(a - b) > 1e-9 * max(abs(a), abs(b), 1.0):
            return False
    return True


def test_shapes_whose_task_loop_product_could_leave_int64_are_refused(ctx):
    """G*L is formed in int64 (the oracle uses unbounded integers): shapes with M*N*max(K,16) above 2^62 are an argument
    error in every call that evaluates Phi or a prediction, and the largest launchable shape is far below that."""
    wt.wt_fit(ctx, wt.make_grid(W=4, I=2, p=2, k_anchors=K_ANCHORS), _synthetic_samples(_keys(ctx), 4, 2))
    c, _ = wt.wt_config_get(ctx, 0)
    big = 2 ** 30
    for call in (lambda: wt.wt_select(ctx, big, big, 2 ** 21), lambda: wt.wt_predict_us(ctx, big, big, 2 ** 21, c),
                 lambda: wt.wt_wave_count(ctx, 2 ** 31, 2 ** 31, 8, c), lambda: wt.wt_select_grouped(ctx, 4, big, big, 2 ** 21),
                 lambda: wt.wt_wave_count_grouped(ctx, [big, big - 1], big, 2 ** 21, c)):
        with pytest.raises(wt.WtError) as e:
            call()
        assert e.value.status == wt.WT_ERR_INVALID_ARG
    G, L, w = wt.wt_wave_count(ctx, 2 ** 24, 2 ** 24, 2 ** 14, c)            # 2^62 exactly: accepted, exact
    assert (G, L) == geo.phi_gemm(2 ** 24, 2 ** 24, 2 ** 14, c.bm, c.bn, c.bk, c.split)
    assert wt.wt_select(ctx, 2 ** 24, 2 ** 24, 2 ** 14).id >= 0


def test_select_is_fast_and_allocates_nothing_visible(ctx):
    W, I = 8, 2
    samples = _synthetic_samples(_keys(ctx), W, I)
    wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=4, k_anchors=K_ANCHORS), samples)
    mean_ns, p99_ns = wt.wt_select_bench(ctx, wt_synth.stream_shapes(2000), repeats=3)
    assert mean_ns < 10_000        # target: <= 10 us per decision


def test_bad_table_file(ctx, tmp_path):
    p = tmp_path / "junk.wt"
    p.write_bytes(b"not a table")
    with pytest.raises(wt.WtError) as e:
        wt.wt_load(ctx, str(p))
    assert e.value.status == wt.WT_ERR_IO
    with pytest.raises(wt.WtError):
        wt.wt_load(ctx, str(tmp_path / "missing.wt"))


def test_fit_objective_argument_checks_and_header_word(ctx, tmp_path):
    """wt_grid.weighting takes WT_FIT_ABSOLUTE or WT_FIT_RELATIVE only; relative residuals need positive latencies;
    the objective is recorded in header word 15, and a file whose word 15 is zero (every file written before the
    field existed) loads as an absolutely fitted table."""
    import struct

    keys = _keys(ctx)
    samples = _synthetic_samples(keys, 4, 2)
    with pytest.raises(wt.WtError) as e:
        wt.wt_fit(ctx, wt.make_grid(W=4, I=2, p=2, k_anchors=K_ANCHORS, weighting=2), samples)
    assert e.value.status == wt.WT_ERR_INVALID_ARG
    bad = samples.copy()
    bad["mean_us"][5] = 0.0
    with pytest.raises(wt.WtError) as e:
        wt.wt_fit(ctx, wt.make_grid(W=4, I=2, p=2, k_anchors=K_ANCHORS, weighting=wt.WT_FIT_RELATIVE), bad)
    assert e.value.status == wt.WT_ERR_INVALID_ARG
    wt.wt_fit(ctx, wt.make_grid(W=4, I=2, p=2, k_anchors=K_ANCHORS, weighting=wt.WT_FIT_ABSOLUTE), bad)   # fine absolutely
    wt.wt_fit(ctx, wt.make_grid(W=4, I=2, p=2, k_anchors=K_ANCHORS, weighting=wt.WT_FIT_RELATIVE), samples)
    path = str(tmp_path / "rel.wt")
    wt.wt_save(ctx, path)
    raw = bytearray(open(path, "rb").read())
    assert struct.unpack_from("<I", raw, 60)[0] == 1
    pick = wt.wt_select(ctx, 4096, 4096, 4096).id
    struct.pack_into("<I", raw, 60, 0)
    old = str(tmp_path / "old.wt")
    open(old, "wb").write(bytes(raw))
    wt.wt_load(ctx, old)
    assert osel.read_table(old, **SPLIT_LIMITS)[1]["weighting"] == 0 and wt.wt_select(ctx, 4096, 4096, 4096).id == pick
    struct.pack_into("<I", raw, 60, 7)
    open(old, "wb").write(bytes(raw))
    with pytest.raises(wt.WtError):
        wt.wt_load(ctx, old)


def test_family_table_file_header_is_checked(ctx, tmp_path):
    """A version-4 file (row-band families) whose header is tampered with is refused, never half-loaded: a version the
    library does not know, a family count beyond the mode's, version 4 with no family, a truncated or padded file;
    and a file written with tile-row families read as row-band ones (version word changed) selects differently or
    is refused, but the context keeps working on its previous table either way."""
    import struct

    keys = _keys(ctx)
    W, W_row, I, p = 4, 2, 2, 2
    near = _synthetic_samples(keys, W, I, noise_seed=3)
    rows = []
    for k, kd in enumerate(keys):
        Wk = W_row if kd.split == 1 else min(W_row, W_SPLIT)
        for sm in smp.band_sample_set(kd.cap, Wk, I, 16, kd.bm, kd.split):
            if sm.g == 0 or not geo.split_fits(sm.m * kd.bm, sm.n * kd.bn, kd.bm, kd.bn, kd.split, SPLIT_LIMITS["ws_elems"], SPLIT_LIMITS["max_split_tiles"]):
                continue
            for L in smp.loop_anchors(K_ANCHORS, kd.bk, kd.split):
                for micro in range(3):
                    rows.append((k, micro, sm.g, L, sm.w, 1, 3.0 + 0.01 * sm.g + 0.2 * L + 0.1 * micro))
    samples = np.concatenate([near, np.array(rows, dtype=wt.SAMPLE_DTYPE)])
    wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_row=W_row, row_fams=1, W_split=W_SPLIT, row_mode=1), samples)
    good = str(tmp_path / "good.wt")
    wt.wt_save(ctx, good)
    raw = open(good, "rb").read()
    assert struct.unpack_from("<I", raw, 4)[0] == 4 and struct.unpack_from("<2I", raw, 52) == (W_row, 1)
    ref = [wt.wt_select(ctx, M, N, K).id for (M, N, K) in wt_synth.sweep_shapes()]

    def tampered(offset, value, tail=None):
        b = bytearray(raw)
        struct.pack_into("<I", b, offset, value)
        q = str(tmp_path / f"t{offset}_{value}.wt")
        open(q, "wb").write(bytes(b) if tail is None else tail(bytes(b)))
        return q

    for q in (tampered(4, 5), tampered(4, 0), tampered(56, 5), tampered(56, 0), tampered(52, 1 << 20),
              tampered(4, 4, tail=lambda b: b[:-8]), tampered(4, 4, tail=lambda b: b + b"\0" * 8)):
        with pytest.raises(wt.WtError):
            wt.wt_load(ctx, q)
        assert [wt.wt_select(ctx, M, N, K).id for (M, N, K) in wt_synth.sweep_shapes()] == ref      # table untouched
    # version 2 = the same bytes read as ONE tile-row family: loads, and consults the family by tile rows instead of by M
    v2 = tampered(4, 2)
    c2 = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
    try:
        wt.wt_load(c2, v2)
        t2, _ = osel.read_table(v2, **SPLIT_LIMITS)
        assert t2.row_mode == 0 and t2.row_fams == 1
        for (M, N, K) in wt_synth.sweep_shapes():
            key, micro, _ = osel.select(t2, M, N, K)
            assert wt.wt_select(c2, M, N, K).id == 3 * key + micro
    finally:
        wt.wt_destroy(c2)


@pytest.mark.parametrize("model", [wt.WT_MODEL_LINEAR, wt.WT_MODEL_STEP])
def test_ablation_models_parity(ctx, tmp_path, model):
    """Step and Linear tables built by the library equal the oracle's (coefficients to 1e-9, anchors
    and lookups exactly)."""
    W, I, p = 10, 4, 4
    keys = _keys(ctx)
    samples = _synthetic_samples(keys, W, I, noise_seed=9)
    wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, model=model), samples)
    path = str(tmp_path / "abl.wt")
    wt.wt_save(ctx, path)
    table, _ = osel.read_table(path, **SPLIT_LIMITS)
    want = ofit.fit_tables([tuple(r)[:5] + (float(r["mean_us"]),) for r in samples], keys, W, p, model=model, max_anchors=MAX_ANCHORS)
    for k in range(len(keys)):
        for got_b, want_b in list(zip(table.local[k], want.local[k])) + [(table.ext[k], want.ext[k])]:
            assert got_b.status == want_b.status
            if want_b.status:
                assert got_b.anchors == want_b.anchors
                scale = max(abs(x) for x in want_b.theta) or 1.0
                assert np.allclose(got_b.theta, want_b.theta, rtol=1e-9, atol=1e-12 * scale) or \
                    _pred_close(got_b.theta, want_b.theta, keys[k])
    for (M, N, K) in wt_synth.sweep_shapes() + wt_synth.stream_shapes(500):
        key, micro, t = osel.select(table, M, N, K)
        c = wt.wt_select(ctx, M, N, K)
        kd = keys[key]
        assert (c.bm, c.bn, c.bk, c.nwave, c.stages, c.swizzle, c.split) == (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, micro, kd.split)
    with pytest.raises(wt.WtError):
        wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, model=7), samples)


def test_occupancy_aware_capacity_mode(tmp_path):
    """Capacity = 256 x resident blocks per CU: wave counts, table and lookups follow those wider waves;
    the file records the mode and wt_load restores it."""
    c = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
    try:
        wt.wt_set_capacity_mode(c, wt.WT_CAP_CU_TIMES_OCC)
        keys = _keys(c, occ_aware=True)
        cfg, res = wt.wt_config_get(c, 3 * 31)          # a key with several resident blocks per CU
        assert res.occ > 1
        G, L, w = wt.wt_wave_count(c, 4096, 4096, 4096, cfg)
        assert w == geo.wave_count(G, 256 * res.occ) < geo.wave_count(G, 256)
        W, I = 8, 4
        samples = _synthetic_samples(keys, W, I, noise_seed=3)
        wt.wt_fit(c, wt.make_grid(W=W, I=I, p=3, k_anchors=K_ANCHORS), samples)
        path = str(tmp_path / "occ.wt")
        wt.wt_save(c, path)
        table, meta = osel.read_table(path, **SPLIT_LIMITS)
        assert meta["key_mode"] == 0 and table.keys == keys
        c2 = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
        assert wt.wt_wave_count(c2, 4096, 4096, 4096, cfg)[2] == geo.wave_count(G, 256)
        wt.wt_load(c2, path)
        assert wt.wt_wave_count(c2, 4096, 4096, 4096, cfg)[2] == w
        for (M, N, K) in wt_synth.sweep_shapes() + wt_synth.stream_shapes(500):
            key, micro, t = osel.select(table, M, N, K)
            for cc in (c, c2):
                s = wt.wt_select(cc, M, N, K)
                assert s.id == 3 * key + micro and wt.wt_predict_us(cc, M, N, K, s) == t
        wt.wt_destroy(c2)
        wt.wt_set_capacity_mode(c, wt.WT_CAP_CU_ONLY)       # switching discards the table
        with pytest.raises(wt.WtError):
            wt.wt_select(c, 64, 64, 64)
    finally:
        wt.wt_destroy(c)


@pytest.mark.parametrize("row_fams,row_mode", [(1, 0), (3, 0), (1, 1), (4, 1)])
def test_few_row_families_parity(ctx, tmp_path, row_fams, row_mode):
    """Extension: records of 1-, 2- and 4-tile-row grids (row_mode 0, families 1..3) or of 16-, 32-, 64- and 128-row
    matrices (row_mode 1, families 1..4) build further bucket sets; table, file (version 2 with one tile-row family,
    3 with several, 4 with row-band families) and lookups match the oracle exactly."""
    W, W_row, I, p = 8, 3, 4, 4
    keys = _keys(ctx)
    near = _synthetic_samples(keys, W, I, noise_seed=11)
    rows = []
    for f in range(1, row_fams + 1):
        for k, kd in enumerate(keys):
            th = wt_synth.random_theta(900 + 7 * f + k, W_row)
            Wk = W_row if kd.split == 1 else min(W_row, W_SPLIT)
            fam_set = (smp.band_sample_set(kd.cap, Wk, I, smp.ROW_BANDS[f - 1], kd.bm, kd.split) if row_mode else
                       smp.row_sample_set(kd.cap, Wk, I, 1 << (f - 1), kd.split))
            for s in fam_set:
                if s.g == 0 or not geo.split_fits(s.m * kd.bm, s.n * kd.bn, kd.bm, kd.bn, kd.split, SPLIT_LIMITS["ws_elems"], SPLIT_LIMITS["max_split_tiles"]):
                    continue
                for L in smp.loop_anchors(K_ANCHORS, kd.bk, kd.split):
                    for micro in range(3):
                        a, b, c, d = th[s.w - 1]
                        t = (4.0 / (f + 1)) * (kd.bn * kd.bk / 8192.0) * (a * s.g * L + b * s.g) + c * L + d
                        rows.append((k, micro, s.g, L, s.w, f, t * (1.0 + 0.02 * ((micro + k) % 3))))
    samples = np.concatenate([near, np.array(rows, dtype=wt.SAMPLE_DTYPE)])
    grid = wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_row=W_row, row_fams=row_fams, W_split=W_SPLIT, row_mode=row_mode)
    wt.wt_fit(ctx, grid, samples)
    path = str(tmp_path / "row.wt")
    wt.wt_save(ctx, path)
    table, meta = osel.read_table(path, **SPLIT_LIMITS)
    assert meta["W_row"] == W_row and table.W_row == W_row and table.row_fams == row_fams and table.row_mode == row_mode
    assert open(path, "rb").read()[4] == (4 if row_mode else 3 if row_fams > 1 else 2)          # the version word
    want = ofit.fit_tables([(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"]),
                             float(r["mean_us"]), int(r["family"])) for r in samples], keys, W, p, W_row=W_row,
                           row_fams=row_fams, max_anchors=MAX_ANCHORS, row_mode=row_mode)
    for k in range(len(keys)):
        pairs = list(zip(table.local[k], want.local[k])) + [(table.ext[k], want.ext[k])]
        for f in range(row_fams):
            pairs += list(zip(table.row_local[f][k], want.row_local[f][k])) + [(table.row_ext[f][k], want.row_ext[f][k])]
        for got_b, want_b in pairs:
            assert got_b.status == want_b.status and got_b.anchors == want_b.anchors
            scale = max(abs(x) for x in want_b.theta) or 1.0
            assert np.allclose(got_b.theta, want_b.theta, rtol=1e-9, atol=1e-9 * scale) or \
                _pred_close(got_b.theta, want_b.theta, keys[k])
    ctx2 = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_F32)
    wt.wt_load(ctx2, path)
    used = [0, 0, 0, 0, 0]
    for (M, N, K) in wt_synth.sweep_shapes() + wt_synth.stream_shapes(2000):
        key, micro, t = osel.select(table, M, N, K)
        used[osel.family_of(table, M, keys[key].bm)] += 1
        for cc in (ctx, ctx2):
            c = wt.wt_select(cc, M, N, K)
            assert c.id == 3 * key + micro and wt.wt_predict_us(cc, M, N, K, c) == t
    assert all(u > 30 for u in used[:row_fams + 1])
    wt.wt_destroy(ctx2)
    n_near, *_ = wt.wt_sample_plan(ctx, wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_split=W_SPLIT))
    n_both, *_ = wt.wt_sample_plan(ctx, grid)
    assert n_both - n_near == len(rows)          # the plan adds exactly the few-row workloads
    if row_mode:
        # a band's workloads have exactly the band's rows (the last tile row partial), not full tile rows: with the
        # near-square grids left out, the A operand of the 16-row family never exceeds 16 rows of the longest K
        only = wt.make_grid(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_row=W_row, row_fams=1, W_split=W_SPLIT, row_mode=1, skip_near=1)
        _, bytesA, _, _ = wt.wt_sample_plan(ctx, only)
        k_max = max(geo.ceil_div(max(K_ANCHORS), kd.bk * kd.split) * kd.bk * kd.split for kd in keys)
        assert bytesA == 16 * k_max * 2
    for bad in (dict(row_mode=2), dict(row_mode=0, row_fams=4), dict(row_mode=1, row_fams=5)):
        kw = dict(W=W, I=I, p=p, k_anchors=K_ANCHORS, W_row=W_row, row_fams=1, W_split=W_SPLIT)
        kw.update(bad)
        with pytest.raises(wt.WtError) as e:
            wt.wt_fit(ctx, wt.make_grid(**kw), samples)
        assert e.value.status == wt.WT_ERR_INVALID_ARG
        with pytest.raises(wt.WtError):
            wt.wt_sample_plan(ctx, wt.make_grid(**kw))


@pytest.mark.parametrize("tiles", [(1, 1), (1, 61), (3, 80), (5, 29), (7, 8), (16, 43), (38, 12), (64, 32), (9, 9)])
def test_rasterisation_is_a_bijection(tiles):
    """The kernel's block -> tile mapping, evaluated on the host: every mode visits every tile exactly once.  On a grid
    at least as wide as tall, mode 0 is column-major and modes 1/2 hand each XCD (block index mod 8) a contiguous range
    of the banded order (bands of 4 / 8 tile rows, column by column); grids of at most 8 rows are one band whatever the
    mode; a taller grid is walked like the transposed one with rows and columns exchanged."""
    tm_n, tn_n = tiles
    total = tm_n * tn_n
    for sw in (0, 1, 2):
        seen = [wt.wt_tile_coords(tm_n, tn_n, sw, b) for b in range(total)]
        assert sorted(seen) == [(i, j) for i in range(tm_n) for j in range(tn_n)]
    modes = [[wt.wt_tile_coords(tm_n, tn_n, sw, b) for b in range(total)] for sw in (0, 1, 2)]
    mirrored = tm_n > tn_n
    short, long_ = min(tm_n, tn_n), max(tm_n, tn_n)
    back = (lambda rc: (rc[1], rc[0])) if mirrored else (lambda rc: rc)      # (short index, long index) -> (tm, tn)
    if short > 8:    # mode 0 runs down the short side first and the three modes differ
        assert modes[0] == [back((b % short, b // short)) for b in range(total)]
        assert modes[0] != modes[1] != modes[2]
    else:            # at most 8 rows (columns, mirrored): one band under every mode
        assert modes[0] == modes[1] == modes[2]
    per, rem = divmod(total, 8)
    for sw, band in ((1, 4 if short > 8 else 8), (2, 8)):
        order = []                               # banded order on the wide orientation
        for g0 in range(0, short, band):
            gm = min(band, short - g0)
            order += [back((g0 + i, j)) for j in range(long_) for i in range(gm)]
        for x in range(8):
            mine = [wt.wt_tile_coords(tm_n, tn_n, sw, b) for b in range(x, total, 8)]
            start = x * per + min(x, rem)
            assert mine == order[start:start + len(mine)]
    with pytest.raises(wt.WtError):
        wt.wt_tile_coords(tm_n, tn_n, 3, 0)
    with pytest.raises(wt.WtError):
        wt.wt_tile_coords(tm_n, tn_n, 0, total)
