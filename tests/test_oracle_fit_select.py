"""Pins for oracle/fit.py, oracle/select.py and oracle/exhaustive.py: closed forms, exact
rational least squares, known generating surfaces, and brute force over the generating
function."""
from fractions import Fraction

import numpy as np
import pytest

import wt_synth
from _pins import load_pins
from oracle import exhaustive as oex
from oracle import fit as ofit
from oracle import geometry as geo
from oracle import sampler as smp
from oracle import select as osel

P = load_pins()


def _exact_ls(rows, cols):
    """Exact rational least squares through the normal equations (Gauss-Jordan on Fractions)."""
    X = [[Fraction(f(r)) for f in cols] for r in rows]
    y = [Fraction(r[2]) for r in rows]
    n = len(cols)
    A = [[sum(X[k][i] * X[k][j] for k in range(len(X))) for j in range(n)]
         + [sum(X[k][i] * y[k] for k in range(len(X)))] for i in range(n)]
    for c in range(n):
        piv = next(r for r in range(c, n) if A[r][c] != 0)
        A[c], A[piv] = A[piv], A[c]
        A[c] = [v / A[c][c] for v in A[c]]
        for r in range(n):
            if r != c:
                A[r] = [vr - A[r][c] * vc for vr, vc in zip(A[r], A[c])]
    return [float(A[i][n]) for i in range(n)]


FULL = (lambda r: r[0] * r[1], lambda r: r[0], lambda r: r[1], lambda r: 1)


def test_two_by_two_closed_form():
    # four points on a 2x2 grid are interpolated exactly:
    # alpha = (T11 - T12 - T21 + T22) / ((G1-G2)(L1-L2))
    G1, G2, L1, L2 = 300, 500, 16, 80
    T = {(G1, L1): 10.0, (G1, L2): 31.0, (G2, L1): 14.5, (G2, L2): 52.0}
    rows = [(g, l, t) for (g, l), t in T.items()]
    (a, b, c, d), status = ofit.fit_bilinear(rows)
    assert status == 0b1111
    alpha = (T[G1, L1] - T[G1, L2] - T[G2, L1] + T[G2, L2]) / ((G1 - G2) * (L1 - L2))
    assert abs(a - alpha) < 1e-15
    for g, l, t in rows:
        assert abs(a * g * l + b * g + c * l + d - t) < 1e-11


def test_fit_matches_exact_rational_least_squares():
    rng = np.random.default_rng(4)
    Gs, Ls = [9985, 10050, 10111, 10240], [16, 32, 48, 64, 80]
    rows = [(g, l, int(rng.integers(100, 100000))) for g in Gs for l in Ls]   # integer "latencies"
    theta, _ = ofit.fit_bilinear(rows)
    want = _exact_ls(rows, FULL)
    # compare through predictions and through coefficients (well-conditioned after centring)
    assert np.allclose(theta, want, rtol=1e-8, atol=0)


def test_recovers_known_surface_far_from_origin():
    th = (3.1e-4, 2.0e-2, 0.7, 5.0)
    rows = [(g, l, th[0] * g * l + th[1] * g + th[2] * l + th[3])
            for g in (20225, 20300, 20449, 20480) for l in (8, 16, 24, 32, 40)]
    got, _ = ofit.fit_bilinear(rows)
    assert np.allclose(got, th, rtol=1e-9)


def test_one_dimensional_reductions():
    rows = [(g, 32, 2.5 * g + 7.0 + e) for g, e in zip((10, 20, 30, 40), (0.1, -0.2, 0.05, 0.05))]
    (a, b, c, d), status = ofit.fit_bilinear(rows)
    slope, icpt = np.polyfit([r[0] for r in rows], [r[2] for r in rows], 1)
    assert status == 0b1010 and a == 0 and c == 0
    assert abs(b - slope) < 1e-12 and abs(d - icpt) < 1e-10
    rows = [(77, l, 0.5 * l + 1.0) for l in (16, 32, 64)]
    (a, b, c, d), status = ofit.fit_bilinear(rows)
    assert status == 0b1100 and a == 0 and b == 0 and abs(c - 0.5) < 1e-13 and abs(d - 1.0) < 1e-12
    (a, b, c, d), status = ofit.fit_bilinear([(5, 6, 2.0), (5, 6, 4.0)])
    assert status == 0b1000 and (a, b, c) == (0, 0, 0) and d == 3.0
    assert ofit.fit_bilinear([]) == ((0.0, 0.0, 0.0, 0.0), 0)


def test_shared_micro_minimises_the_average_not_each_point():
    # micro 0 wins at three grid sizes by a hair, micro 1 wins the average by a lot
    S = ofit.Sample
    recs = [S(0, 0, 10, 4, 1, 1.0), S(0, 0, 20, 4, 1, 1.0), S(0, 0, 30, 4, 1, 1.0), S(0, 0, 40, 4, 1, 9.0),
            S(0, 1, 10, 4, 1, 1.1), S(0, 1, 20, 4, 1, 1.1), S(0, 1, 30, 4, 1, 1.1), S(0, 1, 40, 4, 1, 2.0)]
    micro, rows = ofit.shared_micro(recs)
    assert micro == 1 and sorted(rows) == [(10, 4, 1.1), (20, 4, 1.1), (30, 4, 1.1), (40, 4, 2.0)]
    # ties go to the lowest id; a micro missing a grid size is ineligible
    tie = [S(0, 2, 10, 4, 1, 1.0), S(0, 1, 10, 4, 1, 1.0)]
    assert ofit.shared_micro(tie)[0] == 1
    part = [S(0, 0, 10, 4, 1, 0.1), S(0, 1, 10, 4, 1, 1.0), S(0, 1, 20, 4, 1, 1.0)]
    assert ofit.shared_micro(part)[0] == 1
    assert ofit.shared_micro([S(0, 0, 10, 4, 1, 1.0), S(0, 1, 20, 4, 1, 1.0)]) is None


# ---- a synthetic tuning problem with a known answer -------------------------------------------
KEYS = [ofit.KeyDesc(256, 256, 64, 4, 2, 1, 256), ofit.KeyDesc(128, 128, 64, 4, 2, 2, 512),
        ofit.KeyDesc(64, 64, 64, 4, 2, 5, 1280), ofit.KeyDesc(128, 64, 32, 4, 3, 3, 768),
        ofit.KeyDesc(16, 64, 128, 1, 2, 8, 2048)]
K_ANCHORS = (1024, 2048, 3072, 4096, 5120)
N_MICRO = 3


def _surface_theta(key, w, W, seed=21):
    """Per-<key, w> generating coefficients; waves beyond W continue the last bucket's."""
    th = wt_synth.random_theta(seed + 97 * key, W + 1)
    return th[min(w, W) - 1]


def _latency(key, micro, G, L, W, micro_penalty):
    kd = KEYS[key]
    w = geo.wave_count(G, kd.cap)
    a, b, c, d = _surface_theta(key, w, W)
    base = a * G * L + b * G + c * L + d
    return base * (1.0 + micro_penalty(key, micro, L))


def _make_samples(W, I, micro_penalty):
    out = []
    for k, kd in enumerate(KEYS):
        for s in smp.sample_set(kd.cap, W, I):
            for L in smp.loop_anchors(K_ANCHORS, kd.bk):
                for mi in range(N_MICRO):
                    out.append(ofit.Sample(k, mi, s.g, L, s.w, _latency(k, mi, s.g, L, W, micro_penalty)))
    return out


def _penalty(key, micro, L):
    # best micro depends on the loop count: micro 0 below L=40, micro 2 from 40 up; micro 1 never
    best = 0 if L < 40 else 2
    return 0.0 if micro == best else 0.05 * (1 + micro)


def test_fit_recovers_every_bucket_and_the_step_surface():
    W, I = 6, 4
    table = ofit.fit_tables(_make_samples(W, I, _penalty), KEYS, W, p=3)
    for k in range(len(KEYS)):
        for w in range(1, W + 1):
            b = table.local[k][w - 1]
            assert b.status == 0b1111
            assert np.allclose(b.theta, _surface_theta(k, w, W), rtol=1e-7)
            La = smp.loop_anchors(K_ANCHORS, KEYS[k].bk)
            assert [a[0] for a in b.anchors] == La
            assert [a[1] for a in b.anchors] == [0 if L < 40 else 2 for L in La]
    # pure step surface T = mu * ceil(G/cap) * L (zero-variance simulation scaled by L): inside
    # bucket w the fit must find gamma = mu*w and nothing else -> buckets are isolated and w is
    # computed with the right capacity
    mu = float(P["fig4_mu"])
    samples = [ofit.Sample(k, 0, s.g, L, s.w, mu * geo.wave_count(s.g, kd.cap) * L)
               for k, kd in enumerate(KEYS) for s in smp.sample_set(kd.cap, W, I)
               for L in smp.loop_anchors(K_ANCHORS, kd.bk)]
    step = ofit.fit_tables(samples, KEYS, W, p=1)
    for k in range(len(KEYS)):
        for w in range(1, W + 1):
            a, b, c, d = step.local[k][w - 1].theta
            assert abs(c - mu * w) < 1e-6 * mu and abs(a) < 1e-9 and abs(b) < 1e-7 and abs(d) < 1e-3
        assert abs(step.ext[k].theta[2] - mu * W) < 1e-6 * mu      # p=1: ext is the last wave


def test_ext_merges_exactly_the_last_p_waves():
    W, I, p = 8, 4, 3
    samples = _make_samples(W, I, _penalty)
    table = ofit.fit_tables(samples, KEYS, W, p)
    for k in range(len(KEYS)):
        merged = [s for s in samples if s.key == k and W - p + 1 <= s.w <= W]
        rows = []
        for L in sorted({s.L for s in merged}):
            micro, r = ofit.shared_micro([s for s in merged if s.L == L])
            rows += r
        assert len(rows) == p * I * len(smp.loop_anchors(K_ANCHORS, KEYS[k].bk))
        want, _ = ofit.fit_bilinear(rows)
        assert np.allclose(table.ext[k].theta, want, rtol=1e-12)
    # W < p: the merge starts at wave 1
    t2 = ofit.fit_tables(_make_samples(2, 2, _penalty), KEYS, 2, p=10)
    assert all(b.status == 0b1111 for b in t2.ext)


def test_select_equals_brute_force_over_the_generating_function():
    W, I = 6, 4
    table = ofit.fit_tables(_make_samples(W, I, _penalty), KEYS, W, p=3)
    shapes = [(m, n, k) for m in (1, 17, 100, 256, 333, 1024, 2000) for (n, k) in ((4096, 4096), (1536, 2048), (2304, 5120))]
    n_in_range = 0
    for (M, N, K) in shapes:
        cand = []
        for kid, kd in enumerate(KEYS):
            G, L = geo.phi_gemm(M, N, K, kd.bm, kd.bn, kd.bk)
            if geo.wave_count(G, kd.cap) > W:
                cand = None
                break
            for mi in range(N_MICRO):
                cand.append(((kid, mi), _latency(kid, mi, G, L, W, _penalty)))
        if cand is None:
            continue
        n_in_range += 1
        (bk, bm), bt = oex.argmin_config(cand)
        key, micro, t = osel.select(table, M, N, K)
        assert key == bk and abs(t - bt) <= 1e-7 * bt
        # the micro comes from the nearest anchor; at the anchors' own L it is the generating best
        L = geo.phi_gemm(M, N, K, *KEYS[key][:3])[1]
        if L in smp.loop_anchors(K_ANCHORS, KEYS[key].bk):
            assert micro == bm
    assert n_in_range >= 10


def test_extrapolation_rule_switches_on_w_greater_than_W():
    W = 3
    table = ofit.fit_tables(_make_samples(W, 4, _penalty), KEYS, W, p=2)
    for b in table.ext:                       # make the ext entries unmistakable
        b.theta = (0.0, 0.0, 0.0, 1.0e9)
    table.ext[2].theta = (0.0, 0.0, 0.0, 123.0)
    table.ext[2].anchors = [(16, 1), (80, 2)]
    # 16384 x 16384: every key needs far more than 3 waves -> all use ext, key 2 wins
    key, micro, t = osel.select(table, 16384, 16384, 4096)
    assert (key, t) == (2, 123.0) and micro == 2          # L = 64 is nearer to 80 than to 16
    # a small shape stays inside the profiled range and must not see the ext entries
    key, _, t = osel.select(table, 256, 256, 1024)
    assert t < 1.0e6
    # an unfitted local bucket falls back to ext
    table.local[0][0].status = 0
    assert osel.bucket_for(table, 0, 1) is table.ext[0]
    assert osel.bucket_for(table, 0, 2) is table.local[0][1]
    assert osel.bucket_for(table, 0, W + 1) is table.ext[0]


def test_nearest_anchor_cases():
    anchors = [(16, 5), (32, 6), (48, 7)]
    assert osel.nearest_anchor(anchors, 1) == (16, 5)        # below the first
    assert osel.nearest_anchor(anchors, 500) == (48, 7)      # above the last
    assert osel.nearest_anchor(anchors, 24) == (16, 5)       # exactly mid-way -> smaller anchor
    assert osel.nearest_anchor(anchors, 25) == (32, 6)
    assert osel.nearest_anchor(anchors, 32) == (32, 6)


def test_stage_one_ties_keep_the_lowest_key():
    keys = [ofit.KeyDesc(64, 64, 64, 4, 2, 1, 256)] * 3
    mk = lambda th: ofit.Bucket(theta=th, status=15, anchors=[(8, 1)])
    table = ofit.DualTable(W=1, keys=keys, local=[[mk((0, 0, 0, 2.0))], [mk((0, 0, 0, 1.0))], [mk((0, 0, 0, 1.0))]],
                           ext=[mk((0, 0, 0, 9.0))] * 3)
    assert osel.select(table, 64, 64, 64)[:2] == (1, 1)


def test_predict_is_the_bilinear_form():
    assert osel.predict((2.0, 3.0, 5.0, 7.0), 11, 13) == 2 * 143 + 33 + 65 + 7
    assert osel.predict((0.5, 0.0, 0.0, 0.0), 3, 5) == 7.5


def test_exhaustive_helpers():
    assert oex.argmin_config([(0, 3.0), (1, float("nan")), (2, 1.0), (3, 1.0)]) == (2, 1.0)
    with pytest.raises(ValueError):
        oex.argmin_config([(0, float("inf"))])
    res = oex.search([1, 2], [10, 20, 30], lambda s, c: abs(c - 15 * s))
    assert res == [(10, 5), (30, 0)]
    assert oex.fraction_of_best(2.0, 1.0) == 0.5
    assert abs(oex.geomean([0.5, 2.0]) - 1.0) < 1e-15


# ---- ablation models (Sec. 5.4): Step and Linear ---------------------------------------------------
def test_step_model_recovers_a_pure_step_surface():
    # T = w * (a*L + b) exactly -> the Step fit returns a and b, bucket w holds (0,0,a*w,b*w), and a
    # query beyond W is priced by the linear envelope a/cap, b/cap
    a, b, W = 0.37, 4.5, 5
    samples = [ofit.Sample(k, mi, s.g, L, s.w, geo.wave_count(s.g, kd.cap) * (a * L + b) * (1.0 + 0.1 * mi))
               for k, kd in enumerate(KEYS) for s in smp.sample_set(kd.cap, W, 4)
               for L in smp.loop_anchors(K_ANCHORS, kd.bk) for mi in range(2)]
    t = ofit.fit_tables(samples, KEYS, W, p=2, model=ofit.MODEL_STEP)
    for k, kd in enumerate(KEYS):
        for w in range(1, W + 1):
            th = t.local[k][w - 1].theta
            assert th[0] == 0 and th[1] == 0 and abs(th[2] - a * w) < 1e-9 and abs(th[3] - b * w) < 1e-8
            assert all(m == 0 for _, m in t.local[k][w - 1].anchors)       # micro 0 is 10 % faster
        assert np.allclose(t.ext[k].theta, (a / kd.cap, b / kd.cap, 0, 0), rtol=1e-9)
        # inside a wave the Step model is flat in G
        G1, G2 = kd.cap + 1, 2 * kd.cap
        assert osel.predict(t.local[k][1].theta, G1, 32) == osel.predict(t.local[k][1].theta, G2, 32)


def test_linear_model_is_one_global_bilinear_per_key():
    W = 6
    samples = _make_samples(W, 4, _penalty)
    t = ofit.fit_tables(samples, KEYS, W, p=2, model=ofit.MODEL_LINEAR)
    full = ofit.fit_tables(samples, KEYS, W, p=W)           # ext over all waves = the global fit
    for k in range(len(KEYS)):
        assert all(b.status == 0 for b in t.local[k])
        assert t.ext[k].theta == full.ext[k].theta and t.ext[k].anchors == full.ext[k].anchors
        assert osel.bucket_for(t, k, 1) is t.ext[k] and osel.bucket_for(t, k, W + 3) is t.ext[k]
    # on data that really has per-wave structure the global fit is worse than the bucketed one
    err_lin = err_full = 0.0
    for s in samples:
        if s.micro == 0 and s.key == 1:
            truth = _latency(s.key, s.micro, s.G, s.L, W, lambda *a: 0.0)
            err_lin += abs(osel.predict(t.ext[1].theta, s.G, s.L) - truth) / truth
            err_full += abs(osel.predict(full.local[1][s.w - 1].theta, s.G, s.L) - truth) / truth
    assert err_full < 1e-6 < err_lin


# ---- single-tile-row family (extension beyond the paper's near-square sampler) ----------------------
def _row_samples(W_row, I, slow=3.0):
    """1 x g grids whose latency surface is `slow` times the near-square one (B streamed from HBM)."""
    out = []
    for k, kd in enumerate(KEYS):
        for s in smp.row_sample_set(kd.cap, W_row, I):
            for L in smp.loop_anchors(K_ANCHORS, kd.bk):
                for mi in range(N_MICRO):
                    out.append(ofit.Sample(k, mi, s.g, L, s.w, slow * _latency(k, mi, s.g, L, 6, _penalty), 1))
    return out


def test_single_row_family_is_fitted_and_used_only_for_one_tile_row():
    W, W_row, I = 6, 2, 4
    near = _make_samples(W, I, _penalty)
    table = ofit.fit_tables(near + _row_samples(W_row, I), KEYS, W, p=3, W_row=W_row)
    plain = ofit.fit_tables(near, KEYS, W, p=3)
    assert table.W_row == W_row and plain.W_row == 0
    for k in range(len(KEYS)):
        # the paper's buckets are untouched by the extra family
        assert [b.theta for b in table.local[k]] == [b.theta for b in plain.local[k]]
        assert table.ext[k].theta == plain.ext[k].theta
        for w in range(1, W_row + 1):
            assert np.allclose(table.row_local[0][k][w - 1].theta, 3.0 * _surface_theta(k, w, 6), rtol=1e-7)
    kd = KEYS[1]                                   # 128 x 128 x 64
    # M <= BM: one tile row -> row family; M = BM + 1: two tile rows -> the paper's buckets
    assert osel.bucket_for(table, 1, 1, 1) is table.row_local[0][1][0]
    assert osel.bucket_for(table, 1, W_row + 1, 1) is table.row_ext[0][1]
    assert osel.bucket_for(table, 1, 1, 2) is table.local[1][0]          # no 2-row family in this table
    assert osel.bucket_for(table, 1, 1, 0) is table.local[1][0]
    assert osel.bucket_for(plain, 1, 1, 1) is plain.local[1][0]
    t1 = osel.predict(osel.bucket_for(table, 1, 1, 1).theta, 32, 64)
    t0 = osel.predict(osel.bucket_for(table, 1, 1, 0).theta, 32, 64)
    assert abs(t1 - 3.0 * t0) < 1e-6 * t1
    # a skinny shape: every key with BM >= M is priced 3x higher than in the plain table, so the pick
    # moves to what the generating function says is best under the slow surface
    M, N, K = 16, 4096, 4096
    cand = []
    for kid, kd in enumerate(KEYS):
        G, L = geo.phi_gemm(M, N, K, kd.bm, kd.bn, kd.bk)
        for mi in range(N_MICRO):
            cand.append(((kid, mi), (3.0 if M <= kd.bm else 1.0) * _latency(kid, mi, G, L, W, _penalty)))
    (bk, _), bt = oex.argmin_config(cand)
    key, _, t = osel.select(table, M, N, K)
    assert key == bk and abs(t - bt) < 1e-6 * bt
    # a key without row records falls back to its near-square buckets
    t2 = ofit.fit_tables(near + [s for s in _row_samples(W_row, I) if s.key != 0], KEYS, W, p=3, W_row=W_row)
    assert osel.bucket_for(t2, 0, 1, 1) is t2.local[0][0]


def test_few_row_families_are_chosen_by_tile_rows():
    """Three families (1, 2, 4 tile rows), each with its own latency surface (x3, x2, x1.5 of the
    near-square one): a shape is priced by the family of its tile-row count under every key, and by the
    paper's buckets from 8 tile rows on."""
    W, W_row, I = 6, 2, 4
    near = _make_samples(W, I, _penalty)
    slow = {1: 3.0, 2: 2.0, 3: 1.5}
    extra = []
    for f, m in ((1, 1), (2, 2), (3, 4)):
        for k, kd in enumerate(KEYS):
            for s in smp.row_sample_set(kd.cap, W_row, I, m):
                if s.g == 0:
                    continue
                assert s.g == s.m * s.n and s.m == m
                for L in smp.loop_anchors(K_ANCHORS, kd.bk):
                    for mi in range(N_MICRO):
                        extra.append(ofit.Sample(k, mi, s.g, L, s.w, slow[f] * _latency(k, mi, s.g, L, 6, _penalty), f))
    table = ofit.fit_tables(near + extra, KEYS, W, p=3, W_row=W_row, row_fams=3)
    assert table.row_fams == 3
    assert [smp.row_family(r) for r in (0, 1, 2, 3, 4, 7, 8, 100)] == [1, 1, 2, 2, 3, 3, 0, 0]
    kd = KEYS[1]                                   # 128 x 128 x 64
    for M, f in ((100, 1), (128, 1), (129, 2), (384, 2), (385, 3), (896, 3), (897, 0)):
        fam = smp.row_family(geo.ceil_div(M, kd.bm))
        assert fam == f
        b = osel.bucket_for(table, 1, 1, fam)
        t0 = osel.predict(table.local[1][0].theta, 40, 64)
        assert abs(osel.predict(b.theta, 40, 64) - slow.get(f, 1.0) * t0) < 1e-6 * t0
    # Stage I uses, for every key, the family of that key's own tile-row count
    M, N, K = 200, 4096, 4096
    cand = []
    for kid, kd in enumerate(KEYS):
        G, L = geo.phi_gemm(M, N, K, kd.bm, kd.bn, kd.bk)
        f = smp.row_family(geo.ceil_div(M, kd.bm))
        for mi in range(N_MICRO):
            cand.append(((kid, mi), slow.get(f, 1.0) * _latency(kid, mi, G, L, W, _penalty)))
    (bk, _), bt = oex.argmin_config(cand)
    key, _, t = osel.select(table, M, N, K)
    assert key == bk and abs(t - bt) < 1e-6 * bt


def test_row_band_families_are_chosen_by_m_for_every_key_alike():
    """Row-band families (row_mode 1): family f holds matrices of 16, 32, 64, 128 rows under EVERY key, and a shape
    consults the family of the smallest band holding its M whatever the key's tile height.  Hand values of the band
    rule and of the sample sets; then Stage I on a table whose bands have surfaces x3, x2 of the near-square one:
    every key is priced from the same band, where the tile-row rule would mix families across tile heights."""
    assert [smp.band_family(M) for M in (0, 1, 16, 17, 32, 33, 64, 65, 128, 129, 5000)] == [1, 1, 1, 2, 2, 3, 3, 4, 4, 0, 0]
    # 64 rows under a 16-row tile: 4 tile rows; under a 256-row tile: one (partial) tile row.  cap 256, I = 4, wave 1,
    # sub-intervals end at 64, 128, 192, 256: widest n with 4n <= b is 16, 32, 48, 64
    s16 = smp.band_sample_set(256, 1, 4, 64, 16)
    assert [(x.g, x.m, x.n) for x in s16] == [(64, 4, 16), (128, 4, 32), (192, 4, 48), (256, 4, 64)]
    s256 = smp.band_sample_set(256, 1, 4, 64, 256)
    assert [(x.g, x.m, x.n) for x in s256] == [(64, 1, 64), (128, 1, 128), (192, 1, 192), (256, 1, 256)]
    # split in two: task counts are multiples of 2 * m; 17 rows under a 16-row tile are 2 tile rows
    assert [(x.g, x.m, x.n) for x in smp.band_sample_set(256, 1, 2, 17, 16, S=2)] == [(128, 2, 32), (256, 2, 64)]
    for rows in smp.ROW_BANDS:
        for bm in (16, 64, 256):
            for x in smp.band_sample_set(256, 3, 4, rows, bm):
                a, b = smp.sub_interval(x.w, x.i, 256, 4)
                m = geo.ceil_div(rows, bm)
                assert x.g == 0 or (x.m == m and a <= x.g <= b and x.g == m * x.n and m * (x.n + 1) > b)

    W, W_row, I = 6, 2, 4
    near = _make_samples(W, I, _penalty)
    slow = {1: 3.0, 2: 2.0}
    extra = []
    for f in (1, 2):
        for k, kd in enumerate(KEYS):
            for x in smp.band_sample_set(kd.cap, W_row, I, smp.ROW_BANDS[f - 1], kd.bm):
                if x.g == 0:
                    continue
                for L in smp.loop_anchors(K_ANCHORS, kd.bk):
                    for mi in range(N_MICRO):
                        extra.append(ofit.Sample(k, mi, x.g, L, x.w, slow[f] * _latency(k, mi, x.g, L, 6, _penalty), f))
    table = ofit.fit_tables(near + extra, KEYS, W, p=3, W_row=W_row, row_fams=2, row_mode=1)
    tiles = ofit.fit_tables(near + extra, KEYS, W, p=3, W_row=W_row, row_fams=2, row_mode=0)
    assert table.row_mode == 1 and table.row_fams == 2 and tiles.row_mode == 0
    for M, f in ((1, 1), (16, 1), (17, 2), (32, 2), (33, 3), (200, 0)):
        for kid, kd in enumerate(KEYS):
            assert osel.family_of(table, M, kd.bm) == f                 # the same family under every key
    for kid in range(len(KEYS)):                                        # a band the table lacks: the paper's buckets
        assert osel.bucket_for(table, kid, 1, 3) is table.local[kid][0]
        assert osel.bucket_for(table, kid, 1, 2) is table.row_local[1][kid][0]
    # the tile-row rule on the same M = 30: two tile rows under the 16-row key, one under the 256-row key
    assert (osel.family_of(tiles, 30, 16), osel.family_of(tiles, 30, 256)) == (2, 1)
    assert osel.family_of(ofit.fit_tables(near, KEYS, W, p=3), 5, 16) == 0          # no families in the table
    for (M, N, K) in ((12, 4096, 4096), (30, 4096, 2048), (33, 4096, 4096)):
        f = smp.band_family(M) if smp.band_family(M) <= 2 else 0
        cand = []
        for kid, kd in enumerate(KEYS):
            G, L = geo.phi_gemm(M, N, K, kd.bm, kd.bn, kd.bk)
            for mi in range(N_MICRO):
                cand.append(((kid, mi), slow.get(f, 1.0) * _latency(kid, mi, G, L, W, _penalty)))
        (bk, _), bt = oex.argmin_config(cand)
        key, _, t = osel.select(table, M, N, K)
        assert key == bk and abs(t - bt) < 1e-6 * bt
    # the grouped selectors take the band of one group's rows (uniform reading) or of the mean group (real counts)
    kd = KEYS[4]                                     # <16, 64, 128>: 4 groups of 10 rows are 4 x 64 tasks of band 1
    G, L = geo.phi_grouped([10] * 4, 4096, 4096, kd.bm, kd.bn, kd.bk)
    b = osel.bucket_for(table, 4, geo.wave_count(G, kd.cap), 1)
    assert b is table.row_local[0][4][0]
    got = osel.select_grouped(table, 4, 40, 4096, 4096)
    assert got == osel.select_grouped_rows(table, [10, 10, 10, 10], 4096, 4096)
    if got[0] == 4:
        assert got[2] == osel.predict(b.theta, G, L)


def test_thin_anchors_keeps_ends_and_an_even_spread():
    """Buckets with more loop counts than the table holds keep ranks floor(i*(n-1)/7): hand values."""
    a15 = [(L, L % 3) for L in range(10, 25)]
    assert ofit.thin_anchors(a15, 8) == [a15[i] for i in (0, 2, 4, 6, 8, 10, 12, 14)]
    a9 = [(L, 0) for L in range(9)]
    assert ofit.thin_anchors(a9, 8) == [a9[i] for i in (0, 1, 2, 3, 4, 5, 6, 8)]
    a8 = [(L, 1) for L in range(8)]
    assert ofit.thin_anchors(a8, 8) == a8 and ofit.thin_anchors(a8[:3], 8) == a8[:3]
    assert ofit.thin_anchors(a15, 2) == [a15[0], a15[-1]]
    assert ofit.thin_anchors(a15) == a15          # no limit given (the method as stated): every anchor is kept


def test_select_attn_hand_worked_two_keys():
    """Two attention keys <T_Q, T_KV> = <64, 32> and <256, 64> with hand-set planes: S_q = 300, S_kv = 1000, 8 heads.
    Key 0: G = 8*ceil(300/64) = 40, L = ceil(1000/32) = 32 -> T = 0.01*40*32 + 1 = 13.8.
    Key 1: G = 8*ceil(300/256) = 16, L = ceil(1000/64) = 16 -> T = 0.05*16*16 + 2 = 14.8.  Key 0 wins; its anchors
    (L = 10 -> micro 2, L = 40 -> micro 0): 32 is nearer to 40.  At S_kv = 4000 (L = 125 / 63) key 1 wins:
    0.01*40*125 + 1 = 51 against 0.05*16*63 + 2 = 52.4 -> still key 0; at 64 heads and w > W the ext tuples decide."""
    keys = [ofit.KeyDesc(64, 1, 32, 2, 1, 1, 256), ofit.KeyDesc(256, 1, 64, 8, 1, 1, 256)]
    b0 = ofit.Bucket(theta=(0.01, 0.0, 0.0, 1.0), status=15, anchors=[(10, 2), (40, 0)])
    b1 = ofit.Bucket(theta=(0.05, 0.0, 0.0, 2.0), status=15, anchors=[(16, 1)])
    e0 = ofit.Bucket(theta=(0.02, 0.0, 0.0, 0.0), status=15, anchors=[(10, 1)])
    e1 = ofit.Bucket(theta=(0.01, 0.0, 0.0, 0.0), status=15, anchors=[(16, 2)])
    table = ofit.DualTable(W=1, keys=keys, local=[[b0], [b1]], ext=[e0, e1])
    k, micro, t = osel.select_attn(table, 8, 300, 1000)
    assert (k, micro) == (0, 0) and t == pytest.approx(13.8)
    k, micro, t = osel.select_attn(table, 8, 300, 4000)
    assert (k, micro) == (0, 0) and t == pytest.approx(51.0)
    # 64 heads, S_q = 1024: key 0 has G = 1024 (w = 4 > W), key 1 has G = 256 (w = 1, local bucket)
    # key 0 ext: 0.02*1024*32 = 655.36; key 1 local: 0.05*256*16 + 2 = 206.8 -> key 1, micro of its only anchor
    k, micro, t = osel.select_attn(table, 64, 1024, 1024)
    assert (k, micro) == (1, 1) and t == pytest.approx(206.8)
    # 128 heads: both beyond W -> ext tuples: key 0: 0.02*2048*32 = 1310.72; key 1: 0.01*512*16 = 81.92
    k, micro, t = osel.select_attn(table, 128, 1024, 1024)
    assert (k, micro) == (1, 2) and t == pytest.approx(81.92)


def test_select_attn_varlen_hand_worked_and_equal_lengths():
    """Two prompts of 100 and 900 tokens (queries = keys), 8 heads, keys <64, 32> and <256, 64>, planes T = a*G*L + d.
    Real lengths:  key 0: tiles 2 + 15 = 17, iterations 2*4 + 15*29 = 443, L = round(26.06) = 26, G = 136,
                          T = 0.01*136*26 + 1 = 36.36
                   key 1: tiles 1 + 4 = 5, iterations 1*2 + 4*15 = 62, L = round(12.4) = 12, G = 40,
                          T = 0.06*40*12 + 7 = 35.8   <- wins; its anchors L = 8 and 16 are equally far: the smaller.
    Mean length 500 (what a selector that sees only totals prices): key 0: G = 16*8 = 128, L = 16 -> 21.48 <- wins,
    anchors 10 and 40: 10; key 1: G = 16*2 = 32, L = 8 -> 22.36.  So the case tells the two readings apart."""
    keys = [ofit.KeyDesc(64, 1, 32, 2, 1, 1, 256), ofit.KeyDesc(256, 1, 64, 8, 1, 1, 256)]
    b0 = ofit.Bucket(theta=(0.01, 0.0, 0.0, 1.0), status=15, anchors=[(10, 2), (40, 0)])
    b1 = ofit.Bucket(theta=(0.06, 0.0, 0.0, 7.0), status=15, anchors=[(8, 1), (16, 2)])
    e0 = ofit.Bucket(theta=(0.02, 0.0, 0.0, 0.0), status=15, anchors=[(10, 1)])
    e1 = ofit.Bucket(theta=(0.01, 0.0, 0.0, 0.0), status=15, anchors=[(16, 2)])
    table = ofit.DualTable(W=1, keys=keys, local=[[b0], [b1]], ext=[e0, e1])
    k, micro, t = osel.select_attn_varlen(table, 8, [100, 900], [100, 900])
    assert (k, micro) == (1, 1) and t == pytest.approx(35.8)
    k, micro, t = osel.select_attn(table, 2 * 8, 500, 500)
    assert (k, micro) == (0, 2) and t == pytest.approx(21.48)
    # no block at all: G = L = 0 lies outside every wave bucket, the extrapolation constants decide (a tie at 0: key 0)
    assert osel.select_attn_varlen(table, 8, [0, 0], [5, 5])[0] == 0
    # equal lengths: the fixed-length selector with the batch folded into the heads
    rng = np.random.default_rng(3)
    for _ in range(200):
        b, H = int(rng.integers(1, 9)), int(rng.integers(1, 33))
        S_q, S_kv = int(rng.integers(1, 3000)), int(rng.integers(1, 6000))
        assert osel.select_attn_varlen(table, H, [S_q] * b, [S_kv] * b) == osel.select_attn(table, b * H, S_q, S_kv)


def test_r_squared_exact_surface_hand_value_and_constant_rows():
    """Coefficient of determination R^2 = 1 - SS_res/SS_tot (the statistic Sec. 3.3 / Fig. 5 quotes for the G- and
    L-linearity of a wave).  (i) rows lying on the plane -> exactly 1; (ii) a hand case: T = (1, 2, 6) at
    (G, L) = (1,0), (2,0), (3,0) against the line T-hat = 2G - 1 = (1, 3, 5): SS_res = 0 + 1 + 1 = 2, mean 3,
    SS_tot = 4 + 1 + 9 = 14 -> R^2 = 1 - 2/14 = 6/7; (iii) a model no better than the mean -> 0; worse than the mean
    -> negative; (iv) constant rows have SS_tot = 0 and are defined as 1; (v) the least-squares fit of noisy rows
    maximises R^2: perturbing any coefficient lowers it."""
    theta = (0.003, 0.25, 1.5, 7.0)
    rows = [(g, l, theta[0] * g * l + theta[1] * g + theta[2] * l + theta[3]) for g in (260, 300, 410, 512) for l in (16, 48, 80)]
    assert ofit.r_squared(rows, theta) == pytest.approx(1.0, abs=1e-14)
    hand = [(1, 0, 1.0), (2, 0, 2.0), (3, 0, 6.0)]
    assert ofit.r_squared(hand, (0.0, 2.0, 0.0, -1.0)) == pytest.approx(6.0 / 7.0, abs=1e-15)
    assert ofit.r_squared(hand, (0.0, 0.0, 0.0, 3.0)) == pytest.approx(0.0, abs=1e-15)
    assert ofit.r_squared(hand, (0.0, 0.0, 0.0, 10.0)) < 0.0
    assert ofit.r_squared([(1, 1, 5.0), (2, 3, 5.0)], (0.0, 0.0, 0.0, 4.0)) == 1.0
    rng = np.random.default_rng(8)
    noisy = [(g, l, t * (1.0 + 0.05 * rng.standard_normal())) for (g, l, t) in rows]
    best, _ = ofit.fit_bilinear(noisy)
    r2 = ofit.r_squared(noisy, best)
    assert 0.9 < r2 < 1.0
    for i in range(4):
        worse = list(best)
        worse[i] *= 1.02
        assert ofit.r_squared(noisy, tuple(worse)) < r2


# ---- relative least squares (every record weighs 1/T^2) ----------------------------------------------
def test_relative_fit_recovers_an_exact_surface_and_differs_from_the_absolute_fit_on_noise():
    th = (3e-4, 0.02, 0.5, 7.0)
    rows = [(g, l, th[0] * g * l + th[1] * g + th[2] * l + th[3]) for g in (260, 300, 390, 512) for l in (4, 16, 64, 448)]
    got, status = ofit.fit_bilinear(rows, relative=True)
    assert status == 0b1111 and np.allclose(got, th, rtol=1e-9)
    noisy = [(g, l, t * (1.0 + 0.05 * ((i * 7) % 5 - 2) / 2)) for i, (g, l, t) in enumerate(rows)]
    a, _ = ofit.fit_bilinear(noisy)
    r, _ = ofit.fit_bilinear(noisy, relative=True)
    assert not np.allclose(a, r, rtol=1e-4)

    def sum_sq(theta, rel):
        return sum(((theta[0] * g * l + theta[1] * g + theta[2] * l + theta[3] - t) / (t if rel else 1.0)) ** 2
                   for g, l, t in noisy)
    # each fit is the better one under its own objective
    assert sum_sq(r, True) < sum_sq(a, True) and sum_sq(a, False) < sum_sq(r, False)


def test_relative_fit_matches_exact_rational_weighted_normal_equations():
    """The minimiser of sum(((x.theta - T)/T)^2) solves (X^T D X) theta = X^T D T with D = diag(1/T^2): solved here
    in exact rationals, in the raw variables (no centring, no scaling), by Gauss-Jordan elimination."""
    rows = [(257, 8, Fraction(31, 4)), (257, 40, Fraction(97, 4)), (300, 8, Fraction(17, 2)), (300, 40, Fraction(121, 4)),
            (390, 8, Fraction(45, 4)), (390, 40, Fraction(151, 4)), (512, 8, Fraction(27, 2)), (512, 40, Fraction(95, 2)),
            (512, 224, Fraction(1001, 4)), (257, 224, Fraction(533, 4))]
    X = [[Fraction(g * l), Fraction(g), Fraction(l), Fraction(1)] for g, l, _ in rows]
    A = [[sum(X[n][i] * X[n][j] / rows[n][2] ** 2 for n in range(len(rows))) for j in range(4)] for i in range(4)]
    b = [sum(X[n][i] / rows[n][2] for n in range(len(rows))) for i in range(4)]     # x * T / T^2
    for c in range(4):
        piv = next(r for r in range(c, 4) if A[r][c] != 0)
        A[c], A[piv], b[c], b[piv] = A[piv], A[c], b[piv], b[c]
        for r in range(4):
            if r != c:
                f = A[r][c] / A[c][c]
                A[r] = [x - f * y for x, y in zip(A[r], A[c])]
                b[r] -= f * b[c]
    exact = [float(b[i] / A[i][i]) for i in range(4)]
    got, status = ofit.fit_bilinear([(g, l, float(t)) for g, l, t in rows], relative=True)
    assert status == 0b1111
    pred = lambda th, g, l: th[0] * g * l + th[1] * g + th[2] * l + th[3]
    for g, l, _ in rows:      # coefficients cancel heavily: compare through the predictions they give
        assert abs(pred(got, g, l) - pred(exact, g, l)) <= 1e-9 * abs(pred(exact, g, l))


def test_relative_fit_of_a_constant_is_the_ratio_of_inverse_sums():
    # one grid size, one loop count: d minimises sum((d - T)^2 / T^2)  =>  d = sum(1/T) / sum(1/T^2)
    got, status = ofit.fit_bilinear([(64, 8, 1.0), (64, 8, 2.0)], relative=True)
    assert status == 0b1000 and got[:3] == (0.0, 0.0, 0.0) and abs(got[3] - 1.2) < 1e-12
    # a single distinct G: slope and intercept in L, again by hand -- T(L=1) in {1, 2}, T(L=3) = 4:
    # weights 1, 1/4, 1/16; normal equations of c*L + d:  [[1+1/4+9/16, 1+1/4+3/16],[.., 1+1/4+1/16]] [c d] = [1+1/2+3/4, 1+1/2+1/4]
    got, status = ofit.fit_bilinear([(64, 1, 1.0), (64, 1, 2.0), (64, 3, 4.0)], relative=True)
    A = np.array([[29 / 16, 23 / 16], [23 / 16, 21 / 16]])
    c, d = np.linalg.solve(A, np.array([9 / 4, 7 / 4]))
    assert status == 0b1100 and abs(got[2] - c) < 1e-12 and abs(got[3] - d) < 1e-12
    with pytest.raises(ValueError):
        ofit.fit_bilinear([(64, 8, 0.0), (64, 8, 2.0)], relative=True)
