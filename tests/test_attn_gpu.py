"""GPU parity: wt_attn (through the C ABI) against the fp64 oracle, element by element.

Tolerance: |O - O_ref| <= 2e-2 * max(|O_ref|, rms(O_ref)) per element, rms over the rows compared -- the same
reading of "2e-2 per element, bf16 out" as for the GEMM (a purely relative error is undefined where O_ref crosses
zero, and an absolute floor would be vacuous at long KV lengths, where outputs average thousands of N(0,1) values
and have rms 0.01-0.02).  Expected error: inputs are bf16; scores and the online softmax are fp32; probabilities
are rounded to bf16 before they multiply V (2^-9 relative per term, independent over the keys -> about 1e-3 of the
output's rms) and the output is rounded to bf16 (2^-9 relative).
"""
import math

import numpy as np
import pytest
import torch

import paper_2604_10187_amd as wt
import wt_synth
from gpu_util import all_configs, dev_bits, note
from oracle import attention as oa
from oracle import gemm as og

pytestmark = pytest.mark.gpu

ELEM_TOL = 2e-2
SCALE = 1.0 / math.sqrt(128.0)


@pytest.fixture(scope="module")
def ctx():
    c = wt.wt_create(0, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    yield c
    wt.wt_destroy(c)


def run_attn(ctx, cfg, qb, kb, vb, causal, scale=SCALE):
    S_q, H_q, _ = qb.shape
    S_kv, H_kv, _ = kb.shape
    dQ, dK, dV = (dev_bits(x.reshape(-1, 128)).view(torch.bfloat16) for x in (qb, kb, vb))
    dO = torch.full((max(S_q, 1) * H_q, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    wt.wt_attn(ctx, H_q, H_kv, S_q, S_kv, dQ, dK, dV, dO, scale, causal, cfg, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    return dO.float().cpu().numpy()[: S_q * H_q].reshape(S_q, H_q, 128)


def reference(qb, kb, vb, causal, scale=SCALE):
    dec = lambda b: og.bf16_bits_to_f64(b.reshape(-1, 128)).reshape(b.shape)
    return oa.attention(dec(qb), dec(kb), dec(vb), scale, causal)


# largest scaled errors seen in this session (printed by the last test): scaled by the rms of everything compared,
# and by the rms of the element's own output row (one query of one head, 128 values)
WORST = {"err": 0.0, "what": "", "err_row": 0.0, "what_row": ""}


def _scaled(diff, want, rms):
    scale = np.maximum(np.abs(want), rms)
    return np.divide(diff, scale, out=np.where(diff > 0, np.inf, 0.0), where=scale > 0)   # all-zero reference: exact


def check(got, want, what):
    """Both bounds must hold: every element within 2e-2 of max(|O_ref|, rms over all compared elements), and within
    2e-2 of max(|O_ref|, rms of its own 128-value output row).  The second is the tighter one wherever rows differ
    in scale (under a causal mask a late row averages hundreds of keys and is ten times smaller than an early one)."""
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    if not want.size:
        return
    diff = np.abs(got - want)
    err = _scaled(diff, want, math.sqrt(float(np.mean(np.square(want)))))
    err_row = _scaled(diff, want, np.sqrt(np.mean(np.square(want), axis=-1, keepdims=True)))
    if float(err.max()) > WORST["err"]:
        WORST.update(err=float(err.max()), what=what)
    if float(err_row.max()) > WORST["err_row"]:
        WORST.update(err_row=float(err_row.max()), what_row=what)
    assert err.max() <= ELEM_TOL, f"{what}: max scaled error {err.max():.4g} at {np.unravel_index(err.argmax(), err.shape)}"
    assert err_row.max() <= ELEM_TOL, f"{what}: max row-scaled error {err_row.max():.4g} at {np.unravel_index(err_row.argmax(), err_row.shape)}"


def test_every_config_is_launchable(ctx):
    assert wt.wt_key_count(ctx) >= 8
    for cfg, res in all_configs(ctx):
        assert res.occ >= 1 and res.lds_bytes <= 160 * 1024, cfg


def test_every_config_matches_the_oracle_on_ragged_shapes(ctx):
    """Every <T_Q, T_KV, wavefronts, order>: several query tiles and KV tiles with ragged tails in both, grouped
    heads (3 query heads per KV head)."""
    for cfg, _ in all_configs(ctx):
        S_q, S_kv, H_q, H_kv = 2 * cfg.bm + 19, 3 * cfg.bk + 21, 6, 2
        note(f"attn cfg={cfg.astuple()} S_q={S_q} S_kv={S_kv}")
        qb, kb, vb = wt_synth.attn_operands(S_q, S_kv, H_q, H_kv, 300 + cfg.id)
        check(run_attn(ctx, cfg, qb, kb, vb, 0), reference(qb, kb, vb, False), f"{cfg}")


def test_causal_matches_the_oracle(ctx):
    """Causal masking with the queries aligned to the end of the keys: square prefill and a prefix of 77 cached
    tokens, for every structural key (order 0 and 2)."""
    for cfg, _ in all_configs(ctx):
        if cfg.swizzle == 1:
            continue
        for S_q, S_kv in ((2 * cfg.bm + 5, 2 * cfg.bm + 5), (cfg.bm + 40, cfg.bm + 117)):
            note(f"attn causal cfg={cfg.astuple()} S_q={S_q} S_kv={S_kv}")
            qb, kb, vb = wt_synth.attn_operands(S_q, S_kv, 4, 4, 500 + cfg.id)
            check(run_attn(ctx, cfg, qb, kb, vb, 1), reference(qb, kb, vb, True), f"causal {cfg} {S_q}x{S_kv}")


def test_batched_launch_equals_one_launch_per_sequence(ctx):
    """wt_attn_batched on [batch, S, H, 128] operands: every sequence against the fp64 oracle, and bit for bit what
    wt_attn writes for that sequence alone; every structural key under every block order, ragged lengths, grouped
    heads, causal and not (Table 2's attention row with the batch folded into the head count)."""
    batch, H_q, H_kv = 3, 4, 2
    for cfg, _ in all_configs(ctx):
        S_q, S_kv = cfg.bm + 37, 2 * cfg.bk + 9 + cfg.bm
        seqs = [wt_synth.attn_operands(S_q, S_kv, H_q, H_kv, 900 + 7 * cfg.id + b) for b in range(batch)]
        qb, kb, vb = (np.stack([s[i] for s in seqs]) for i in range(3))
        dQ, dK, dV = (dev_bits(x.reshape(-1, 128)).view(torch.bfloat16) for x in (qb, kb, vb))
        for causal in (0, 1):
            note(f"attn batched cfg={cfg.astuple()} S_q={S_q} S_kv={S_kv} causal={causal}")
            dO = torch.full((batch * S_q * H_q, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
            wt.wt_attn_batched(ctx, batch, H_q, H_kv, S_q, S_kv, dQ, dK, dV, dO, SCALE, causal, cfg,
                               stream=torch.cuda.current_stream())
            torch.cuda.synchronize()
            got = dO.float().cpu().numpy().reshape(batch, S_q, H_q, 128)
            for b in range(batch):
                check(got[b], reference(qb[b], kb[b], vb[b], bool(causal)), f"batched {cfg} seq {b} causal {causal}")
                assert np.array_equal(got[b], run_attn(ctx, cfg, qb[b], kb[b], vb[b], causal)), (cfg, b, causal)
    # Phi of a batched launch: the batch multiplies the head count
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 128, 1, 64, 4, 1, 0))
    G, L, w = wt.wt_wave_count(ctx, 1000, batch * 32, 3000, cfg)
    assert (G, L) == (batch * 32 * 8, 47) and w == -(-G // 256)
    # batch = 0 is a no-op; a negative batch is refused
    wt.wt_attn_batched(ctx, 0, H_q, H_kv, S_q, S_kv, dQ, dK, dV, dO, SCALE, 0, cfg, stream=torch.cuda.current_stream())
    with pytest.raises(wt.WtError):
        wt.wt_attn_batched(ctx, -1, H_q, H_kv, S_q, S_kv, dQ, dK, dV, dO, SCALE, 0, cfg, stream=torch.cuda.current_stream())


def test_variable_length_batch_equals_one_launch_per_sequence(ctx):
    """wt_attn_varlen: sequences of different lengths packed back to back, offsets resident on the device -- an empty
    sequence, one shorter than a tile, several tiles with ragged tails, decode-like (1 query, long context) and a
    causal sequence with fewer keys than queries.  Every sequence against the oracle and bit for bit against wt_attn on
    that sequence alone, for every structural key (one block order each)."""
    H_q, H_kv = 4, 2
    lens = [(0, 0), (5, 9), (300, 300), (1, 700), (130, 257), (64, 40), (517, 517)]
    batch = len(lens)
    seqs = [wt_synth.attn_operands(max(sq, 1), max(sk, 1), H_q, H_kv, 1300 + b) for b, (sq, sk) in enumerate(lens)]
    qb = np.concatenate([s[0][:sq] for s, (sq, sk) in zip(seqs, lens)])
    kb = np.concatenate([s[1][:sk] for s, (sq, sk) in zip(seqs, lens)])
    vb = np.concatenate([s[2][:sk] for s, (sq, sk) in zip(seqs, lens)])
    cu_q = np.concatenate([[0], np.cumsum([l[0] for l in lens])]).astype(np.int32)
    cu_kv = np.concatenate([[0], np.cumsum([l[1] for l in lens])]).astype(np.int32)
    tq, tkv = int(cu_q[-1]), int(cu_kv[-1])
    dQ, dK, dV = (dev_bits(x.reshape(-1, 128)).view(torch.bfloat16) for x in (qb, kb, vb))
    dcq, dck = torch.from_numpy(cu_q).cuda(), torch.from_numpy(cu_kv).cuda()
    for cfg, _ in all_configs(ctx):
        if cfg.swizzle != (cfg.id // 3) % 3:
            continue
        for causal in (0, 1):
            note(f"attn varlen cfg={cfg.astuple()} causal={causal}")
            dO = torch.full((tq * H_q, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
            wt.wt_attn_varlen(ctx, batch, H_q, H_kv, tq, tkv, dcq, dck, dQ, dK, dV, dO, SCALE, causal, cfg,
                              stream=torch.cuda.current_stream())
            torch.cuda.synchronize()
            got = dO.float().cpu().numpy().reshape(tq, H_q, 128)
            assert np.isfinite(got).all()
            for b, (sq, sk) in enumerate(lens):
                if sq == 0:
                    continue
                mine = got[cu_q[b]:cu_q[b + 1]]
                q1, k1, v1 = qb[cu_q[b]:cu_q[b + 1]], kb[cu_kv[b]:cu_kv[b + 1]], vb[cu_kv[b]:cu_kv[b + 1]]
                if causal and sk < sq:
                    # queries i with i + (sk - sq) < 0 see no key: zeros; the rest see keys 0 .. i + sk - sq
                    assert not mine[: sq - sk].any()
                    check(mine[sq - sk:], reference(q1[sq - sk:], k1, v1, True), f"varlen {cfg} seq {b} causal short")
                    continue
                check(mine, reference(q1, k1, v1, bool(causal)), f"varlen {cfg} seq {b} causal {causal}")
                assert np.array_equal(mine, run_attn(ctx, cfg, q1, k1, v1, causal)), (cfg, b, causal)
    # offsets that point outside the tensors are clipped, never followed: the launch completes and writes nothing wild
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 128, 1, 64, 4, 1, 0))
    bad = torch.tensor([0, -5, 10 ** 9, 7, tq + 99, tq, tq, tq], dtype=torch.int32, device="cuda")
    guard = torch.full(((tq + 8) * H_q, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    wt.wt_attn_varlen(ctx, batch, H_q, H_kv, tq, tkv, bad, bad, dQ, dK, dV, guard, SCALE, 0, cfg, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert (guard[tq * H_q:] == 7.0).all() and torch.isfinite(guard.float()).all()


def test_sharp_softmax_and_scale(ctx):
    """Queries with gain 6 make the softmax nearly one-hot (large score range): exercises the running maximum
    and the rescaling; also a non-default scale."""
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 128, 1, 64, 4, 1, 0))
    qb, kb, vb = wt_synth.attn_operands(200, 700, 4, 2, 71, q_gain=6.0)
    check(run_attn(ctx, cfg, qb, kb, vb, 0), reference(qb, kb, vb, False), "sharp")
    check(run_attn(ctx, cfg, qb, kb, vb, 0, scale=0.31), reference(qb, kb, vb, False, scale=0.31), "scale 0.31")


def test_degenerate_sizes(ctx):
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 64, 1, 32, 2, 1, 2))
    for S_q, S_kv in ((1, 1), (1, 33), (65, 1), (3, 0)):
        note(f"attn degenerate S_q={S_q} S_kv={S_kv}")
        qb, kb, vb = wt_synth.attn_operands(S_q, S_kv, 2, 1, 90 + S_q + S_kv)
        check(run_attn(ctx, cfg, qb, kb, vb, 0), reference(qb, kb, vb, False), f"{S_q}x{S_kv}")
    # S_q = 0 is a no-op
    wt.wt_attn(ctx, 2, 1, 0, 5, None, None, None, None, SCALE, 0, cfg)
    torch.cuda.synchronize()


def test_full_size_sampled_rows(ctx):
    """16384 x 16384, 16 heads (4 KV heads), the launch configuration the evaluation times: the oracle computes a
    sample of query rows one by one (each a softmax over all 16384 keys), non-causal and causal."""
    S, H_q, H_kv = 16384, 16, 4
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 256, 1, 64, 8, 1, 2))
    note(f"attn full size S={S} cfg={cfg.astuple()}")
    qb, kb, vb = wt_synth.attn_operands(S, S, H_q, H_kv, 77)
    dec = lambda b: og.bf16_bits_to_f64(b.reshape(-1, 128)).reshape(b.shape)
    K64, V64 = dec(kb), dec(vb)
    rows = [0, 1, 255, 256, 4097, 8191, 12345, 16383]
    for causal in (0, 1):
        got = run_attn(ctx, cfg, qb, kb, vb, causal)
        for i in rows:
            q1 = dec(qb[i:i + 1])
            keys = i + 1 if causal else S       # S_q == S_kv: query i sees keys 0..i
            want = oa.attention(q1, K64[:keys], V64[:keys], SCALE, False)
            check(got[i:i + 1], want, f"full-size row {i} causal={causal}")


def test_bench_shape_under_the_selected_config(ctx):
    """The shape bench.py reports (8192 x 8192, 32 query / 8 KV heads) under the configuration wt_select returns from
    the shipped attention table: sampled query rows against the oracle."""
    import os

    S, H_q, H_kv = 8192, 32, 8
    sel = wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    try:
        wt.wt_load(sel, os.path.join(os.path.dirname(wt.LIB_PATH), "tables", "mi355x_attn.wt"))
        pick = wt.wt_select(sel, S, H_q, S)
    finally:
        wt.wt_destroy(sel)
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, pick.bm, 1, pick.bk, pick.nwave, 1, pick.swizzle))
    note(f"attn bench shape S={S} H={H_q}/{H_kv} cfg={cfg.astuple()}")
    qb, kb, vb = wt_synth.attn_operands(S, S, H_q, H_kv, 78)
    dec = lambda b: og.bf16_bits_to_f64(b.reshape(-1, 128)).reshape(b.shape)
    K64, V64 = dec(kb), dec(vb)
    got = run_attn(ctx, cfg, qb, kb, vb, 0)
    for i in (0, 255, 256, 4095, 8191):
        want = oa.attention(dec(qb[i:i + 1]), K64, V64, SCALE, False)
        check(got[i:i + 1], want, f"bench-shape row {i}")


def test_ragged_batch_under_the_varlen_selectors_pick(ctx):
    """A ragged causal prefill batch (four prompts, 8 query / 2 KV heads) under the configuration that
    wt_select_attn_varlen returns from the shipped table for its real lengths: the pick is the oracle's, and every
    sequence of the launch is checked against the fp64 oracle."""
    import os
    from oracle import select as osel

    lens, H_q, H_kv = [700, 90, 1500, 33], 8, 2
    path = os.path.join(os.path.dirname(wt.LIB_PATH), "tables", "mi355x_attn.wt")
    wt.wt_load(ctx, path)
    pick = wt.wt_select_attn_varlen(ctx, lens, lens, H_q)
    table, _ = osel.read_table(path)
    key, micro, _ = osel.select_attn_varlen(table, H_q, lens, lens)
    kd = table.keys[key]
    assert (pick.bm, pick.bk, pick.nwave, pick.swizzle) == (kd.bm, kd.bk, kd.nwave, micro)
    note(f"attn ragged batch lens={lens} H={H_q}/{H_kv} cfg={pick.astuple()}")
    seqs = [wt_synth.attn_operands(s, s, H_q, H_kv, 1700 + b) for b, s in enumerate(lens)]
    qb, kb, vb = (np.concatenate([s[i] for s in seqs]) for i in range(3))
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    total = sum(lens)
    dQ, dK, dV = (dev_bits(x.reshape(-1, 128)).view(torch.bfloat16) for x in (qb, kb, vb))
    dO = torch.full((total * H_q, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    wt.wt_attn_varlen(ctx, len(lens), H_q, H_kv, total, total, cu, cu, dQ, dK, dV, dO, SCALE, 1, pick,
                      stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = dO.float().cpu().numpy().reshape(total, H_q, 128)
    off = 0
    for b, s in enumerate(lens):
        check(got[off:off + s], reference(*seqs[b], True), f"ragged batch seq {b}")
        off += s


def test_many_heads_and_decode_like_shapes(ctx):
    """128 query heads on 2 KV heads (the widest grouping of the test ranges), a single query against 20 000 keys
    (one block per head, 157-313 KV tiles, ragged tail), and a causal single query (sees every key)."""
    cfg_a, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 128, 1, 128, 4, 1, 1))
    cfg_b, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 64, 1, 64, 2, 1, 2))
    for cfg, (S_q, S_kv, H_q, H_kv), causal in ((cfg_a, (70, 300, 128, 2), 0), (cfg_b, (1, 20000, 8, 4), 0),
                                                 (cfg_a, (1, 20000, 8, 4), 1), (cfg_b, (33, 5000, 16, 16), 1)):
        note(f"attn cfg={cfg.astuple()} S_q={S_q} S_kv={S_kv} H={H_q}/{H_kv} causal={causal}")
        qb, kb, vb = wt_synth.attn_operands(S_q, S_kv, H_q, H_kv, 7000 + S_q + H_q)
        check(run_attn(ctx, cfg, qb, kb, vb, causal), reference(qb, kb, vb, bool(causal)), f"{S_q}x{S_kv} H={H_q}/{H_kv}")


def test_hip_graph_replay(ctx):
    """wt_attn neither allocates nor synchronises: a captured launch replays bit-identically, with eager launches
    and synchronisations between the replays."""
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 256, 1, 64, 8, 1, 2))
    S_q, S_kv, H_q, H_kv = 700, 1500, 8, 2
    qb, kb, vb = wt_synth.attn_operands(S_q, S_kv, H_q, H_kv, 4242)
    dQ, dK, dV = (dev_bits(x.reshape(-1, 128)).view(torch.bfloat16) for x in (qb, kb, vb))
    eager = torch.empty((S_q * H_q, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(eager)
    wt.wt_attn(ctx, H_q, H_kv, S_q, S_kv, dQ, dK, dV, eager, SCALE, 1, cfg, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    check(eager.float().cpu().numpy().reshape(S_q, H_q, 128), reference(qb, kb, vb, True), "eager")
    cur = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(cur)
    with torch.cuda.stream(side):       # warm-up on a side stream, as torch asks before a capture
        wt.wt_attn(ctx, H_q, H_kv, S_q, S_kv, dQ, dK, dV, out, SCALE, 1, cfg, stream=side)
    cur.wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        wt.wt_attn(ctx, H_q, H_kv, S_q, S_kv, dQ, dK, dV, out, SCALE, 1, cfg, stream=torch.cuda.current_stream())
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager launch"
        wt.wt_attn(ctx, H_q, H_kv, S_q, S_kv, dQ, dK, dV, eager, SCALE, 1, cfg, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()


def test_profile_fit_select_round_trip(ctx):
    """wt_profile_sparse on an attention context: the records are the plan the oracle derives (head-aligned grid
    sizes, KV multipliers, Eq. 6), every latency is positive, and a table fitted from them selects one of the
    profiled keys with a finite prediction."""
    heads, W, I, mult = 16, 2, 3, (100, 200, 300)
    first, count = 2, 2
    grid = wt.make_grid(W=W, I=I, k_anchors=mult, warmup=1, iters=1, key_first=first, key_count=count, n_heads=heads)
    n, bQ, bKV, bO = wt.wt_sample_plan(ctx, grid)
    note(f"attn profile: {n} records, Q {bQ >> 20} MiB, KV {bKV >> 20} MiB")
    scrQ = torch.randn(bQ // 2, device="cuda").to(torch.bfloat16)
    scrKV = torch.randn(bKV // 2, device="cuda").to(torch.bfloat16)
    scrO = torch.empty(bO // 2, dtype=torch.bfloat16, device="cuda")
    recs = wt.wt_profile_sparse(ctx, grid, scrQ, scrKV, scrO, stream=torch.cuda.current_stream())
    want = []
    for k in range(first, first + count):
        cfg, res = wt.wt_config_get(ctx, 3 * k)
        for s in oa.sample_set_heads(256, W, I, heads):
            if s.g == 0:
                continue
            S_q, _ = oa.instantiate_attn(s.g, 1, heads, cfg.bm, cfg.bk)
            for L in oa.kv_loop_counts(S_q, cfg.bk, mult):
                want += [(k, m, s.g, L, s.w) for m in range(3)]
    assert len(recs) == n == len(want)
    assert [(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"])) for r in recs] == want
    assert (recs["mean_us"] > 0).all() and np.isfinite(recs["mean_us"]).all()
    # more work takes longer: within a key and micro, the largest (G, L) is slower than the smallest
    r0 = recs[(recs["key_id"] == first) & (recs["micro_id"] == 0)]
    assert r0["mean_us"][np.argmax(r0["G"] * r0["L"])] > r0["mean_us"][np.argmin(r0["G"] * r0["L"])]
    c2 = wt.wt_create(-1, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    try:
        wt.wt_fit(c2, grid, recs)
        for (S_q, S_kv, H) in ((512, 512, 16), (4096, 8192, 32), (100, 100, 64)):
            pick = wt.wt_select(c2, S_q, H, S_kv)
            _, res = wt.wt_config_get(c2, pick.id)
            assert first <= res.key_id < first + count
            assert np.isfinite(wt.wt_predict_us(c2, S_q, H, S_kv, pick))
    finally:
        wt.wt_destroy(c2)


def test_argument_errors(ctx):
    cfg, _ = wt.wt_config_get(ctx, 0)
    t = torch.zeros(64 * 4 * 128, dtype=torch.bfloat16, device="cuda")
    for args in ((4, 3, 8, 8), (0, 1, 8, 8), (4, 4, -1, 8)):
        with pytest.raises(wt.WtError):
            wt.wt_attn(ctx, args[0], args[1], args[2], args[3], t, t, t, t, SCALE, 0, cfg)
    with pytest.raises(wt.WtError):   # causal with fewer keys than queries
        wt.wt_attn(ctx, 4, 4, 16, 8, t, t, t, t, SCALE, 1, cfg)
    for bad_scale in (0.0, -0.5, float("nan"), float("inf")):
        with pytest.raises(wt.WtError):
            wt.wt_attn(ctx, 4, 4, 8, 8, t, t, t, t, bad_scale, 0, cfg)
    with pytest.raises(wt.WtError):   # a GEMM call on an attention context
        wt.wt_gemm(ctx, 8, 8, 8, t, t, t, cfg)
    bad = wt.wt_cfg(64, 1, 48, 2, 1, 0, 1, -1)
    with pytest.raises(wt.WtError):
        wt.wt_attn(ctx, 4, 4, 8, 8, t, t, t, t, SCALE, 0, bad)


def test_zz_report_worst_scaled_error():
    """Not a check of its own: prints the largest |O - O_ref| / max(|O_ref|, rms) the checks above saw."""
    note(f"attention parity: worst scaled error {WORST['err']:.3e} ({WORST['what']}); "
         f"worst row-scaled error {WORST['err_row']:.3e} ({WORST['what_row']}); bound {ELEM_TOL}")
    assert WORST["err"] <= ELEM_TOL and WORST["err_row"] <= ELEM_TOL
