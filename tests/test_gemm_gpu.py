"""GPU parity: wt_gemm (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2604_10187_amd as wt
import wt_synth
from gpu_util import all_configs, note, run_gemm, run_gemm_grouped
from oracle import gemm as og

pytestmark = pytest.mark.gpu

F32_REL_FROB = 1e-3     # fp32 output: ||C - C_ref||_F / ||C_ref||_F
BF16_ELEM = 2e-2        # bf16 output: |C - C_ref| / max(|C_ref|, rms(C_ref)) per element


@pytest.fixture(scope="module")
def ctx_f32():
    c = wt.wt_create(0, wt.WT_BF16, wt.WT_OUT_F32)
    yield c
    wt.wt_destroy(c)


@pytest.fixture(scope="module")
def ctx_bf16():
    c = wt.wt_create(0, wt.WT_BF16, wt.WT_OUT_BF16)
    yield c
    wt.wt_destroy(c)


def _bf16_case(M, N, K, seed, kind):
    a32, b32 = wt_synth.gemm_operands(M, N, K, seed, kind)
    return wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)


def test_every_config_is_launchable(ctx_f32):
    for cfg, res in all_configs(ctx_f32):
        assert res.occ >= 1, f"{cfg} does not fit the device"
        assert res.lds_bytes <= 160 * 1024


def test_integer_matrices_bit_exact_every_config(ctx_f32):
    """Integer entries in [-8,8]: all partial sums are exact in fp32, so every configuration --
    every tile shape, stage count and rasterisation -- must reproduce the oracle bit for bit,
    including ragged M/N edges and a K that is not a multiple of BK."""
    for cfg, res in all_configs(ctx_f32):
        M, N, K = 2 * cfg.bm + 17, cfg.bn + 33, 2 * cfg.bk + 24
        note(f"int-exact cfg={cfg.astuple()} shape={(M, N, K)}")
        ab, bb = _bf16_case(M, N, K, 100 + cfg.id, "int")
        want = og.gemm_c(ab, bb)
        got = run_gemm(ctx_f32, cfg, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
        assert np.array_equal(got, want), f"{cfg}: max diff {np.abs(got - want).max()}"


def test_rasterisation_modes_cover_every_tile_once(ctx_f32):
    """Many-tile grids with ragged group and XCD remainders (38 x 12 and 5 x 29 tiles): every
    rasterisation mode must still compute every tile exactly once -- bit-exact on integer inputs."""
    for (tiles_m, tiles_n) in ((38, 12), (5, 29), (1, 61)):
        for sw in (0, 1, 2):
            cfg, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, 64, 64, 64, 4, 2, sw))
            M, N, K = 64 * (tiles_m - 1) + 5, 64 * (tiles_n - 1) + 3, 136
            note(f"rasterisation sw={sw} grid={tiles_m}x{tiles_n}")
            ab, bb = _bf16_case(M, N, K, 700 + sw, "int")
            got = run_gemm(ctx_f32, cfg, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
            assert np.array_equal(got, og.gemm_c(ab, bb))


def test_config1_256_cubed_normal(ctx_f32):
    """Single bf16 GEMM M=N=K=256, N(0,1) inputs, fp32 accumulate/out, over the
    BM,BN in {64,128} x BK in {32,64} x stages in {1,2} grid where the registry has it."""
    ab, bb = _bf16_case(256, 256, 256, 1001, "normal")
    want = og.gemm_c(ab, bb)
    n = 0
    for cfg, res in all_configs(ctx_f32):
        if cfg.bm in (64, 128) and cfg.bn in (64, 128) and cfg.bk in (32, 64):
            note(f"cfg1 cfg={cfg.astuple()}")
            got = run_gemm(ctx_f32, cfg, ab, bb, wt.WT_OUT_F32)
            assert og.rel_frobenius(got, want) <= F32_REL_FROB
            assert og.rel_frobenius(got, want) <= 1e-5      # fp32 accumulation of 256 terms
            n += 1
    assert n >= 8


@pytest.mark.parametrize("M", [1, 16, 17, 64, 100, 333])
def test_ragged_m_normal(ctx_f32, M):
    N, K = 1000, 1032
    ab, bb = _bf16_case(M, N, K, wt_synth.shape_seed(1002, M, N, K), "normal")
    want = og.gemm_c(ab, bb)
    for cfg, res in all_configs(ctx_f32):
        if cfg.swizzle != (M % 3):
            continue
        note(f"ragged M={M} cfg={cfg.astuple()}")
        got = run_gemm(ctx_f32, cfg, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
        assert og.rel_frobenius(got, want) <= 1e-5


def test_bf16_output(ctx_bf16):
    M, N, K = 300, 520, 1024
    ab, bb = _bf16_case(M, N, K, 1004, "normal")
    want = og.gemm_c(ab, bb)
    for cfg, res in all_configs(ctx_bf16):
        if cfg.swizzle != 1:
            continue
        note(f"bf16-out cfg={cfg.astuple()}")
        got = run_gemm(ctx_bf16, cfg, ab, bb, wt.WT_OUT_BF16)
        assert og.max_scaled_err(got, want) <= BF16_ELEM
        assert og.max_scaled_err(got, want) <= 2.0 ** -8    # one bf16 rounding of an fp32 sum


def test_unaligned_output_rows_and_pointer(ctx_f32, ctx_bf16):
    """The line-wise epilogue needs 16-byte aligned rows of C; everything else falls back to element-wise stores.
    Integer inputs (bit-exact) on kernels that stage C through LDS and on one that does not: N a multiple of 8 with C
    16-byte aligned (line-wise path), the same C shifted by one element (pointer unaligned), N = 8k + 4 (bf16 rows
    unaligned, fp32 rows aligned) and N odd; untouched guard elements before and after C stay NaN."""
    keys = ((256, 256, 64, 4, 2, 0), (256, 256, 64, 8, 2, 2), (128, 128, 64, 4, 3, 1), (128, 64, 128, 4, 2, 0),
            (64, 64, 64, 4, 2, 0), (16, 64, 128, 4, 2, 0), (128, 128, 64, 4, 3, 0, 2))
    for ctx, dt in ((ctx_f32, torch.float32), (ctx_bf16, torch.bfloat16)):
        for fields in keys:
            cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, *fields))
            for (M, N) in ((cfg.bm + 37, 2 * cfg.bn + 8), (cfg.bm + 37, cfg.bn + 12), (70, cfg.bn + 33)):
                K = 2 * cfg.bk * cfg.split + 24
                ab, bb = _bf16_case(M, N, K, 900 + N, "int")
                want = torch.from_numpy(og.gemm_c(ab, bb).astype(np.float32))   # exact integers below 2^24
                if dt == torch.bfloat16:
                    want = want.to(torch.bfloat16).float()      # one round-to-nearest-even of the exact sum
                dA = torch.from_numpy(ab.view(np.int16).copy()).cuda()
                dB = torch.from_numpy(bb.view(np.int16).copy()).cuda()
                for shift in (0, 1):
                    note(f"epilogue paths cfg={cfg.astuple()} out={dt} shape={(M, N, K)} shift={shift}")
                    buf = torch.full((M * N + 16,), float("nan"), dtype=dt, device="cuda")
                    dC = buf[8 + shift: 8 + shift + M * N].view(M, N)
                    assert (dC.data_ptr() % 16 == 0) == (shift == 0)
                    wt.wt_gemm(ctx, M, N, K, dA, dB, dC, cfg, stream=torch.cuda.current_stream())
                    torch.cuda.synchronize()
                    assert torch.equal(dC.float().cpu(), want), f"{cfg} {dt} N={N} shift={shift}"
                    guard = torch.cat([buf[: 8 + shift], buf[8 + shift + M * N:]])
                    assert torch.isnan(guard).all(), "wrote outside C"


def test_outputs_beyond_the_streaming_threshold_bit_exact(ctx_f32, ctx_bf16):
    """A C of more than 128 MiB is written with non-temporal stores (the line-wise epilogue's other branch): integer
    inputs, bit-exact against the oracle, fp32 and bf16 out, one block per task."""
    for ctx, dt, (M, N) in ((ctx_f32, wt.WT_OUT_F32, (6144, 5640)), (ctx_bf16, wt.WT_OUT_BF16, (8200, 8328))):
        K = 136
        assert M * N * (4 if dt == wt.WT_OUT_F32 else 2) > 128 << 20
        ab, bb = _bf16_case(M, N, K, 990 + dt, "int")
        want = og.gemm_c(ab, bb).astype(np.float32)
        if dt == wt.WT_OUT_BF16:
            want = torch.from_numpy(want).to(torch.bfloat16).float().numpy()
        for fields in ((256, 256, 64, 4, 2, 0), (128, 128, 64, 4, 3, 1), (256, 128, 64, 8, 2, 2)):
            cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, *fields))
            note(f"streaming C cfg={cfg.astuple()} out={dt} shape={(M, N, K)}")
            got = run_gemm(ctx, cfg, ab, bb, dt, fill=float("nan"))
            assert np.array_equal(got, want), f"{cfg}"


def _split_configs(ctx):
    return [(c, r) for c, r in all_configs(ctx) if c.split > 1]


def test_split_k_normal_inputs_repeated_launches(ctx_f32, ctx_bf16):
    """Split-K configurations on N(0,1) data with many k-tiles per split, a ragged K tail in the last
    split, ragged M/N, and three launches in a row into fresh outputs: every launch must leave the
    arrival counters clean for the next, and -- the partial tiles being added in split order whatever
    the arrival order -- produce the same bits each time."""
    M, N, K = 333, 1000, 4104
    ab, bb = _bf16_case(M, N, K, wt_synth.shape_seed(1002, M, N, K), "normal")
    want = og.gemm_c(ab, bb)
    assert len(_split_configs(ctx_f32)) >= 3 * 15
    for cfg, res in _split_configs(ctx_f32):
        if cfg.swizzle != cfg.id % 3:
            continue
        note(f"split-K f32 cfg={cfg.astuple()}")
        first = None
        for rep in range(3):
            got = run_gemm(ctx_f32, cfg, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
            assert og.rel_frobenius(got, want) <= 1e-5
            first = got if first is None else first
            assert np.array_equal(got, first)
    for cfg, res in _split_configs(ctx_bf16):
        if cfg.swizzle != 1 or cfg.split != 4:
            continue
        note(f"split-K bf16-out cfg={cfg.astuple()}")
        got = run_gemm(ctx_bf16, cfg, ab, bb, wt.WT_OUT_BF16)
        assert og.max_scaled_err(got, want) <= BF16_ELEM
        assert og.max_scaled_err(got, want) <= 2.0 ** -8


def test_split_k_many_tiles_and_unsplit_between(ctx_f32):
    """A grid of several hundred tiles x 4 splits (more tasks than can be resident at once, so splits
    of one tile run far apart in time), interleaved with an unsplit launch on the same stream."""
    cfg, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, 64, 64, 128, 4, 3, 1, 4))
    plain, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, 64, 64, 128, 4, 3, 1, 1))
    M, N, K = 64 * 19 + 7, 64 * 23 + 9, 2048 + 64
    note(f"split-K many tiles cfg={cfg.astuple()} shape={(M, N, K)}")
    ab, bb = _bf16_case(M, N, K, 4242, "int")
    want = og.gemm_c(ab, bb)
    for c in (cfg, plain, cfg):
        got = run_gemm(ctx_f32, c, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
        assert np.array_equal(got, want)


def test_split_k_workspace_limit(ctx_f32):
    """Shapes whose partial tiles exceed the context's workspace are refused, not truncated."""
    cfg, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, 128, 128, 64, 4, 3, 0, 8))
    dA = torch.zeros(8, dtype=torch.int16, device="cuda")
    M = N = 128 * 23                          # 23 x 23 tiles x 8 x 128 x 128 floats > 2^26
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx_f32, M, N, 8, dA, dA, dA, cfg, stream=torch.cuda.current_stream())
    assert e.value.status == wt.WT_ERR_INFEASIBLE


# ---- HIP graph capture -------------------------------------------------------------------------------
def test_launches_replay_from_a_hip_graph(ctx_f32):
    """wt_gemm neither allocates nor synchronises, so a sequence of launches (an unsplit one, two split-K
    ones that share the context's workspace and counters, a grouped one) can be captured into a HIP graph.
    Every replay -- with eager launches and synchronisations between replays -- must reproduce the eager
    result bit for bit."""
    cases = [((300, 520, 1032), (128, 128, 64, 4, 3, 1, 1)), ((130, 1000, 4104), (64, 64, 128, 4, 3, 2, 4)),
             ((64, 777, 2056), (16, 64, 256, 4, 3, 0, 2))]
    bufs, eager = [], []
    cur = torch.cuda.current_stream()
    for (M, N, K), f in cases:
        ab, bb = _bf16_case(M, N, K, 9100 + M, "normal")
        cfg, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, *f))
        dA, dB = torch.from_numpy(ab.view(np.int16).copy()).cuda(), torch.from_numpy(bb.view(np.int16).copy()).cuda()
        bufs.append((M, N, K, cfg, dA, dB, torch.empty((M, N), dtype=torch.float32, device="cuda")))
    counts = [40, 0, 200, 7]
    off = wt_synth.group_offsets(counts)
    gab, _ = wt_synth.gemm_operands(int(off[-1]), 8, 520, 9200)
    gbb, _ = wt_synth.gemm_operands(4 * 300, 8, 520, 9201)
    gA = torch.from_numpy(wt_synth.to_bf16_bits(gab).view(np.int16).copy()).cuda()
    gB = torch.from_numpy(wt_synth.to_bf16_bits(gbb).view(np.int16).copy()).cuda()
    gC = torch.empty((int(off[-1]), 300), dtype=torch.float32, device="cuda")
    gOff = torch.from_numpy(off.copy()).cuda()
    gcfg, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, 32, 64, 128, 4, 3, 1))

    def launch_all(stream):
        for (M, N, K, cfg, dA, dB, dC) in bufs:
            wt.wt_gemm(ctx_f32, M, N, K, dA, dB, dC, cfg, stream=stream)
        wt.wt_gemm_grouped(ctx_f32, 4, gOff, int(off[-1]), 300, 520, gA, gB, gC, gcfg, stream=stream)

    note("graph: eager reference")
    launch_all(cur)
    torch.cuda.synchronize()
    eager = [b[6].clone() for b in bufs] + [gC.clone()]
    side = torch.cuda.Stream()
    side.wait_stream(cur)
    with torch.cuda.stream(side):       # warm-up on a side stream, as torch asks before a capture
        launch_all(side)
    cur.wait_stream(side)
    torch.cuda.synchronize()
    note("graph: capture")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launch_all(torch.cuda.current_stream())
    for rep in range(3):
        for b in bufs:
            b[6].fill_(float("nan"))
        gC.fill_(float("nan"))
        note(f"graph: replay {rep}")
        g.replay()
        torch.cuda.synchronize()
        got = [b[6] for b in bufs] + [gC]
        assert all(torch.equal(x, y) for x, y in zip(got, eager)), f"replay {rep}"
        launch_all(cur)                 # eager work between replays
        torch.cuda.synchronize()
        assert all(torch.equal(x, y) for x, y in zip(got, eager))


# ---- persistent launches ---------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [1, 2])
def test_persistent_launch_bit_exact(ctx_f32, mode):
    """Grid clamped to the resident block count (mode 1: fixed stride through the task list, mode 2: tasks drawn from
    the device-side queue, which every launch must leave at zero for the next): on problems with more tasks than
    that, every structural key (split-K ones included) must give the bits of the one-block-per-task launch and of
    the oracle.  Where the kernel has room it requests the next task's first k-tiles before the current epilogue."""
    import math

    wt.wt_set_persistent(ctx_f32, mode)
    try:
        for cfg, res in all_configs(ctx_f32):
            if cfg.swizzle != cfg.id // 3 % 3:
                continue
            # tiles, so that tasks exceed what is resident (every third key: by more than two rounds)
            need = ((256 * res.occ) // cfg.split) * (3 if cfg.id % 9 == 0 and cfg.bm * cfg.bn <= 128 * 128 else 1) + 37
            tm = max(2, math.isqrt(need))
            tn = -(-need // tm) + 1
            M, N, K = tm * cfg.bm - 3, tn * cfg.bn - 5, cfg.split * cfg.bk * (1 + cfg.id % 4) + 24
            G, L, w = wt.wt_wave_count(ctx_f32, M, N, K, cfg)
            assert G > 256 * res.occ
            note(f"persistent mode={mode} cfg={cfg.astuple()} shape={(M, N, K)} tasks={G} resident={256 * res.occ}")
            ab, bb = _bf16_case(M, N, K, 300 + cfg.id, "int")
            got = run_gemm(ctx_f32, cfg, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
            assert np.array_equal(got, og.gemm_c(ab, bb)), f"{cfg}"
    finally:
        wt.wt_set_persistent(ctx_f32, False)


@pytest.mark.parametrize("mode", [1, 2])
def test_persistent_grouped_and_normal(ctx_bf16, mode):
    """Persistent launch of a grouped problem (surplus blocks past the last row tile) and of an N(0,1)
    problem spanning several waves, bf16 out."""
    wt.wt_set_persistent(ctx_bf16, mode)
    try:
        counts = [700, 0, 33, 1, 900, 64, 2000]
        off = wt_synth.group_offsets(counts)
        E, N, K = len(counts), 1000, 264
        a32, _ = wt_synth.gemm_operands(int(off[-1]), 8, K, 8901)
        b32, _ = wt_synth.gemm_operands(E * N, 8, K, 8902)
        ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32).reshape(E, N, K)
        want = og.grouped_gemm_c(ab, bb, off)
        for fields in ((64, 64, 64, 4, 2, 1), (32, 64, 128, 4, 3, 2), (128, 128, 64, 4, 3, 0)):
            cfg, _ = wt.wt_config_get(ctx_bf16, wt.wt_config_find(ctx_bf16, *fields))
            note(f"persistent grouped cfg={cfg.astuple()}")
            got = run_gemm_grouped(ctx_bf16, cfg, ab, bb, off, wt.WT_OUT_BF16)
            assert og.max_scaled_err(got, want) <= 2.0 ** -8
        M, N, K = 2500, 3000, 1032
        ab, bb = _bf16_case(M, N, K, 8903, "normal")
        want = og.gemm_c(ab, bb)
        for fields in ((64, 64, 128, 4, 3, 1), (128, 128, 64, 4, 4, 2), (64, 64, 128, 4, 3, 0, 2)):
            cfg, _ = wt.wt_config_get(ctx_bf16, wt.wt_config_find(ctx_bf16, *fields))
            note(f"persistent normal cfg={cfg.astuple()}")
            got = run_gemm(ctx_bf16, cfg, ab, bb, wt.WT_OUT_BF16)
            assert og.max_scaled_err(got, want) <= 2.0 ** -8
    finally:
        wt.wt_set_persistent(ctx_bf16, False)


# ---- grouped GEMM ---------------------------------------------------------------------------------
def test_grouped_integer_bit_exact(ctx_f32):
    """Ragged groups (one empty, one of a single row, sizes that are no multiple of any tile) on integer
    data: every unsplit structural key, one rasterisation mode each, must equal the oracle's per-group
    products bit for bit, and must leave rows of no group untouched."""
    counts = [130, 0, 17, 1, 300, 64]
    off = wt_synth.group_offsets(counts)
    E, N, K = len(counts), 200, 136
    M_total = int(off[-1]) + 5                        # five trailing rows belong to no group
    a32, _ = wt_synth.gemm_operands(M_total, 8, K, 8801, "int")
    b32, _ = wt_synth.gemm_operands(E * N, 8, K, 8802, "int")
    ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32).reshape(E, N, K)
    want = og.grouped_gemm_c(ab, bb, off)
    n = 0
    for cfg, res in all_configs(ctx_f32):
        if cfg.split != 1 or cfg.swizzle != (cfg.id // 3) % 3:
            continue
        note(f"grouped int-exact cfg={cfg.astuple()}")
        got = run_gemm_grouped(ctx_f32, cfg, ab, bb, off, wt.WT_OUT_F32, fill=float("nan"))
        assert np.array_equal(got[:off[-1]], want[:off[-1]]), f"{cfg}"
        assert np.isnan(got[off[-1]:]).all()
        n += 1
    assert n >= 50
    split_cfg = next(c for c, _ in all_configs(ctx_f32) if c.split > 1)
    with pytest.raises(wt.WtError) as e:
        run_gemm_grouped(ctx_f32, split_cfg, ab, bb, off, wt.WT_OUT_F32)
    assert e.value.status == wt.WT_ERR_UNSUPPORTED_CFG


def test_grouped_moe_layer_normal(ctx_bf16):
    """A 128-expert / top-8 layer's fused gate+up projection (N = 1536, K = 2048) for 256 tokens with a
    skewed synthetic routing, N(0,1) data, bf16 out, under three configurations."""
    E, top_k, N, K = wt_synth.MOE_LAYERS[0]
    counts = wt_synth.moe_routing(256, E, top_k, seed=77, skew=1.2)
    off = wt_synth.group_offsets(counts)
    M_total = int(off[-1])
    assert M_total == 256 * top_k and counts.min() == 0
    a32, _ = wt_synth.gemm_operands(M_total, 8, K, 8811)
    b32, _ = wt_synth.gemm_operands(E * N, 8, K, 8812)
    ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32).reshape(E, N, K)
    want = og.grouped_gemm_c(ab, bb, off)
    for fields in ((16, 64, 128, 4, 5, 0), (64, 64, 128, 4, 3, 1), (128, 128, 64, 4, 3, 2)):
        cfg, _ = wt.wt_config_get(ctx_bf16, wt.wt_config_find(ctx_bf16, *fields))
        note(f"grouped MoE layer cfg={cfg.astuple()} rows={M_total}")
        got = run_gemm_grouped(ctx_bf16, cfg, ab, bb, off, wt.WT_OUT_BF16)
        assert og.max_scaled_err(got, want) <= BF16_ELEM
        assert og.max_scaled_err(got, want) <= 2.0 ** -8
    # the same launch under what the two grouped selectors return from the shipped table (the uniform reading of the
    # routing, and its real counts): both are the oracle's picks on that table, and both launches are correct
    import os
    from oracle import select as osel
    from _pins import split_limits
    path = os.path.join(os.path.dirname(wt.LIB_PATH), "tables", "mi355x_in0_out1.wt")
    sel = wt.wt_create(-1, wt.WT_BF16, wt.WT_OUT_BF16)
    try:
        wt.wt_load(sel, path)
        picks = [wt.wt_select_grouped(sel, E, M_total, N, K), wt.wt_select_grouped_rows(sel, counts, N, K)]
    finally:
        wt.wt_destroy(sel)
    table, _ = osel.read_table(path, **split_limits())
    wants = [osel.select_grouped(table, E, M_total, N, K), osel.select_grouped_rows(table, counts.tolist(), N, K)]
    for pick, (key, micro, _) in zip(picks, wants):
        kd = table.keys[key]
        assert (pick.bm, pick.bn, pick.bk, pick.nwave, pick.stages, pick.swizzle, pick.split) == \
            (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, micro, 1)
        cfg, _ = wt.wt_config_get(ctx_bf16, wt.wt_config_find(ctx_bf16, pick.bm, pick.bn, pick.bk, pick.nwave, pick.stages, pick.swizzle))
        note(f"grouped MoE layer under the selector's pick cfg={cfg.astuple()}")
        got = run_gemm_grouped(ctx_bf16, cfg, ab, bb, off, wt.WT_OUT_BF16)
        assert og.max_scaled_err(got, want) <= 2.0 ** -8


def test_degenerate_shapes_and_errors(ctx_f32):
    cfg, _ = wt.wt_config_get(ctx_f32, 0)
    stream = torch.cuda.current_stream()
    dA = torch.zeros(64, dtype=torch.int16, device="cuda")
    dC = torch.full((4, 8), 7.0, dtype=torch.float32, device="cuda")
    wt.wt_gemm(ctx_f32, 0, 8, 16, dA, dA, dC, cfg, stream=stream)       # M = 0: nothing happens
    wt.wt_gemm(ctx_f32, 4, 0, 16, dA, dA, dC, cfg, stream=stream)       # N = 0
    torch.cuda.synchronize()
    assert torch.all(dC == 7.0)
    wt.wt_gemm(ctx_f32, 4, 8, 0, None, None, dC, cfg, stream=stream)    # K = 0: C = 0
    torch.cuda.synchronize()
    assert torch.all(dC == 0.0)
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx_f32, 4, 8, 12, dA, dA, dC, cfg, stream=stream)   # K not a multiple of 8
    assert e.value.status == wt.WT_ERR_INVALID_ARG
    bad = wt.wt_cfg(100, 100, 64, 4, 2, 0, 1, -1)
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx_f32, 4, 8, 16, dA, dA, dC, bad, stream=stream)
    assert e.value.status == wt.WT_ERR_UNSUPPORTED_CFG
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx_f32, 4, 8, 16, None, dA, dC, cfg, stream=stream)
    assert e.value.status == wt.WT_ERR_INVALID_ARG


# ---- fp8 e4m3 ----------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def ctx_fp8_f32():
    c = wt.wt_create(0, wt.WT_FP8_E4M3, wt.WT_OUT_F32)
    yield c
    wt.wt_destroy(c)


@pytest.fixture(scope="module")
def ctx_fp8_bf16():
    c = wt.wt_create(0, wt.WT_FP8_E4M3, wt.WT_OUT_BF16)
    yield c
    wt.wt_destroy(c)


def test_fp8_integer_matrices_bit_exact_every_config(ctx_fp8_f32):
    """Integers in [-8,8] are exact in e4m3; with unit scales the fp32 result must equal the oracle
    bit for bit for every fp8 configuration (ragged edges, K not a multiple of BK)."""
    for cfg, res in all_configs(ctx_fp8_f32):
        assert res.occ >= 1
        M, N, K = cfg.bm + 17, 2 * cfg.bn + 5, 2 * cfg.bk + 48
        note(f"fp8 int-exact cfg={cfg.astuple()} shape={(M, N, K)}")
        a32, b32 = wt_synth.gemm_operands(M, N, K, 500 + cfg.id, "int")
        aq = torch.from_numpy(a32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        bq = torch.from_numpy(b32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        want = og.gemm_c(aq, bq, "e4m3", 1.0, 1.0)
        got = run_gemm(ctx_fp8_f32, cfg, aq, bq, wt.WT_OUT_F32, 1.0, 1.0, fill=float("nan"))
        assert np.array_equal(got, want), f"{cfg}: max diff {np.abs(got - want).max()}"


def test_flagship_kernels_every_k_tile_count_bit_exact(ctx_f32, ctx_fp8_f32):
    """The two large-prefill kernels (bf16 256x256x64 and fp8 256x256x128 on four wavefronts) run their k-tiles in a
    software pipeline whose prologue issues two k-tiles and, for fp8, handles k-tiles in pairs: every k-tile count
    from 1 to 6, with and without a partial last k-tile, ragged M and N, integer data, bit for bit."""
    for ctx, kind, fields, align in ((ctx_f32, "bf16", (256, 256, 64, 4, 2, 1), 8), (ctx_fp8_f32, "e4m3", (256, 256, 128, 4, 2, 1), 16)):
        cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, *fields))
        M, N = 300, 523
        for tiles in range(1, 7):
            for K in (tiles * cfg.bk, (tiles - 1) * cfg.bk + align, (tiles - 1) * cfg.bk + cfg.bk - align):
                note(f"k-tile counts {kind} cfg={cfg.astuple()} K={K}")
                a32, b32 = wt_synth.gemm_operands(M, N, K, 7100 + K, "int")
                if kind == "bf16":
                    ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)
                    want = og.gemm_c(ab, bb, "bf16")
                    got = run_gemm(ctx, cfg, ab, bb, wt.WT_OUT_F32, fill=float("nan"))
                else:
                    ab = torch.from_numpy(a32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                    bb = torch.from_numpy(b32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                    want = og.gemm_c(ab, bb, "e4m3", 1.0, 1.0)
                    got = run_gemm(ctx, cfg, ab, bb, wt.WT_OUT_F32, 1.0, 1.0, fill=float("nan"))
                assert np.array_equal(got, want), f"{kind} K={K}: max diff {np.abs(got - want).max()}"


def test_fp8_scaled_normal_inputs(ctx_fp8_f32, ctx_fp8_bf16):
    """N(0,1) inputs quantised with per-tensor scales s = amax/448; C = sA*sB*sum(qA*qB)."""
    M, N, K = 200, 333, 1040
    a32, b32 = wt_synth.gemm_operands(M, N, K, 1004)
    aq, sa = wt_synth.to_e4m3_bits(a32)
    bq, sb = wt_synth.to_e4m3_bits(b32)
    want = og.gemm_c(aq, bq, "e4m3", sa, sb)
    for cfg, res in all_configs(ctx_fp8_f32):
        if cfg.swizzle != 2:
            continue
        note(f"fp8 normal f32-out cfg={cfg.astuple()}")
        got = run_gemm(ctx_fp8_f32, cfg, aq, bq, wt.WT_OUT_F32, float(sa), float(sb))
        # the fp8 MFMA sums its 64/128 products in a wide-but-truncating adder tree before the fp32
        # accumulate; the observed error is ~1.5e-5, far inside the 1e-3 bar
        assert og.rel_frobenius(got, want) <= F32_REL_FROB
        assert og.rel_frobenius(got, want) <= 1e-4
    for cfg, res in all_configs(ctx_fp8_bf16):
        if cfg.swizzle != 0:
            continue
        note(f"fp8 normal bf16-out cfg={cfg.astuple()}")
        got = run_gemm(ctx_fp8_bf16, cfg, aq, bq, wt.WT_OUT_BF16, float(sa), float(sb))
        assert og.max_scaled_err(got, want) <= BF16_ELEM


def test_fp8_grouped_and_persistent_bit_exact(ctx_fp8_f32):
    """fp8 inputs through the grouped and the persistent launch paths (integer data, unit scales)."""
    counts = [70, 0, 5, 129]
    off = wt_synth.group_offsets(counts)
    E, N, K = len(counts), 150, 304
    a32, _ = wt_synth.gemm_operands(int(off[-1]), 16, K, 8921, "int")
    b32, _ = wt_synth.gemm_operands(E * N, 16, K, 8922, "int")
    aq = torch.from_numpy(a32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    bq = torch.from_numpy(b32).to(torch.float8_e4m3fn).view(torch.uint8).numpy().reshape(E, N, K)
    want = og.grouped_gemm_c(aq, bq, off, "e4m3", 1.0, 1.0)
    one = torch.ones(1, dtype=torch.float32, device="cuda")
    dOff = torch.from_numpy(off.copy()).cuda()
    dA, dB = torch.from_numpy(aq.copy()).cuda(), torch.from_numpy(bq.reshape(E * N, K).copy()).cuda()
    for persistent in (0, 1, 2):
        wt.wt_set_persistent(ctx_fp8_f32, persistent)
        try:
            for cfg, res in all_configs(ctx_fp8_f32):
                if cfg.split != 1 or cfg.swizzle != (cfg.id // 3) % 3:
                    continue
                note(f"fp8 grouped persistent={persistent} cfg={cfg.astuple()}")
                dC = torch.full((int(off[-1]), N), float("nan"), dtype=torch.float32, device="cuda")
                wt.wt_gemm_grouped(ctx_fp8_f32, E, dOff, int(off[-1]), N, K, dA, dB, dC, cfg, one, one,
                                   stream=torch.cuda.current_stream())
                torch.cuda.synchronize()
                assert np.array_equal(dC.cpu().numpy(), want), f"{cfg}"
        finally:
            wt.wt_set_persistent(ctx_fp8_f32, False)


# ---- full-size shapes, checked on sampled rows / columns / edge tiles ----------------------------
def _sampled_check(ctx, cfg, M, N, K, in_type, out_type, seed, n_rows=12, n_cols=6):
    """Run the full-size GEMM on the GPU and compare complete sampled rows and columns (random ones
    plus the first and last of each dimension) with fp64 dot products."""
    rng = np.random.default_rng(seed)
    a32, b32 = wt_synth.gemm_operands(M, N, K, seed)
    if in_type == wt.WT_BF16:
        ab, bb, sa, sb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32), None, None
        a, b = og.decode(ab, "bf16"), og.decode(bb, "bf16")
    else:
        (ab, sa), (bb, sb) = wt_synth.to_e4m3_bits(a32), wt_synth.to_e4m3_bits(b32)
        a, b = og.decode(ab, "e4m3", sa), og.decode(bb, "e4m3", sb)
        sa, sb = float(sa), float(sb)
    del a32, b32
    got = run_gemm(ctx, cfg, ab, bb, out_type, sa, sb)
    rows = sorted({0, M - 1, *rng.integers(0, M, size=min(n_rows, M)).tolist()})
    cols = sorted({0, N - 1, *rng.integers(0, N, size=min(n_cols, N)).tolist()})
    want_r, want_c = og.rows_f64(a, b, rows), og.cols_f64(a, b, cols)
    if out_type == wt.WT_OUT_F32:
        assert og.rel_frobenius(got[rows], want_r) <= F32_REL_FROB
        assert og.rel_frobenius(got[:, cols], want_c) <= F32_REL_FROB
    else:
        # per-element bound relative to max(|C_ref|, rms): rms over the sampled rows
        assert og.max_scaled_err(got[rows], want_r) <= BF16_ELEM
        assert og.max_scaled_err(got[:, cols], want_c) <= BF16_ELEM
    assert np.isfinite(got).all()


def _large_prefill_configs(ctx, in_type, four_wave, eight_wave):
    """The configuration bench.py times on 16384 x 8192 x 8192 (wt_select on the shipped table) and the two 256 x 256
    kernels it chooses between, whatever the table says today."""
    import os

    from paper_2604_10187_amd import tune

    cfgs = {}
    path = tune.table_path(in_type, wt.WT_OUT_BF16)
    if os.path.exists(path):
        wt.wt_load(ctx, path)
        pick = wt.wt_select(ctx, 16384, 8192, 8192)
        cfgs[pick.id] = pick
    for fields in (four_wave, eight_wave):
        c, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, *fields))
        cfgs.setdefault(c.id, c)
    return list(cfgs.values())


def test_large_prefill_bf16_sampled(ctx_bf16):
    """16384 x 8192 x 8192, bf16 in / bf16 out, under the selector's pick and both flagship kernels."""
    for cfg in _large_prefill_configs(ctx_bf16, wt.WT_BF16, (256, 256, 64, 4, 2, 0), (256, 256, 64, 8, 2, 2)):
        note(f"large prefill bf16 cfg={cfg.astuple()}")
        _sampled_check(ctx_bf16, cfg, 16384, 8192, 8192, wt.WT_BF16, wt.WT_OUT_BF16, 1004, n_rows=8, n_cols=4)


def test_large_prefill_fp8_sampled(ctx_fp8_bf16):
    for cfg in _large_prefill_configs(ctx_fp8_bf16, wt.WT_FP8_E4M3, (256, 256, 128, 4, 2, 1), (256, 256, 128, 8, 2, 0)):
        note(f"large prefill fp8 cfg={cfg.astuple()}")
        _sampled_check(ctx_fp8_bf16, cfg, 16384, 8192, 8192, wt.WT_FP8_E4M3, wt.WT_OUT_BF16, 1014, n_rows=8, n_cols=4)


def test_sweep_shapes_full_size_under_selected_config(ctx_bf16):
    """The 27 LLM-projection shapes at full size, each under the configuration bench.py times for it
    (wt_select on the shipped dual table; a fixed fallback configuration if no table is shipped)."""
    import os

    from paper_2604_10187_amd import tune

    path = tune.table_path(wt.WT_BF16, wt.WT_OUT_BF16)
    have_table = os.path.exists(path)
    if have_table:
        wt.wt_load(ctx_bf16, path)
    for (M, N, K) in wt_synth.sweep_shapes():
        if have_table:
            cfg = wt.wt_select(ctx_bf16, M, N, K)
        else:
            cfg, _ = wt.wt_config_get(ctx_bf16, wt.wt_config_find(ctx_bf16, 128, 128, 64, 4, 2, 0))
        note(f"sweep {M}x{N}x{K} cfg={cfg.astuple()}")
        _sampled_check(ctx_bf16, cfg, M, N, K, wt.WT_BF16, wt.WT_OUT_BF16, wt_synth.shape_seed(1002, M, N, K),
                       n_rows=6, n_cols=3)


def test_stream_and_wave_stress_shapes_full_size_under_selected_config(ctx_bf16):
    """Seeded picks from the 10 000-shape runtime stream (K = 8192 and 28672, where wt_select often
    chooses split-K) and from the wave-quantisation stress set, at full size under wt_select's
    configuration, checked on sampled rows and columns."""
    import os

    from paper_2604_10187_amd import tune

    path = tune.table_path(wt.WT_BF16, wt.WT_OUT_BF16)
    if not os.path.exists(path):
        pytest.skip("no shipped dual table")
    wt.wt_load(ctx_bf16, path)
    stream = wt_synth.stream_shapes()
    rng = np.random.default_rng(77)
    shapes = [stream[i] for i in rng.choice(len(stream), size=10, replace=False)]
    shapes += [s for s in stream if s[2] == 28672 and 100 <= s[0] <= 300][:2]        # split-K territory
    shapes += wt_synth.wave_stress_shapes()[15::37]
    n_split = 0
    for (M, N, K) in shapes:
        cfg = wt.wt_select(ctx_bf16, M, N, K)
        n_split += cfg.split > 1
        note(f"stream/wave {M}x{N}x{K} cfg={cfg.astuple()}")
        _sampled_check(ctx_bf16, cfg, M, N, K, wt.WT_BF16, wt.WT_OUT_BF16, wt_synth.shape_seed(1005, M, N, K),
                       n_rows=4, n_cols=2)
    assert n_split >= 2


def test_wave_count_on_device_context(ctx_f32):
    """Wave counts reported by the library on the device context equal the oracle's (bit-exact
    integers) in both capacity modes: 256 CUs, and 256 x the occupancy the HIP runtime reports."""
    from oracle import geometry as geo

    for cfg, res in all_configs(ctx_f32)[::3]:
        for (M, N, K) in [(16384, 8192, 8192), (4096, 11008, 4096), (333, 4096, 11008), (1, 4096, 4096)]:
            G, L = geo.phi_gemm(M, N, K, cfg.bm, cfg.bn, cfg.bk, cfg.split)
            assert wt.wt_wave_count(ctx_f32, M, N, K, cfg) == (G, L, geo.wave_count(G, geo.capacity(1)))
    wt.wt_set_capacity_mode(ctx_f32, wt.WT_CAP_CU_TIMES_OCC)
    for cfg, res in all_configs(ctx_f32)[::3]:
        G, L = geo.phi_gemm(4096, 11008, 4096, cfg.bm, cfg.bn, cfg.bk, cfg.split)
        assert wt.wt_wave_count(ctx_f32, 4096, 11008, 4096, cfg) == (G, L, geo.wave_count(G, geo.capacity(res.occ)))
    wt.wt_set_capacity_mode(ctx_f32, wt.WT_CAP_CU_ONLY)


# ---- sparse profiling on the device -> fit -> select, against the oracle at every step --------------------------
RT_W, RT_I, RT_P, RT_ANCHORS, RT_WSPLIT = 3, 2, 2, (1024, 2048), 2
RT_SLICES = ((15, 3), (61, 2))      # three unsplit keys and two split-K keys of the bf16 registry


@pytest.fixture(scope="module")
def device_records(ctx_bf16):
    """One reduced sparse profile on the GPU, shared by the model variants below: slices of the registry's keys,
    W = 3 waves (2 for split-K keys), I = 2, two K anchors, 1 warm-up + 2 timed launches."""
    out = []
    for (first, count) in RT_SLICES:
        grid = wt.make_grid(W=RT_W, I=RT_I, p=RT_P, k_anchors=RT_ANCHORS, warmup=1, iters=2, key_first=first,
                            key_count=count, W_split=RT_WSPLIT)
        n, bA, bB, bC = wt.wt_sample_plan(ctx_bf16, grid)
        scrA = torch.zeros(bA // 2, dtype=torch.bfloat16, device="cuda")
        scrB = torch.zeros(bB // 2, dtype=torch.bfloat16, device="cuda")
        scrC = torch.empty(bC, dtype=torch.uint8, device="cuda")
        note(f"profile_sparse keys {first}..{first + count - 1}, {n} records")
        recs = wt.wt_profile_sparse(ctx_bf16, grid, scrA, scrB, scrC, stream=torch.cuda.current_stream())
        assert len(recs) == n
        out.append(recs)
        del scrA, scrB, scrC
    return out


def test_device_records_are_the_oracles_plan(ctx_bf16, device_records):
    """Every record <key, micro, G, L, w, family> of wt_profile_sparse, in order, is what the oracle derives:
    sample_set (Eq. 3-4) x loop anchors x micros, instantiated by Eq. 5 so that Phi of the workload gives back
    (G, L); split-K keys over their own task counts and only W_split waves."""
    from _pins import split_limits
    from oracle import geometry as geo
    from oracle import sampler as smp

    lim = split_limits()
    for (first, count), recs in zip(RT_SLICES, device_records):
        want = []
        for k in range(first, first + count):
            cfg, res = wt.wt_config_get(ctx_bf16, 3 * k)
            assert res.key_id == k
            S = cfg.split
            W = RT_W if S == 1 else min(RT_W, RT_WSPLIT)
            for smpl in smp.sample_set(256, W, RT_I, S=S):
                if smpl.g == 0 or not geo.split_fits(smpl.m * cfg.bm, smpl.n * cfg.bn, cfg.bm, cfg.bn, S,
                                                     lim["ws_elems"], lim["max_split_tiles"]):
                    continue
                for L in smp.loop_anchors(RT_ANCHORS, cfg.bk, S):
                    M, N, K = smp.instantiate(smpl.m, smpl.n, L, cfg.bm, cfg.bn, cfg.bk, S)
                    assert geo.phi_gemm(M, N, K, cfg.bm, cfg.bn, cfg.bk, S) == (smpl.g, L)
                    assert geo.wave_count(smpl.g, 256) == smpl.w
                    want += [(k, m, smpl.g, L, smpl.w, 0) for m in range(3)]
        got = [(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"]), int(r["family"])) for r in recs]
        assert got == want
        assert np.all(recs["mean_us"] > 0) and np.isfinite(recs["mean_us"]).all()
    # more work takes longer: for one key and micro, the largest G*L is slower than the smallest
    r0 = device_records[0]
    r0 = r0[(r0["key_id"] == RT_SLICES[0][0]) & (r0["micro_id"] == 0)]
    assert r0["mean_us"][np.argmax(r0["G"] * r0["L"])] > r0["mean_us"][np.argmin(r0["G"] * r0["L"])]


@pytest.mark.parametrize("model,weighting", [(wt.WT_MODEL_WAVE_BILINEAR, 0), (wt.WT_MODEL_LINEAR, 0),
                                             (wt.WT_MODEL_STEP, 0), (wt.WT_MODEL_WAVE_BILINEAR, 1)])
def test_profile_fit_select_round_trip_on_device(ctx_bf16, tmp_path, device_records, model, weighting):
    """Device records -> wt_fit under each latency model (the method and its two ablations, Sec. 5.4; the method also
    with relative residuals, the objective of the shipped tables) -> wt_save; the table equals the oracle's fit of
    the same records (coefficients to 1e-9, status and anchors exactly), and the oracle's selector on the saved
    file returns exactly what wt_select returns, prediction included."""
    from _pins import lib_limits, split_limits
    from oracle import fit as ofit
    from oracle import select as osel

    recs = np.concatenate(device_records)
    grid = wt.make_grid(W=RT_W, I=RT_I, p=RT_P, k_anchors=RT_ANCHORS, W_split=RT_WSPLIT, model=model, weighting=weighting)
    wt.wt_fit(ctx_bf16, grid, recs)
    path = str(tmp_path / f"t{model}_{weighting}.wt")
    wt.wt_save(ctx_bf16, path)
    table, _ = osel.read_table(path, **split_limits())
    profiled = {k for (first, count) in RT_SLICES for k in range(first, first + count)}
    want = ofit.fit_tables([(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"]),
                             float(r["mean_us"])) for r in recs], table.keys, RT_W, RT_P, model=model,
                           max_anchors=lib_limits()["max_anchors"], relative=bool(weighting))
    n_fitted = 0
    for k in range(len(table.keys)):
        for got_b, want_b in list(zip(table.local[k], want.local[k])) + [(table.ext[k], want.ext[k])]:
            assert got_b.status == want_b.status, (k, model)
            assert (got_b.status != 0) <= (k in profiled)
            if not want_b.status:
                continue
            n_fitted += 1
            assert got_b.anchors == want_b.anchors
            # compare through predictions over the bucket's own range (coefficients cancel heavily)
            for (G, L) in ((1, 1), (256, 16), (700, 64), (2048, 160)):
                a, b = osel.predict(got_b.theta, G, L), osel.predict(want_b.theta, G, L)
                assert abs(a - b) <= 1e-9 * max(abs(b), max(abs(x) for x in want_b.theta)), (k, model, G, L, a, b)
    assert n_fitted >= len(profiled)
    picked = set()
    for (M, N, K) in wt_synth.sweep_shapes() + wt_synth.stream_shapes(300):
        key, micro, t = osel.select(table, M, N, K)
        c = wt.wt_select(ctx_bf16, M, N, K)
        kd = table.keys[key]
        assert (c.bm, c.bn, c.bk, c.nwave, c.stages, c.swizzle, c.split) == (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, micro, kd.split)
        assert wt.wt_predict_us(ctx_bf16, M, N, K, c) == t      # the same bits
        assert key in profiled
        picked.add(key)
    assert len(picked) >= 2


def test_row_band_families_profile_fit_select_on_device(ctx_bf16, tmp_path, device_records):
    """The row-band few-row families end to end on the GPU: wt_profile_sparse with row_mode = WT_ROWS_BAND profiles, for
    two families, matrices of exactly 16 and 32 rows under every key of the slice; the records are the oracle's plan
    (band_sample_set x loop anchors x micros, family tagged, Phi of the 16- or 32-row workload giving back G and L);
    fitted together with the near-square records the table file is version 4 and equals the oracle's fit; shapes with
    M <= 32 are then priced from the family of their band under every key alike, bit for bit as the oracle prices them."""
    from _pins import lib_limits, split_limits
    from oracle import fit as ofit
    from oracle import geometry as geo
    from oracle import sampler as smp
    from oracle import select as osel

    W_row, fams = 2, 2
    lim = split_limits()
    band_recs = []
    for (first, count) in RT_SLICES:
        grid = wt.make_grid(W=RT_W, I=RT_I, p=RT_P, k_anchors=RT_ANCHORS, warmup=1, iters=2, key_first=first, key_count=count,
                            W_split=RT_WSPLIT, W_row=W_row, row_fams=fams, row_mode=wt.WT_ROWS_BAND, skip_near=1)
        n, bA, bB, bC = wt.wt_sample_plan(ctx_bf16, grid)
        scrA = torch.zeros(bA // 2, dtype=torch.bfloat16, device="cuda")
        scrB = torch.zeros(bB // 2, dtype=torch.bfloat16, device="cuda")
        scrC = torch.empty(bC, dtype=torch.uint8, device="cuda")
        note(f"profile_sparse row-band families keys {first}..{first + count - 1}, {n} records")
        recs = wt.wt_profile_sparse(ctx_bf16, grid, scrA, scrB, scrC, stream=torch.cuda.current_stream())
        assert len(recs) == n
        want = []
        for k in range(first, first + count):
            cfg, _ = wt.wt_config_get(ctx_bf16, 3 * k)
            S = cfg.split
            Wk = W_row if S == 1 else min(W_row, RT_WSPLIT)
            for f in range(1, fams + 1):
                rows = smp.ROW_BANDS[f - 1]
                for smpl in smp.band_sample_set(256, Wk, RT_I, rows, cfg.bm, S):
                    if smpl.g == 0 or not geo.split_fits(smpl.m * cfg.bm, smpl.n * cfg.bn, cfg.bm, cfg.bn, S,
                                                         lim["ws_elems"], lim["max_split_tiles"]):
                        continue
                    for L in smp.loop_anchors(RT_ANCHORS, cfg.bk, S):
                        assert geo.phi_gemm(rows, smpl.n * cfg.bn, L * S * cfg.bk, cfg.bm, cfg.bn, cfg.bk, S) == (smpl.g, L)
                        want += [(k, m, smpl.g, L, smpl.w, f) for m in range(3)]
        got = [(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"]), int(r["family"])) for r in recs]
        assert got == want
        assert np.all(recs["mean_us"] > 0) and np.isfinite(recs["mean_us"]).all()
        band_recs.append(recs)
        del scrA, scrB, scrC
    recs = np.concatenate(list(device_records) + band_recs)
    grid = wt.make_grid(W=RT_W, I=RT_I, p=RT_P, k_anchors=RT_ANCHORS, W_split=RT_WSPLIT, W_row=W_row, row_fams=fams,
                        row_mode=wt.WT_ROWS_BAND, weighting=1)
    wt.wt_fit(ctx_bf16, grid, recs)
    path = str(tmp_path / "bands.wt")
    wt.wt_save(ctx_bf16, path)
    assert open(path, "rb").read()[4] == 4
    table, _ = osel.read_table(path, **lim)
    assert (table.W_row, table.row_fams, table.row_mode) == (W_row, fams, 1)
    want_t = ofit.fit_tables([(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"]),
                               float(r["mean_us"]), int(r["family"])) for r in recs], table.keys, RT_W, RT_P, W_row=W_row,
                             row_fams=fams, row_mode=1, max_anchors=lib_limits()["max_anchors"], relative=True)
    profiled = {k for (first, count) in RT_SLICES for k in range(first, first + count)}
    n_fitted = 0
    for k in profiled:
        for f in range(fams):
            for got_b, want_b in list(zip(table.row_local[f][k], want_t.row_local[f][k])) + [(table.row_ext[f][k], want_t.row_ext[f][k])]:
                assert got_b.status == want_b.status and got_b.anchors == want_b.anchors, (k, f)
                if not want_b.status:
                    continue
                n_fitted += 1
                for (G, L) in ((1, 1), (256, 16), (500, 32)):
                    a, b = osel.predict(got_b.theta, G, L), osel.predict(want_b.theta, G, L)
                    assert abs(a - b) <= 1e-9 * max(abs(b), max(abs(x) for x in want_b.theta)), (k, f, G, L, a, b)
    assert n_fitted >= 2 * len(profiled)
    used = {0: 0, 1: 0, 2: 0, 3: 0, 4: 0}
    for (M, N, K) in wt_synth.sweep_shapes() + wt_synth.stream_shapes(300):
        key, micro, t = osel.select(table, M, N, K)
        c = wt.wt_select(ctx_bf16, M, N, K)
        kd = table.keys[key]
        assert (c.bm, c.bn, c.bk, c.nwave, c.stages, c.swizzle, c.split) == (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, micro, kd.split)
        assert wt.wt_predict_us(ctx_bf16, M, N, K, c) == t
        used[osel.family_of(table, M, kd.bm)] += 1
    assert used[1] > 10 and used[2] > 5 and used[0] > 50
