"""GPU parity: wt_gemm (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2604_10187_amd as wt
import wt_synth
from gpu_util import all_configs, note, run_gemm
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
    bad = wt.wt_cfg(100, 100, 64, 4, 2, 0, -1)
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx_f32, 4, 8, 16, dA, dA, dC, bad, stream=stream)
    assert e.value.status == wt.WT_ERR_UNSUPPORTED_CFG
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm(ctx_f32, 4, 8, 16, None, dA, dC, cfg, stream=stream)
    assert e.value.status == wt.WT_ERR_INVALID_ARG
