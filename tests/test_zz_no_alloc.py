"""GPU: wt_gemm_noalloc (split-K partial tiles in the library's static device array) against wt_gemm (partial
tiles in the context's workspace) and against the CPU oracle, through the C ABI.

Both entry points run the same kernels and add the S partial tiles in split order, so their outputs must agree
bit for bit; each case makes two calls in a row on the shared array, the second on a smaller input, so that
whatever the first call left behind (partial tiles, counters) is there when the second one starts."""
import numpy as np
import pytest
import torch

import paper_2604_10187_amd as wt
import wt_synth
from gpu_util import dev_bits, note
from oracle import gemm as og

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctxs():
    a = wt.wt_create(0, wt.WT_BF16, wt.WT_OUT_F32)
    b = wt.wt_create(0, wt.WT_BF16, wt.WT_OUT_BF16)
    yield a, b
    wt.wt_destroy(a)
    wt.wt_destroy(b)


def _both(ctx, cfg, ab, bb, out_dtype):
    M, K = ab.shape
    N = bb.shape[0]
    dA, dB = dev_bits(ab), dev_bits(bb)
    ref = torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda")
    got = torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda")
    s = torch.cuda.current_stream()
    wt.wt_gemm(ctx, M, N, K, dA, dB, ref, cfg, stream=s)
    wt.wt_gemm_noalloc(ctx, M, N, K, dA, dB, got, cfg, stream=s)
    torch.cuda.synchronize()
    return got, ref


# (bm, bn, bk, nwave, stages, split): split-K keys of the bf16 registry with S = 2, 4, 8, and one unsplit key
KEYS = ((64, 64, 128, 4, 3, 2), (128, 256, 64, 4, 3, 4), (64, 64, 128, 4, 3, 8), (16, 64, 256, 4, 3, 4),
        (256, 256, 64, 8, 2, 2), (128, 128, 64, 4, 3, 1))


@pytest.mark.parametrize("fields", KEYS)
def test_two_calls_in_a_row_match_wt_gemm_and_the_oracle(ctxs, fields):
    ctx_f32, ctx_bf16 = ctxs
    bm, bn, bk, nw, st, S = fields
    for sw in (0, 2):
        cfg, _ = wt.wt_config_get(ctx_f32, wt.wt_config_find(ctx_f32, bm, bn, bk, nw, st, sw, S))
        # first call: several tiles, ragged edges, a K that leaves the last split short; second call: smaller
        shapes = ((3 * bm + 17, 2 * bn + 33, 5 * S * bk + 24), (bm + 5, bn - 7, 2 * S * bk + 8))
        for call, (M, N, K) in enumerate(shapes):
            note(f"noalloc cfg={cfg.astuple()} call {call} shape={(M, N, K)} int")
            a32, b32 = wt_synth.gemm_operands(M, N, K, 4000 + 7 * call + S, "int")
            ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)
            got, ref = _both(ctx_f32, cfg, ab, bb, torch.float32)
            assert torch.equal(got, ref), f"{cfg} call {call}: differs from wt_gemm"
            assert np.array_equal(got.cpu().numpy(), og.gemm_c(ab, bb)), f"{cfg} call {call}: differs from the oracle"
    # N(0,1) operands, bf16 out: still the same bits as wt_gemm, and within the per-element bound of the oracle
    cfg, _ = wt.wt_config_get(ctx_bf16, wt.wt_config_find(ctx_bf16, bm, bn, bk, nw, st, 1, S))
    for call, (M, N, K) in enumerate(((2 * bm + 9, 3 * bn + 1, 6 * S * bk), (bm, bn, S * bk + 8))):
        note(f"noalloc cfg={cfg.astuple()} call {call} shape={(M, N, K)} normal bf16-out")
        a32, b32 = wt_synth.gemm_operands(M, N, K, 4100 + call + S, "normal")
        ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)
        got, ref = _both(ctx_bf16, cfg, ab, bb, torch.bfloat16)
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        assert og.max_scaled_err(got.float().cpu().numpy(), og.gemm_c(ab, bb)) <= 2e-2


def test_serving_shape_large_first_then_small(ctxs):
    """A shape split-K is selected for in serving (few rows, long K) at full size, then a small one, each against
    wt_gemm bit for bit and on sampled rows against the oracle."""
    _, ctx = ctxs
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 128, 128, 64, 4, 3, 2, 8))
    for call, (M, N, K) in enumerate(((256, 8192, 28672), (100, 640, 4096))):
        note(f"noalloc serving cfg={cfg.astuple()} call {call} shape={(M, N, K)}")
        a32, b32 = wt_synth.gemm_operands(M, N, K, 4200 + call, "normal")
        ab, bb = wt_synth.to_bf16_bits(a32), wt_synth.to_bf16_bits(b32)
        got, ref = _both(ctx, cfg, ab, bb, torch.bfloat16)
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        rows = sorted({0, 1, M // 2, M - 1})
        want = og.gemm_c(ab[rows], bb)
        assert og.max_scaled_err(got.float().cpu().numpy()[rows], want) <= 2e-2


def test_sizes_beyond_the_static_array_are_refused(ctxs):
    """Host-side check only: nothing is launched for a shape whose partial tiles exceed the array."""
    _, ctx = ctxs
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 128, 128, 64, 4, 3, 0, 8))
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")      # never read: the call fails before any launch
    # 128 tiles of 128x128 split in 8 fill the array exactly (2^24 floats); 3 x 43 = 129 tiles do not fit
    assert 128 * 8 * 128 * 128 == wt.WT_NOALLOC_WS_FLOATS
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm_noalloc(ctx, 128 * 3, 128 * 43, 4096, t, t, t, cfg)
    assert e.value.status == wt.WT_ERR_INFEASIBLE
    # more output tiles than counters: 16x16 tiles, split 2
    small, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 16, 16, 256, 1, 4, 0, 2))
    with pytest.raises(wt.WtError) as e:
        wt.wt_gemm_noalloc(ctx, 16 * 256, 16 * 129, 4096, t, t, t, small)
    assert e.value.status == wt.WT_ERR_INFEASIBLE
    torch.cuda.synchronize()


def test_capture_and_replay(ctxs):
    """The use the entry point is for: captured into a HIP graph (counter reset included -- a kernel, not a memset
    node) and replayed several times with eager work between the replays, each replay bit-identical to wt_gemm."""
    _, ctx = ctxs
    cfg, _ = wt.wt_config_get(ctx, wt.wt_config_find(ctx, 64, 64, 128, 4, 3, 1, 4))
    M, N, K = 200, 700, 4104
    a32, b32 = wt_synth.gemm_operands(M, N, K, 4300, "normal")
    dA, dB = dev_bits(wt_synth.to_bf16_bits(a32)), dev_bits(wt_synth.to_bf16_bits(b32))
    ref = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(ref)
    wt.wt_gemm(ctx, M, N, K, dA, dB, ref, cfg, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    cur = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    side.wait_stream(cur)
    with torch.cuda.stream(side):
        wt.wt_gemm_noalloc(ctx, M, N, K, dA, dB, out, cfg, stream=side)
    cur.wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        wt.wt_gemm_noalloc(ctx, M, N, K, dA, dB, out, cfg, stream=torch.cuda.current_stream())
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), f"replay {rep}"
        small = torch.empty((64, 64), dtype=torch.bfloat16, device="cuda")   # eager split-K work on the same array
        wt.wt_gemm_noalloc(ctx, 64, 64, 1024, dA, dB, small, cfg, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
