"""Helpers for the GPU parity tests: device buffers via torch, calls through the C ABI binding."""
import sys

import numpy as np
import torch

import paper_2604_10187_amd as wt


def note(msg):
    """Name the case before touching the GPU, so a fault can be traced to it."""
    print(msg, flush=True)
    sys.stdout.flush()


def dev_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 (bf16) or uint8 (e4m3) storage bits -> device tensor holding the same bytes."""
    if bits.dtype == np.uint16:
        return torch.from_numpy(bits.view(np.int16).copy()).cuda()
    return torch.from_numpy(bits.copy()).cuda()


def run_gemm(ctx, cfg, a_bits, b_bits, out_type, scale_a=None, scale_b=None, fill=None):
    """Launch wt_gemm on storage-encoded operands; returns C as a numpy array (fp32 values)."""
    M, K = a_bits.shape
    N = b_bits.shape[0]
    dA, dB = dev_bits(a_bits), dev_bits(b_bits)
    dt = torch.float32 if out_type == wt.WT_OUT_F32 else torch.bfloat16
    dC = torch.empty((M, N), dtype=dt, device="cuda")
    if fill is not None:
        dC.fill_(fill)
    sA = torch.tensor([scale_a], dtype=torch.float32, device="cuda") if scale_a is not None else None
    sB = torch.tensor([scale_b], dtype=torch.float32, device="cuda") if scale_b is not None else None
    torch.cuda.synchronize()
    wt.wt_gemm(ctx, M, N, K, dA, dB, dC, cfg, sA, sB, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    return dC.float().cpu().numpy()


def run_gemm_grouped(ctx, cfg, a_bits, b_bits, offsets, out_type, fill=None):
    """Launch wt_gemm_grouped; a_bits [M_total, K], b_bits [E, N, K], offsets int32 [E+1] (copied to the GPU)."""
    M, K = a_bits.shape
    E, N, _ = b_bits.shape
    dA, dB = dev_bits(a_bits), dev_bits(b_bits.reshape(E * N, K))
    dOff = torch.from_numpy(np.asarray(offsets, dtype=np.int32).copy()).cuda()
    dt = torch.float32 if out_type == wt.WT_OUT_F32 else torch.bfloat16
    dC = torch.empty((M, N), dtype=dt, device="cuda")
    if fill is not None:
        dC.fill_(fill)
    torch.cuda.synchronize()
    wt.wt_gemm_grouped(ctx, E, dOff, M, N, K, dA, dB, dC, cfg, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    return dC.float().cpu().numpy()


def all_configs(ctx):
    return [wt.wt_config_get(ctx, i) for i in range(wt.wt_config_count(ctx))]
