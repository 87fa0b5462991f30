"""Time one configuration on one shape through the C ABI (also the program profiled under rocprofv3).

    python -m paper_2604_10187_amd.run_one M N K bm bn bk nwave stages swizzle [iters] [in_type] [out_type] [split]

in_type 0 = bf16, 1 = fp8 e4m3; out_type 0 = f32, 1 = bf16; split = blocks per output tile along K (default 1).  N(0,1) operands (fp8: per-tensor scales).

    python -m paper_2604_10187_amd.run_one copy [MiB]

runs three plain device-to-device copies of MiB mebibytes (default 1024) and nothing else: the dispatch of known
size against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled.
"""
import sys

import torch

from . import binding as wt


def copy_of_known_size(mib):
    n = mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)          # one copy kernel per call: reads n*4 bytes, writes n*4 bytes
    torch.cuda.synchronize()
    print(f"copied {n * 4} bytes per dispatch (read) and the same written; 3 dispatches", flush=True)


def main(argv=None):
    argv = list(argv or sys.argv[1:])
    if argv and argv[0] == "copy":
        return copy_of_known_size(int(argv[1]) if len(argv) > 1 else 1024)
    a = [int(x) for x in argv]
    if len(a) < 9:
        print(__doc__)
        sys.exit(2)
    M, N, K, bm, bn, bk, nw, st, sw = a[:9]
    iters = a[9] if len(a) > 9 else 5
    it = a[10] if len(a) > 10 else wt.WT_BF16
    ot = a[11] if len(a) > 11 else wt.WT_OUT_BF16
    split = a[12] if len(a) > 12 else 1
    ctx = wt.wt_create(0, it, ot)
    cfg, res = wt.wt_config_get(ctx, wt.wt_config_find(ctx, bm, bn, bk, nw, st, sw, split))
    A = torch.randn(M, K, device="cuda")
    B = torch.randn(N, K, device="cuda")
    sA = sB = None
    if it == wt.WT_BF16:
        A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)
    else:
        sa, sb = A.abs().max() / 448.0, B.abs().max() / 448.0
        A, B = (A / sa).to(torch.float8_e4m3fn), (B / sb).to(torch.float8_e4m3fn)
        sA, sB = sa.reshape(1).float(), sb.reshape(1).float()
    C = torch.empty(M, N, device="cuda", dtype=torch.bfloat16 if ot == wt.WT_OUT_BF16 else torch.float32)
    us = wt.wt_time_gemm(ctx, M, N, K, A, B, C, cfg, 2, iters, sA, sB, torch.cuda.current_stream())
    esz, osz = (2 if it == wt.WT_BF16 else 1), (2 if ot == wt.WT_OUT_BF16 else 4)
    gbs = (esz * (M * K + N * K) + osz * M * N) / us / 1e3
    print(f"{M}x{N}x{K} cfg={cfg.astuple()} occ={res.occ} regs={res.vgprs} lds={res.lds_bytes}: {us:.1f} us  "
          f"{2 * M * N * K / us / 1e6:.1f} TFLOP/s  {gbs:.0f} GB/s algorithmic", flush=True)
    wt.wt_destroy(ctx)


if __name__ == "__main__":
    main()
