"""Time one attention configuration on one shape through the C ABI (also the program profiled under rocprofv3).

    python -m paper_2604_10187_amd.run_attn S_q S_kv H_q H_kv T_Q T_KV nwave stages order [causal] [iters]

bf16 N(0,1) operands, scale 1/sqrt(128).  Prints mean microseconds and TFLOP/s (4*S_q*S_kv*128*H_q flop, halved
when causal).
"""
import math
import sys

import torch

from . import binding as wt


def main(argv=None):
    a = [int(x) for x in (argv or sys.argv[1:])]
    if len(a) < 9:
        print(__doc__)
        sys.exit(2)
    S_q, S_kv, H_q, H_kv, tq, tkv, nw, st, order = a[:9]
    causal = a[9] if len(a) > 9 else 0
    iters = a[10] if len(a) > 10 else 5
    ctx = wt.wt_create(0, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    cfg, res = wt.wt_config_get(ctx, wt.wt_config_find(ctx, tq, 1, tkv, nw, st, order))
    Q = torch.randn(S_q * H_q, 128, device="cuda").to(torch.bfloat16)
    K = torch.randn(S_kv * H_kv, 128, device="cuda").to(torch.bfloat16)
    V = torch.randn(S_kv * H_kv, 128, device="cuda").to(torch.bfloat16)
    O = torch.empty_like(Q)
    us = wt.wt_time_attn(ctx, H_q, H_kv, S_q, S_kv, Q, K, V, O, 1.0 / math.sqrt(128.0), causal, cfg, 2, iters,
                         torch.cuda.current_stream())
    flop = 4.0 * S_q * S_kv * 128 * H_q * (0.5 if causal else 1.0)
    print(f"attn S_q={S_q} S_kv={S_kv} H={H_q}/{H_kv} cfg={cfg.astuple()} occ={res.occ} regs={res.vgprs} "
          f"lds={res.lds_bytes} causal={causal}: {us:.1f} us  {flop / us / 1e6:.1f} TFLOP/s", flush=True)
    wt.wt_destroy(ctx)


if __name__ == "__main__":
    main()
