"""A plain device-to-device copy of known size, for calibrating rocprofv3's FETCH_SIZE / WRITE_SIZE
counters: run it under `rocprofv3 --pmc FETCH_SIZE` (then WRITE_SIZE) and divide the known byte
count by what the counter reads for the copy kernel's dispatch.

    python -m paper_2604_10187_amd.copy_probe [MiB]
"""
import sys

import torch


def main():
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 1024
    n = mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)          # one elementwise copy kernel: reads n*4 bytes, writes n*4 bytes
    torch.cuda.synchronize()
    print(f"copied {n * 4} bytes per dispatch (read) and the same written; 3 dispatches")


if __name__ == "__main__":
    main()
