"""Offline stage: wave-aware sparse profiling on the GPU, fit, and dual-table file (Sec. 4.2-4.5).

    python -m paper_2604_10187_amd.tune --out tables/mi355x_in0_out1.wt [--W 40 --I 4 ...]
        [--key-first a --key-count n --samples-out file.npy]      # profile a slice of keys only
        [--fit-from a.npy b.npy ...] [--records-out r.npz]        # fit saved records, no GPU

Every step runs inside libwt (wt_profile_sparse, wt_fit, wt_save); this script only allocates the
scratch buffers with torch and moves records between files.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np

from . import binding as wt

TABLE_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tables")
# The paper's five K anchors spanning [1024, 5120] (Sec. 5.1) plus K = 8192: the workloads here reach
# K = 8192..28672, and rows whose stride is a large power of two behave differently in HBM (channel
# aliasing makes the rasterisation mode matter), which no anchor below 8192 shows.
K_ANCHORS = (1024, 2048, 3072, 4096, 5120, 8192)
# Second profiling pass of the shipped GEMM tables: two long-K anchors for the first waves only
# (`--W 12 --k-anchors 16384 28672`, records merged with the first pass by --fit-from).  The serving shapes reach
# K = 28672, 3.5 times beyond the last anchor above; up to 12 waves a bucket then holds eight loop anchors and is
# interpolated in L instead of extrapolated.  Deeper waves of such K would take hours to profile and keep six.
K_ANCHORS_LONG = (16384, 28672)
W_LONG = 12
# Third pass of the shipped GEMM tables: two short-K anchors over the same first waves (`--W 12 --k-anchors 256 512`,
# a few seconds of GPU time).  Below K = 1024 a launch is mostly fixed cost, which no plane through the anchors
# above shows: extrapolated downwards they predict a fraction of a microsecond, or less than nothing, for launches
# that take three.  With anchors from 256 to 28672 a bucket's latencies span two orders of magnitude, so the shipped
# tables are fitted with relative residuals (`--weighting 1`, WT_FIT_RELATIVE).
K_ANCHORS_SHORT = (256, 512)
# Fourth pass of the shipped bf16 table: the 16-row family (`--W-row 8 --row-fams 1 --row-mode 1 --skip-near` with all
# ten anchors above): matrices of exactly 16 rows under every key, eight waves wide.  Shapes with M <= 16 have one tile
# row under every key, their B operand streams from HBM once, and near-square samples of the same G price them 2-3
# times too fast and rank the keys by noise; the family prices every key from the same skinny matrices.
K_ANCHORS_ALL = K_ANCHORS_SHORT + K_ANCHORS + K_ANCHORS_LONG
# Attention contexts: KV-length multipliers of S_q in percent (Sec. 5.1: 1.0 to 3.0).
KV_MULTIPLIERS = (100, 150, 200, 250, 300)


def table_path(in_type: int, out_type: int) -> str:
    if in_type == wt.WT_ATTN_BF16:
        return os.path.join(TABLE_DIR, "mi355x_attn.wt")
    return os.path.join(TABLE_DIR, f"mi355x_in{in_type}_out{out_type}.wt")


def profile(ctx, grid, in_type, out_type, log=print, chunk_keys=1):
    """Run wt_profile_sparse over the grid's key slice in chunks; returns the records."""
    import torch

    nkeys = wt.wt_key_count(ctx)
    first = grid.key_first if grid.key_count > 0 else 0
    count = grid.key_count if grid.key_count > 0 else nkeys
    _, bA, bB, bC = wt.wt_sample_plan(ctx, grid)
    esz = 1 if in_type == wt.WT_FP8_E4M3 else 2
    # finite, non-constant contents; values do not influence timing of dense MFMA work
    scrA = (torch.randn(max(bA // esz, 16), device="cuda") * 0.5).to(torch.bfloat16 if esz == 2 else torch.float8_e4m3fn)
    scrB = (torch.randn(max(bB // esz, 16), device="cuda") * 0.5).to(torch.bfloat16 if esz == 2 else torch.float8_e4m3fn)
    scrC = torch.empty(max(bC, 16), dtype=torch.uint8, device="cuda")
    out = []
    t0 = time.time()
    for k0 in range(first, first + count, chunk_keys):
        kc = min(chunk_keys, first + count - k0)
        g = wt.make_grid(W=grid.W, I=grid.I, tau=(grid.tau_num, grid.tau_den), p=grid.p,
                         k_anchors=[grid.k_anchors[j] for j in range(grid.n_k_anchors)], warmup=grid.warmup,
                         iters=grid.iters, key_first=k0, key_count=kc, max_out_elems=grid.max_out_elems, model=grid.model, W_row=grid.W_row,
                         W_split=grid.W_split, row_fams=grid.row_fams, skip_near=grid.skip_near, n_heads=grid.n_heads,
                         weighting=grid.weighting, row_mode=grid.row_mode)
        recs = wt.wt_profile_sparse(ctx, g, scrA, scrB, scrC, stream=torch.cuda.current_stream())
        out.append(recs)
        log(f"[tune] keys {k0}..{k0 + kc - 1}: {len(recs)} records, {time.time() - t0:.0f}s elapsed")
    return np.concatenate(out) if out else np.zeros(0, dtype=wt.SAMPLE_DTYPE)


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--in-type", type=int, default=wt.WT_BF16)
    ap.add_argument("--out-type", type=int, default=wt.WT_OUT_BF16)
    ap.add_argument("--W", type=int, default=40)
    ap.add_argument("--I", type=int, default=4)
    ap.add_argument("--p", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--k-anchors", type=int, nargs="+", default=None,
                    help="GEMM: K values of the loop anchors; attention: KV-length multipliers in percent of S_q")
    ap.add_argument("--n-heads", type=int, nargs="+", default=[32],
                    help="attention contexts: head counts to profile (records of all of them are fitted together)")
    ap.add_argument("--key-first", type=int, default=0)
    ap.add_argument("--key-count", type=int, default=0)
    ap.add_argument("--max-out-elems", type=int, default=0)
    ap.add_argument("--cap-mode", type=int, default=1, help="1: 256 CUs (the paper's wave count), 0: 256 x resident blocks per CU")
    ap.add_argument("--model", type=int, default=0, help="0 wave-bilinear, 1 linear, 2 step")
    ap.add_argument("--W-row", type=int, default=0, help="extension: waves of single-tile-row grids to profile/fit (0 = off)")
    ap.add_argument("--row-fams", type=int, default=1, help="extension: few-row families to profile/fit when --W-row > 0 (1..3: 1, 2, 4 tile rows)")
    ap.add_argument("--row-mode", type=int, default=0, help="few-row families: 0 grids of 1/2/4 tile rows, 1 grids of 16/32/64/128 rows under every key")
    ap.add_argument("--skip-near", action="store_true", help="profile only the few-row families (records are merged by --fit-from)")
    ap.add_argument("--weighting", type=int, default=0,
                    help="objective of the bucket fits: 0 ordinary least squares (the paper as written), 1 relative residuals")
    ap.add_argument("--W-split", type=int, default=8, help="split-K keys are profiled for the first W-split waves only (0 = all)")
    ap.add_argument("--samples-out", default=None)
    ap.add_argument("--fit-from", nargs="*", default=None)
    ap.add_argument("--records-out", default=None,
                    help="with --out: also write the fitted records and the keys' occupancy as one compressed .npz "
                         "(arrays `samples`, `occ`), the form kept beside the shipped tables")
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    attn = a.in_type == wt.WT_ATTN_BF16
    if a.k_anchors is None:
        a.k_anchors = list(KV_MULTIPLIERS if attn else K_ANCHORS)
    grid = wt.make_grid(W=a.W, I=a.I, p=a.p, k_anchors=a.k_anchors, warmup=a.warmup, iters=a.iters,
                        key_first=a.key_first, key_count=a.key_count, max_out_elems=a.max_out_elems, model=a.model, W_row=a.W_row,
                        W_split=a.W_split, row_fams=a.row_fams, skip_near=int(a.skip_near),
                        n_heads=a.n_heads[0] if attn else 0, weighting=a.weighting, row_mode=a.row_mode)
    if a.fit_from is not None:
        recs = np.concatenate([np.load(f) for f in a.fit_from])
        occ_files = [f.replace(".npy", ".occ.npy") for f in a.fit_from]
        ctx = wt.wt_create(-1, a.in_type, a.out_type)
        wt.wt_set_capacity_mode(ctx, a.cap_mode)
        if all(os.path.exists(f) for f in occ_files):    # wave boundaries = those of the profiling run
            occ = np.load(occ_files[0])
            for k, o in enumerate(occ):
                wt.wt_key_set_occ(ctx, k, int(o))
    else:
        ctx = wt.wt_create(0, a.in_type, a.out_type)
        wt.wt_set_capacity_mode(ctx, a.cap_mode)
        parts = []
        for nh in (a.n_heads if attn else [0]):
            grid.n_heads = nh
            n, bA, bB, bC = wt.wt_sample_plan(ctx, grid)
            print(f"[tune] plan{f' ({nh} heads)' if attn else ''}: {n} records, scratch A {bA >> 20} MiB, B {bB >> 20} MiB, "
                  f"C {bC >> 20} MiB", flush=True)
            parts.append(profile(ctx, grid, a.in_type, a.out_type, log=lambda s: print(s, flush=True)))
        recs = np.concatenate(parts)
        if a.samples_out:
            np.save(a.samples_out, recs)
            occ = np.array([wt.wt_config_get(ctx, 3 * k)[1].occ for k in range(wt.wt_key_count(ctx))], dtype=np.int32)
            np.save(a.samples_out.replace(".npy", ".occ.npy"), occ)
    if a.out:
        wt.wt_fit(ctx, grid, recs)
        os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
        wt.wt_save(ctx, a.out)
        print(f"[tune] fitted {len(recs)} records -> {a.out} ({os.path.getsize(a.out)} bytes)")
        if a.records_out:
            occ = np.array([wt.wt_config_get(ctx, 3 * k)[1].occ for k in range(wt.wt_key_count(ctx))], dtype=np.int32)
            np.savez_compressed(a.records_out, samples=recs, occ=occ)
    wt.wt_destroy(ctx)


if __name__ == "__main__":
    main()
