"""Measurement harness for the synthetic workloads (every GPU step goes through libwt's C ABI).

    python -m paper_2604_10187_amd.evaluate sweep   [--table T] [--out F]   # LLM-projection sweep, 27 shapes
    python -m paper_2604_10187_amd.evaluate wave    [--table T] [--out F]   # M=K=4096, N=128..16384 step 128
    python -m paper_2604_10187_amd.evaluate stream  [--table T] [--out F] [--sample 300]  # 10,000-shape stream
    python -m paper_2604_10187_amd.evaluate large   [--out F]               # 16384x8192x8192 bf16 and fp8
    python -m paper_2604_10187_amd.evaluate attn    [--table T] [--out F] [--sample 48] [--causal]  # attention test set
    python -m paper_2604_10187_amd.evaluate shapes  --set paper|shortk      # shapes in the paper's test ranges / K = 256..2048
    python -m paper_2604_10187_amd.evaluate attn_varlen [--sample 20]       # ragged causal prefill batches (wt_attn_varlen)
    python -m paper_2604_10187_amd.evaluate grouped|persistent|vendor|ablate ...   # see each command's docstring
    (sweep --rotate-mb 1200: every launch on another copy of the weight, so that weights stream from HBM)

"pick" = the configuration wt_select returns; "best" = exhaustive search over the frozen registry
with the same timing protocol (3 warm-up + 5 measured launches, mean; Sec. 4.2).  The pick's time is
read from the exhaustive sweep itself, so the ratio best/pick is <= 1 by construction.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

from . import binding as wt
from . import tune


def _log(*a):
    print(*a, file=sys.stderr, flush=True)


def _dev_operands(torch, M, N, K, in_type, out_type, seed=0):
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 + seed)
    A = torch.randn((M, K), device="cuda", generator=g)
    B = torch.randn((N, K), device="cuda", generator=g)
    if in_type == wt.WT_BF16:
        A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)
        sA = sB = None
    else:
        sa, sb = A.abs().max() / 448.0, B.abs().max() / 448.0
        A, B = (A / sa).to(torch.float8_e4m3fn), (B / sb).to(torch.float8_e4m3fn)
        sA, sB = sa.reshape(1).float(), sb.reshape(1).float()
    C = torch.empty((M, N), device="cuda", dtype=torch.float32 if out_type == wt.WT_OUT_F32 else torch.bfloat16)
    return A, B, C, sA, sB


class Exhaustive:
    """Times every configuration of the registry on one shape; prunes a configuration after one
    timed launch if it is more than `prune` times slower than the best so far."""

    def __init__(self, ctx, torch, in_type, out_type, prune=2.5, warmup=3, iters=5, refine=0, rotate_mb=0):
        self.ctx, self.torch, self.in_type, self.out_type = ctx, torch, in_type, out_type
        self.prune, self.warmup, self.iters, self.refine = prune, warmup, iters, refine
        # rotate_mb > 0: every launch reads another copy of the weight B, the copies adding up to at least rotate_mb
        # megabytes (more than the 256 MB memory-side cache), so that B streams from HBM as the weights of consecutive
        # layers would; launches are then timed from here with events on the launch stream, `iters` rounds over the copies
        self.rotate_mb = rotate_mb
        self.first_pass = {}
        self.cfgs = [wt.wt_config_get(ctx, i) for i in range(wt.wt_config_count(ctx))]
        self.stream = torch.cuda.current_stream()
        self.launches = 0
        self.gpu_s = 0.0

    @staticmethod
    def runnable(c, M, N):
        """Split-K configurations need their partial tiles to fit the context's workspace (wt_gemm refuses
        the launch otherwise): 2^26 floats and at most 2^16 tiles."""
        tiles = -(-M // c.bm) * -(-N // c.bn)
        return c.split == 1 or (tiles <= (1 << 16) and tiles * c.split * c.bm * c.bn <= (1 << 26))

    def _timer(self, M, N, K, A, B, C, sA, sB):
        """time(cfg, warmup, iters) -> mean microseconds per launch, under the protocol in force."""
        if self.rotate_mb <= 0:
            return lambda c, warmup, iters: wt.wt_time_gemm(self.ctx, M, N, K, A, B, C, c, warmup, iters, sA, sB, self.stream)
        torch = self.torch
        n = max(2, -(-self.rotate_mb * 1000000 // (B.numel() * B.element_size())))
        copies = [B] + [B.clone() for _ in range(n - 1)]

        def timed(c, warmup, iters):
            for i in range(min(warmup, 1) * n):
                wt.wt_gemm(self.ctx, M, N, K, A, copies[i % n], C, c, sA, sB, stream=self.stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)
            for i in range(iters * n):
                wt.wt_gemm(self.ctx, M, N, K, A, copies[i % n], C, c, sA, sB, stream=self.stream)
            e1.record(self.stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / (iters * n)
        return timed

    def run(self, M, N, K, must=()):
        A, B, C, sA, sB = _dev_operands(self.torch, M, N, K, self.in_type, self.out_type)
        time_cfg = self._timer(M, N, K, A, B, C, sA, sB)
        times, best = {}, math.inf
        order = sorted(range(len(self.cfgs)), key=lambda i: i not in must)
        for i in order:
            c, r = self.cfgs[i]
            if r.occ < 1 or not self.runnable(c, M, N):
                continue
            if i not in must and best < math.inf:
                t1 = time_cfg(c, 1, 1)
                self.launches += 2
                self.gpu_s += 2 * t1 * 1e-6
                if t1 > self.prune * best:
                    continue
            t = time_cfg(c, self.warmup, self.iters)
            self.launches += self.warmup + self.iters
            self.gpu_s += (self.warmup + self.iters) * t * 1e-6
            times[i] = t
            best = min(best, t)
        # One 3+5 measurement has a few per cent of scatter (clock state, neighbours in the timing order), and the
        # search takes the minimum over up to 240 of them.  With refine > 0 the `refine` fastest configurations and
        # the ones in `must` are measured a second time, in reverse order, and each keeps the smaller of its two
        # means; the first-pass times stay available in self.first_pass.
        self.first_pass = dict(times)
        if self.refine > 0:
            again = sorted(times, key=times.get)[: self.refine] + [i for i in must if i in times]
            for i in reversed(list(dict.fromkeys(again))):
                c, _ = self.cfgs[i]
                t = time_cfg(c, self.warmup, self.iters)
                self.launches += self.warmup + self.iters
                self.gpu_s += (self.warmup + self.iters) * t * 1e-6
                times[i] = min(times[i], t)
        return times


def _open_ctx(a, torch):
    ctx = wt.wt_create(0, a.in_type, a.out_type)
    path = a.table or tune.table_path(a.in_type, a.out_type)
    wt.wt_load(ctx, path)
    return ctx, path


def _pick_vs_best(ctx, ex, shapes):
    rows = []
    t0 = time.time()
    for n, (M, N, K) in enumerate(shapes):
        pick = wt.wt_select(ctx, M, N, K)
        times = ex.run(M, N, K, must=(pick.id,))
        best_id = min(times, key=times.get)
        bc = ex.cfgs[best_id][0]
        fp = ex.first_pass
        rows.append({"M": M, "N": N, "K": K, "pick": list(pick.astuple()), "pick_us": times[pick.id],
                     "frac_single_pass": min(fp.values()) / fp[pick.id],
                     "best": list(bc.astuple()), "best_us": times[best_id], "frac": times[best_id] / times[pick.id],
                     "pick_tflops": 2.0 * M * N * K / times[pick.id] / 1e6,
                     "best_tflops": 2.0 * M * N * K / times[best_id] / 1e6,
                     "pred_us": wt.wt_predict_us(ctx, M, N, K, pick), "n_timed": len(times),
                     "times": {str(i): round(t, 3) for i, t in times.items()}})
        if n % 10 == 0:
            _log(f"[eval] {n + 1}/{len(shapes)} shapes, {time.time() - t0:.0f}s, last frac {rows[-1]['frac']:.3f}")
    fr = np.array([r["frac"] for r in rows])
    f1 = np.array([r["frac_single_pass"] for r in rows])
    summary = {"n_shapes": len(rows), "refine": ex.refine,
               "single_pass": {"geomean_frac": float(np.exp(np.mean(np.log(f1)))), "min_frac": float(f1.min()),
                               "p5_frac": float(np.percentile(f1, 5)), "frac_ge_95": float(np.mean(f1 >= 0.95))},
               "geomean_frac": float(np.exp(np.mean(np.log(fr)))), "min_frac": float(fr.min()),
               "p5_frac": float(np.percentile(fr, 5)), "mean_frac": float(fr.mean()),
               "frac_ge_95": float(np.mean(fr >= 0.95)), "exhaustive_launches": ex.launches,
               "exhaustive_gpu_seconds": ex.gpu_s}
    return rows, summary


def cmd_sweep(a, torch):
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    ex = Exhaustive(ctx, torch, a.in_type, a.out_type, prune=a.prune, refine=a.refine, rotate_mb=a.rotate_mb)
    rows, summary = _pick_vs_best(ctx, ex, wt_synth.sweep_shapes())
    summary["weights_rotated_over_mb"] = a.rotate_mb
    return {"workload": "LLM-projection sweep (27 shapes)" + (", weights rotating through HBM" if a.rotate_mb else ""),
            "table": path, "summary": summary, "rows": rows}


def cmd_shapes(a, torch):
    """Pick vs exhaustive search on a named synthetic shape set: `paper` = shapes in the ranges of the paper's
    Dense-GEMM test set, `shortk` = small launches with K from 256 to 2048 (wt_synth)."""
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    sets = {"paper": ("shapes in the ranges of the paper's Dense-GEMM test set (M 64..16384, N 384..8192, K 2048..8192)",
                      wt_synth.paper_range_shapes),
            "shortk": ("small launches, K in {256..2048}, M 16..4096, N 256..4096", wt_synth.short_k_shapes)}
    name, gen = sets[a.set]
    ex = Exhaustive(ctx, torch, a.in_type, a.out_type, prune=a.prune, refine=a.refine)
    rows, summary = _pick_vs_best(ctx, ex, gen())
    return {"workload": name, "table": path, "summary": summary, "rows": rows}


def cmd_stream(a, torch):
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    shapes = wt_synth.stream_shapes()
    mean_ns, p99_ns = wt.wt_select_bench(ctx, shapes, repeats=5)
    # exhaustive search on a seeded sample of the stream's draws (duplicates collapse into weights, so
    # the score is weighted the way the stream itself weights shapes)
    rng = np.random.default_rng(a.sample_seed)
    draws = [shapes[i] for i in rng.choice(len(shapes), size=min(a.sample, len(shapes)), replace=False)]
    weight = {}
    for sh in draws:
        weight[sh] = weight.get(sh, 0) + 1
    sample = sorted(weight)
    ex = Exhaustive(ctx, torch, a.in_type, a.out_type, prune=a.prune, refine=a.refine, rotate_mb=a.rotate_mb)
    rows, summary = _pick_vs_best(ctx, ex, sample)
    wts = np.array([weight[(r["M"], r["N"], r["K"])] for r in rows], dtype=float)
    fr = np.array([r["frac"] for r in rows])
    for r, w in zip(rows, wts):
        r["weight"] = int(w)
    summary.update({"weights_rotated_over_mb": a.rotate_mb, "stream_shapes": len(shapes), "unique_shapes": len(set(shapes)), "sampled_draws": len(draws),
                    "exhaustive_shapes": len(sample),
                    "weighted_geomean_frac": float(np.exp(np.sum(wts * np.log(fr)) / wts.sum())),
                    "weighted_frac_ge_95": float(np.sum(wts * (fr >= 0.95)) / wts.sum()),
                    "select_mean_us": mean_ns / 1e3, "select_p99_us": p99_ns / 1e3})
    return {"workload": "runtime stream: 10,000 seeded shapes; exhaustive search on a seeded sample of its draws",
            "table": path, "summary": summary, "rows": rows}


def cmd_wave(a, torch):
    """Wave-quantisation stress: latency of fixed configurations vs N, against the table's
    prediction, a step model (T_wave * w) and a single global linear-in-G model (Sec. 3.2, Fig. 3)."""
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    stream = torch.cuda.current_stream()
    shapes = wt_synth.wave_stress_shapes()
    out = {"workload": "wave-quantisation stress: M=K=4096, N=128..16384 step 128", "table": path, "configs": []}
    for fields in a.cfgs:
        cid = wt.wt_config_find(ctx, *fields)
        c, r = wt.wt_config_get(ctx, cid)
        pts = []
        for (M, N, K) in shapes:
            A, B, C, sA, sB = _dev_operands(torch, M, N, K, a.in_type, a.out_type)
            us = wt.wt_time_gemm(ctx, M, N, K, A, B, C, c, 3, 5, sA, sB, stream)
            G, L, w = wt.wt_wave_count(ctx, M, N, K, c)
            pts.append({"N": N, "G": G, "w": w, "us": us, "pred_us": wt.wt_predict_us(ctx, M, N, K, c)})
        us = np.array([p["us"] for p in pts]); G = np.array([p["G"] for p in pts], dtype=float)
        w = np.array([p["w"] for p in pts], dtype=float); pred = np.array([p["pred_us"] for p in pts])
        t_wave = float(np.sum(us * w) / np.sum(w * w))                    # least-squares step model through 0
        lin = np.polyfit(G, us, 1)                                        # global linear model in G
        mape = lambda m: float(np.mean(np.abs(m - us) / us))
        small, large = w <= 3, w > 3
        out["configs"].append({"cfg": list(c.astuple()), "occ": r.occ, "capacity": 256 * r.occ,
                               "mape_wavetune": mape(pred), "mape_step": mape(t_wave * w),
                               "mape_linear": mape(np.polyval(lin, G)),
                               "mape_small_w": {"wavetune": float(np.mean(np.abs(pred - us)[small] / us[small])),
                                                "step": float(np.mean(np.abs(t_wave * w - us)[small] / us[small])),
                                                "linear": float(np.mean(np.abs(np.polyval(lin, G) - us)[small] / us[small]))},
                               "mape_large_w": {"wavetune": float(np.mean(np.abs(pred - us)[large] / us[large])),
                                                "step": float(np.mean(np.abs(t_wave * w - us)[large] / us[large])),
                                                "linear": float(np.mean(np.abs(np.polyval(lin, G) - us)[large] / us[large]))},
                               "points": pts})
        _log(f"[eval] wave cfg {c.astuple()}: MAPE wavetune {out['configs'][-1]['mape_wavetune']:.3f} "
             f"step {out['configs'][-1]['mape_step']:.3f} linear {out['configs'][-1]['mape_linear']:.3f}")
    return out


def cmd_large(a, torch):
    """Large prefill GEMM 16384 x 8192 x 8192, bf16 and fp8 e4m3, bf16 out: best configuration,
    TFLOP/s against the nominal peak and against the measured MFMA-only ceiling."""
    M, N, K = 16384, 8192, 8192
    out = {"workload": f"large prefill GEMM {M}x{N}x{K}, bf16 out", "results": []}
    for in_type, name, peak in ((wt.WT_BF16, "bf16", 2500.0), (wt.WT_FP8_E4M3, "fp8_e4m3", 5000.0)):
        ctx = wt.wt_create(0, in_type, wt.WT_OUT_BF16)
        ex = Exhaustive(ctx, torch, in_type, wt.WT_OUT_BF16, prune=1.5, refine=8)
        ex.run(M, N, K)            # a first pass only to bring the chip to its sustained clock: its times are dropped
        times = ex.run(M, N, K)    # (the first configurations measured on an idle chip would otherwise read slow)
        top = sorted(times.items(), key=lambda kv: kv[1])[:6]
        ceiling = wt.wt_mfma_ceiling(ctx, in_type, 20000, torch.cuda.current_stream())
        res = {"in": name, "nominal_peak_tflops": peak, "mfma_only_ceiling_tflops": ceiling, "top": []}
        for i, us in top:
            tf = 2.0 * M * N * K / us / 1e6
            res["top"].append({"cfg": list(ex.cfgs[i][0].astuple()), "us": us, "tflops": tf,
                               "frac_nominal": tf / peak, "frac_ceiling": tf / ceiling})
        out["results"].append(res)
        _log(f"[eval] large {name}: best {res['top'][0]}")
        wt.wt_destroy(ctx)
    return out


def cmd_grouped(a, torch):
    """Grouped GEMM (MoE expert projections): synthetic skewed routing, every unsplit configuration timed
    with the routing's real group sizes; the pick comes from wt_select_grouped, which sees only the number
    of groups and the total row count (uniform approximation); beside it, the pick of wt_select_grouped_rows,
    which is given the real counts (a router that has synchronised).
    """
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    stream = torch.cuda.current_stream()
    cfgs = [wt.wt_config_get(ctx, i) for i in range(wt.wt_config_count(ctx))]
    rows = []
    for (E, top_k, N, K) in wt_synth.MOE_LAYERS:
        g = torch.Generator(device="cuda")
        g.manual_seed(4000 + E + N)
        B = torch.randn((E * N, K), device="cuda", generator=g).to(torch.bfloat16)
        for tokens in wt_synth.MOE_TOKENS:
            counts = wt_synth.moe_routing(tokens, E, top_k, seed=tokens + E, skew=a.skew)
            M_total = int(counts.sum())
            off = torch.from_numpy(wt_synth.group_offsets(counts)).cuda()
            A = torch.randn((M_total, K), device="cuda", generator=g).to(torch.bfloat16)
            C = torch.empty((M_total, N), device="cuda", dtype=torch.bfloat16)
            pick = wt.wt_select_grouped(ctx, E, M_total, N, K)
            pick_rows = wt.wt_select_grouped_rows(ctx, counts, N, K)
            times, best = {}, math.inf
            for i, (c, r) in enumerate(cfgs):
                if c.split != 1 or r.occ < 1:
                    continue
                if i not in (pick.id, pick_rows.id) and best < math.inf:
                    t1 = wt.wt_time_gemm_grouped(ctx, E, off, M_total, N, K, A, B, C, c, 1, 1, stream=stream)
                    if t1 > a.prune * best:
                        continue
                t = wt.wt_time_gemm_grouped(ctx, E, off, M_total, N, K, A, B, C, c, 3, 5, stream=stream)
                times[i] = t
                best = min(best, t)
            best_id = min(times, key=times.get)
            rows.append({"experts": E, "top_k": top_k, "tokens": tokens, "rows": M_total, "N": N, "K": K,
                         "rows_per_expert_min_max": [int(counts.min()), int(counts.max())],
                         "pick": list(pick.astuple()), "pick_us": times[pick.id],
                         "best": list(cfgs[best_id][0].astuple()), "best_us": times[best_id],
                         "frac": times[best_id] / times[pick.id],
                         "pick_rows": list(pick_rows.astuple()), "frac_rows": times[best_id] / times[pick_rows.id],
                         "pick_tflops": 2.0 * M_total * N * K / times[pick.id] / 1e6,
                         "best_tflops": 2.0 * M_total * N * K / times[best_id] / 1e6, "n_timed": len(times),
                         "times": {str(i): round(t, 3) for i, t in times.items()}})
            _log(f"[eval] grouped E={E} tokens={tokens} N={N} K={K}: frac {rows[-1]['frac']:.3f} (real counts {rows[-1]['frac_rows']:.3f}) "
                 f"pick {rows[-1]['pick_us']:.1f}us {rows[-1]['pick_tflops']:.0f} TF")
            del A, C
        del B
    fr = np.array([r["frac"] for r in rows])
    frr = np.array([r["frac_rows"] for r in rows])
    summary = {"n_cases": len(rows), "geomean_frac": float(np.exp(np.mean(np.log(fr)))), "min_frac": float(fr.min()),
               "frac_ge_95": float(np.mean(fr >= 0.95)),
               "real_counts": {"geomean_frac": float(np.exp(np.mean(np.log(frr)))), "min_frac": float(frr.min()),
                               "frac_ge_95": float(np.mean(frr >= 0.95))}}
    return {"workload": f"grouped GEMM, MoE expert projections, routing probabilities 1/rank^{a.skew}, bf16", "table": path,
            "summary": summary, "rows": rows}


def cmd_persistent(a, torch):
    """Persistent launches (grid clamped to the resident block count; mode 1: blocks walk the task list with a fixed
    stride, mode 2: blocks draw tasks from the device-side queue) against the ordinary one block per task, same
    configuration (wt_select's pick), same protocol, on the sweep, the large prefill and a sample of the stream."""
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    stream = torch.cuda.current_stream()
    rng = np.random.default_rng(2007)
    st = wt_synth.stream_shapes()
    shapes = wt_synth.sweep_shapes() + [(16384, 8192, 8192)] + [st[i] for i in rng.choice(len(st), size=40, replace=False)]
    rows = []
    for (M, N, K) in shapes:
        A, B, C, sA, sB = _dev_operands(torch, M, N, K, a.in_type, a.out_type)
        cfg = wt.wt_select(ctx, M, N, K)
        G, L, w = wt.wt_wave_count(ctx, M, N, K, cfg)
        t = {0: [], 1: [], 2: []}
        for rep in range(2):                     # alternate to cancel clock drift
            for mode in (0, 1, 2):
                wt.wt_set_persistent(ctx, mode)
                t[mode].append(wt.wt_time_gemm(ctx, M, N, K, A, B, C, cfg, 3, 10, sA, sB, stream))
        wt.wt_set_persistent(ctx, 0)
        plain, pers, queue = min(t[0]), min(t[1]), min(t[2])
        rows.append({"M": M, "N": N, "K": K, "cfg": list(cfg.astuple()), "tasks": G, "waves": w,
                     "plain_us": plain, "persistent_us": pers, "queue_us": queue, "speedup": plain / pers,
                     "speedup_queue": plain / queue})
        _log(f"[eval] persistent {M}x{N}x{K} {cfg.astuple()} tasks {G}: {plain:.1f} -> stride {pers:.1f} us "
             f"({plain / pers:.3f}x), queue {queue:.1f} us ({plain / queue:.3f}x)")
    summary = {"n_shapes": len(rows)}
    for key, name in (("speedup", "stride"), ("speedup_queue", "queue")):
        sp = np.array([r[key] for r in rows])
        multi = [r[key] for r in rows if r["waves"] > 1]
        summary[name] = {"geomean_speedup": float(np.exp(np.mean(np.log(sp)))),
                         "geomean_speedup_multi_wave": float(np.exp(np.mean(np.log(multi)))) if multi else None,
                         "min": float(sp.min()), "max": float(sp.max())}
    return {"workload": "persistent (fixed stride / task queue) vs one-block-per-task launch under wt_select's configuration",
            "table": path, "summary": summary, "rows": rows}


def cmd_vendor(a, torch):
    """Context, not a target: the vendor library's GEMM (torch.matmul on ROCm, i.e. hipBLASLt / rocBLAS with its
    own heuristics) on the same shapes and buffers, timed with HIP events around batches of launches like
    wt_time_gemm does, beside this library under wt_select's configuration.  bf16 in, bf16 out."""
    import wt_synth

    ctx, path = _open_ctx(a, torch)
    stream = torch.cuda.current_stream()
    rng = np.random.default_rng(2008)
    st = wt_synth.stream_shapes()
    shapes = wt_synth.sweep_shapes() + [(16384, 8192, 8192)] + [st[i] for i in rng.choice(len(st), size=30, replace=False)]

    def time_matmul(A, B, C, iters=5):
        for _ in range(3):
            torch.matmul(A, B.t(), out=C)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ms = 0.0
        for _pass in range(2):
            e0.record(stream)
            for _ in range(iters):
                torch.matmul(A, B.t(), out=C)
            e1.record(stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            if ms * 1000.0 >= 300.0:
                break
            iters = min(max(int(300.0 / max(ms * 1000.0 / iters, 0.5)) + 1, iters), iters * 64)
        return ms * 1000.0 / iters

    rows = []
    for (M, N, K) in shapes:
        A, B, C, sA, sB = _dev_operands(torch, M, N, K, wt.WT_BF16, wt.WT_OUT_BF16)
        cfg = wt.wt_select(ctx, M, N, K)
        ours = min(wt.wt_time_gemm(ctx, M, N, K, A, B, C, cfg, 3, 5, stream=stream) for _ in range(2))
        vend = min(time_matmul(A, B, C) for _ in range(2))
        rows.append({"M": M, "N": N, "K": K, "cfg": list(cfg.astuple()), "wt_us": ours, "vendor_us": vend,
                     "vendor_over_wt": vend / ours})
        _log(f"[eval] vendor {M}x{N}x{K}: wt {ours:.1f} us, torch.matmul {vend:.1f} us ({vend / ours:.2f}x)")
    r = np.array([x["vendor_over_wt"] for x in rows])
    summary = {"n_shapes": len(rows), "geomean_vendor_over_wt": float(np.exp(np.mean(np.log(r)))),
               "min": float(r.min()), "max": float(r.max()), "torch": torch.__version__}
    return {"workload": "torch.matmul (vendor library) vs wt_gemm under wt_select's configuration, bf16", "table": path,
            "summary": summary, "rows": rows}


def cmd_attn(a, torch):
    """Attention test set (stand-in for Sec. 5.1's: sequence length 64..16384, 16..128 query heads, 2..16 KV
    heads, head dimension 128): wt_select(S_q, N_h, S_kv) on the attention table against exhaustive search over the
    attention registry, plus the best single configuration as the fixed-default baseline and the vendor
    library's scaled_dot_product_attention as context."""
    import wt_synth

    ctx = wt.wt_create(0, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    path = a.table or tune.table_path(wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    wt.wt_load(ctx, path)
    cfgs = [wt.wt_config_get(ctx, i) for i in range(wt.wt_config_count(ctx))]
    stream = torch.cuda.current_stream()
    causal = int(bool(a.causal))
    scale = 1.0 / math.sqrt(128.0)
    rows, t0 = [], time.time()
    for n, (S_q, S_kv, H_q, H_kv) in enumerate(wt_synth.attn_shapes(a.sample, a.sample_seed)):
        g = torch.Generator(device="cuda")
        g.manual_seed(3000 + n)
        Q = torch.randn((S_q * H_q, 128), device="cuda", generator=g).to(torch.bfloat16)
        K = torch.randn((S_kv * H_kv, 128), device="cuda", generator=g).to(torch.bfloat16)
        V = torch.randn((S_kv * H_kv, 128), device="cuda", generator=g).to(torch.bfloat16)
        O = torch.empty_like(Q)
        times = {}
        for i, (c, r) in enumerate(cfgs):
            times[i] = wt.wt_time_attn(ctx, H_q, H_kv, S_q, S_kv, Q, K, V, O, scale, causal, c, 2, 4, stream)
        pick = wt.wt_select(ctx, S_q, H_q, S_kv)
        best_id = min(times, key=times.get)
        flop = 4.0 * S_q * S_kv * 128 * H_q * (0.5 if causal else 1.0)
        q4 = Q.view(S_q, H_q, 128).permute(1, 0, 2)[None]
        k4 = K.view(S_kv, H_kv, 128).permute(1, 0, 2)[None].repeat_interleave(H_q // H_kv, 1)
        v4 = V.view(S_kv, H_kv, 128).permute(1, 0, 2)[None].repeat_interleave(H_q // H_kv, 1)
        for _ in range(2):
            torch.nn.functional.scaled_dot_product_attention(q4, k4, v4, is_causal=bool(causal), scale=scale)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(4):
            torch.nn.functional.scaled_dot_product_attention(q4, k4, v4, is_causal=bool(causal), scale=scale)
        e1.record()
        torch.cuda.synchronize()
        vendor_us = e0.elapsed_time(e1) * 1000.0 / 4
        rows.append({"S_q": S_q, "S_kv": S_kv, "H_q": H_q, "H_kv": H_kv, "pick": list(pick.astuple()),
                     "pick_us": times[pick.id], "best": list(cfgs[best_id][0].astuple()), "best_us": times[best_id],
                     "frac": times[best_id] / times[pick.id], "pick_tflops": flop / times[pick.id] / 1e6,
                     "best_tflops": flop / times[best_id] / 1e6, "vendor_us": vendor_us,
                     "times": {str(i): round(t, 3) for i, t in times.items()}})
        if n % 8 == 0:
            _log(f"[attn] {n + 1} shapes, {time.time() - t0:.0f}s, last frac {rows[-1]['frac']:.3f}")
    fr = np.array([r["frac"] for r in rows])
    gm = lambda x: float(np.exp(np.mean(np.log(np.asarray(x, dtype=np.float64)))))
    # the best single configuration over the whole set = a fixed default
    fixed = min(range(len(cfgs)), key=lambda i: gm([r["times"][str(i)] for r in rows]))
    summary = {"n_shapes": len(rows), "geomean_frac": gm(fr), "min_frac": float(fr.min()),
               "frac_ge_95": float(np.mean(fr >= 0.95)),
               "fixed_default": list(cfgs[fixed][0].astuple()),
               "fixed_default_geomean_frac": gm([r["best_us"] / r["times"][str(fixed)] for r in rows]),
               "speedup_pick_over_fixed_default": gm([r["times"][str(fixed)] / r["pick_us"] for r in rows]),
               "speedup_best_over_fixed_default": gm([r["times"][str(fixed)] / r["best_us"] for r in rows]),
               "vendor_over_pick_geomean": gm([r["vendor_us"] / r["pick_us"] for r in rows]),
               "max_pick_tflops": float(max(r["pick_tflops"] for r in rows))}
    wt.wt_destroy(ctx)
    return {"workload": f"attention test set, {len(rows)} shapes, causal={causal}", "table": path, "causal": causal,
            "summary": summary, "rows": rows}


def cmd_attn_varlen(a, torch):
    """Variable-length prefill batches (the shape of the paper's end-to-end setting, Sec. 5.3: batches of 2/4/8 prompts
    of 512..16384 tokens; 32 query / 4 KV heads of dimension 128): wt_attn_varlen under the pick of
    wt_select_attn_varlen (the host knows the lengths) and, beside it, under wt_select(ceil(total/batch), batch * heads,
    ceil(total/batch)) (a selector that sees only the totals), against exhaustive search over the attention registry
    with the real lengths, causal."""
    import wt_synth

    ctx = wt.wt_create(0, wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    path = a.table or tune.table_path(wt.WT_ATTN_BF16, wt.WT_OUT_BF16)
    wt.wt_load(ctx, path)
    cfgs = [wt.wt_config_get(ctx, i) for i in range(wt.wt_config_count(ctx))]
    stream = torch.cuda.current_stream()
    H_q, H_kv, scale = 32, 4, 1.0 / math.sqrt(128.0)
    rows = []
    for case, lens in enumerate(wt_synth.varlen_batches(a.sample, a.sample_seed)):
        batch, total = len(lens), sum(lens)
        cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), device="cuda")
        g = torch.Generator(device="cuda")
        g.manual_seed(5000 + case)
        Q = torch.randn((total * H_q, 128), device="cuda", generator=g).to(torch.bfloat16)
        K = torch.randn((total * H_kv, 128), device="cuda", generator=g).to(torch.bfloat16)
        V = torch.randn((total * H_kv, 128), device="cuda", generator=g).to(torch.bfloat16)
        O = torch.empty_like(Q)

        def timed(c, iters=4):
            for _ in range(2):
                wt.wt_attn_varlen(ctx, batch, H_q, H_kv, total, total, cu, cu, Q, K, V, O, scale, 1, c, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(iters):
                wt.wt_attn_varlen(ctx, batch, H_q, H_kv, total, total, cu, cu, Q, K, V, O, scale, 1, c, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / iters
        times = {i: timed(c) for i, (c, r) in enumerate(cfgs)}
        mean_len = -(-total // batch)
        pick = wt.wt_select_attn_varlen(ctx, lens, lens, H_q)
        pick_totals = wt.wt_select(ctx, mean_len, batch * H_q, mean_len)
        best = min(times, key=times.get)
        flop = sum(4.0 * s * s * 128 * H_q * 0.5 for s in lens)
        rows.append({"batch": batch, "lens": lens, "pick": list(pick.astuple()), "pick_us": times[pick.id],
                     "best": list(cfgs[best][0].astuple()), "best_us": times[best], "frac": times[best] / times[pick.id],
                     "pick_totals": list(pick_totals.astuple()), "frac_totals": times[best] / times[pick_totals.id],
                     "pick_tflops": flop / times[pick.id] / 1e6, "times": {str(i): round(t, 2) for i, t in times.items()}})
        _log(f"[varlen] case {case}: batch {batch}, {total} tokens, frac {rows[-1]['frac']:.3f}, {rows[-1]['pick_tflops']:.0f} TF")
    fr = np.array([r["frac"] for r in rows])
    gm = lambda x: float(np.exp(np.mean(np.log(np.asarray(x, dtype=np.float64)))))
    fixed = min(range(len(cfgs)), key=lambda i: gm([r["times"][str(i)] for r in rows]))
    ft = np.array([r["frac_totals"] for r in rows])
    summary = {"n_cases": len(rows), "geomean_frac": gm(fr), "min_frac": float(fr.min()), "frac_ge_95": float(np.mean(fr >= 0.95)),
               "totals_only": {"geomean_frac": gm(ft), "min_frac": float(ft.min()), "frac_ge_95": float(np.mean(ft >= 0.95))},
               "fixed_default": list(cfgs[fixed][0].astuple()),
               "fixed_default_geomean_frac": gm([r["best_us"] / r["times"][str(fixed)] for r in rows]),
               "pick_tflops_geomean": gm([r["pick_tflops"] for r in rows])}
    wt.wt_destroy(ctx)
    return {"workload": "variable-length causal prefill batches (2/4/8 prompts of 512..16384 tokens, 32/4 heads)",
            "table": path, "summary": summary, "rows": rows}


def cmd_ablate(a, torch=None):
    """CPU only.  Re-fit the saved profiling records under model / (W, I) variants with wt_fit on a
    host-only context and score each variant's picks against saved exhaustive timings (the `times` of
    a sweep/stream result file).  A pick that the exhaustive run pruned (more than `prune` times slower
    than the best after one launch) is scored at 1/prune."""
    z = np.load(a.samples)
    recs, occ = z["samples"], z["occ"]
    evals = [json.load(open(f)) for f in a.scores]
    rows = [r for e in evals for r in e["rows"]]
    out = {"workload": "ablation of the latency model and of the profiling range, scored on " +
                       ", ".join(e["workload"] for e in evals), "variants": []}
    if "family" not in recs.dtype.names:      # records saved before the family field had its name
        recs = recs.view(wt.SAMPLE_DTYPE)
    W0, I0 = int(recs["w"].max()), a.I
    attn = a.in_type == wt.WT_ATTN_BF16       # rows hold (S_q, H_q, S_kv); anchors are KV multipliers
    anchors = tune.KV_MULTIPLIERS if attn else tune.K_ANCHORS
    shape = (lambda r: (r["S_q"], r["H_q"], r["S_kv"])) if attn else (lambda r: (r["M"], r["N"], r["K"]))

    def score(model, W, I, cap_mode, W_row=0, row_fams=0, weighting=None, short_k=True):
        weighting = a.weighting if weighting is None else weighting
        ctx = wt.wt_create(-1, a.in_type, a.out_type)
        wt.wt_set_capacity_mode(ctx, cap_mode)
        for k, o in enumerate(occ):
            wt.wt_key_set_occ(ctx, k, int(o))
        sub = recs[((recs["family"] == 0) & (recs["w"] <= W)) |
                   ((recs["family"] >= 1) & (recs["family"] <= row_fams) & (recs["w"] <= W_row))]
        if not short_k and not attn:     # leave out the records of loop anchors below K = 1024
            lo = np.array([-(-1024 // (wt.wt_config_get(ctx, 3 * k)[0].bk * wt.wt_config_get(ctx, 3 * k)[0].split))
                           for k in range(len(occ))])
            sub = sub[sub["L"] >= lo[sub["key_id"]]]
        if I < I0:       # sub-intervals of a coarser split are unions of the finer ones: keep each union's top sample
            keep = np.zeros(len(sub), dtype=bool)
            step = I0 // I
            for k in range(len(occ)):
                cap = 256 if cap_mode == 1 else 256 * int(occ[k])
                m = sub["key_id"] == k
                pos = (sub["G"][m] - 1) % cap                       # offset inside the wave region
                idx = np.minimum(pos * I0 // cap, I0 - 1)            # which of the I0 sub-intervals
                keep[np.where(m)[0]] = (idx % step) == (step - 1)
            sub = sub[keep]
        wt.wt_fit(ctx, wt.make_grid(W=W, I=I, p=min(a.p, W), k_anchors=anchors, model=model, W_row=W_row,
                                      row_fams=row_fams, n_heads=32 if attn else 0, weighting=weighting,
                                      row_mode=a.row_mode), sub)
        fr = []
        for r in rows:
            c = wt.wt_select(ctx, *shape(r))
            t = r["times"].get(str(c.id))
            fr.append(r["best_us"] / t if t else 1.0 / a.prune)
        wt.wt_destroy(ctx)
        fr = np.array(fr)
        return {"geomean_frac": float(np.exp(np.mean(np.log(fr)))), "min_frac": float(fr.min()),
                "frac_ge_95": float(np.mean(fr >= 0.95)), "records": int(len(sub))}

    W0 = int(recs["w"][recs["family"] == 0].max())
    Wr = int(recs["w"][recs["family"] >= 1].max()) if (recs["family"] >= 1).any() else 0
    for nf in range(1, int(recs["family"].max()) + 1):
        out["variants"].append({"model": f"wave-bilinear + {nf} few-row families (row_mode {a.row_mode})", "W": W0, "I": I0, "W_row": Wr,
                                **score(0, W0, I0, a.cap_mode, Wr, nf)})
    for name, model in (("wave-bilinear (full)", 0), ("linear", 1), ("step", 2)):
        out["variants"].append({"model": name, "W": W0, "I": I0, **score(model, W0, I0, a.cap_mode)})
    if not attn:
        for wname, wgt in (("relative", 1), ("ordinary", 0)):
            for sname, sk in (("with", True), ("without", False)):
                out["variants"].append({"model": f"wave-bilinear, {wname} least squares, {sname} the K = 256 / 512 anchors",
                                        "W": W0, "I": I0, **score(0, W0, I0, a.cap_mode, weighting=wgt, short_k=sk)})
    for W in sorted({w for w in (2, 5, 10, 20, W0) if w <= W0}):
        for I in sorted({i for i in (1, 2, I0) if I0 % i == 0}):
            if (W, I) != (W0, I0):
                out["variants"].append({"model": "wave-bilinear (full)", "W": W, "I": I, **score(0, W, I, a.cap_mode)})
    for v in out["variants"]:
        _log(f"[ablate] {v}")
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("cmd", choices=["sweep", "wave", "stream", "shapes", "large", "grouped", "persistent", "vendor", "ablate", "attn", "attn_varlen"])
    ap.add_argument("--set", choices=["paper", "shortk"], default="paper", help="shapes: which synthetic shape set")
    ap.add_argument("--causal", action="store_true", help="attn: causal masking (queries aligned to the end of the keys)")
    ap.add_argument("--samples", default=None, help="ablate: .npz with `samples` and `occ`")
    ap.add_argument("--scores", nargs="*", default=[], help="ablate: sweep/stream result files with exhaustive timings")
    ap.add_argument("--cap-mode", type=int, default=1)
    ap.add_argument("--weighting", type=int, default=1, help="ablate: objective of the bucket fits (0 ordinary, 1 relative: the shipped GEMM tables)")
    ap.add_argument("--row-mode", type=int, default=1, help="ablate: what the few-row families of the records hold (0 tile rows, 1 row bands: the shipped bf16 records)")
    ap.add_argument("--I", type=int, default=4)
    ap.add_argument("--p", type=int, default=10)
    ap.add_argument("--in-type", type=int, default=wt.WT_BF16)
    ap.add_argument("--out-type", type=int, default=wt.WT_OUT_BF16)
    ap.add_argument("--table", default=None)
    ap.add_argument("--out", default=None)
    ap.add_argument("--sample", type=int, default=400)
    ap.add_argument("--skew", type=float, default=1.0, help="grouped: routing probabilities ~ 1/rank^skew (0 = uniform)")
    ap.add_argument("--sample-seed", type=int, default=2005, help="stream: seed of the sampled draws")
    ap.add_argument("--prune", type=float, default=2.5)
    ap.add_argument("--rotate-mb", type=int, default=0,
                    help="sweep, stream: time every launch on another copy of the weight, the copies adding up to this many "
                         "megabytes (say 1200), so that weights stream from HBM instead of the memory-side cache")
    ap.add_argument("--refine", type=int, default=0,
                    help="sweep / stream: re-time the N fastest configurations and the pick, keep each one's smaller mean")
    ap.add_argument("--cfgs", type=lambda s: [tuple(int(x) for x in c.split(",")) for c in s.split(";")],
                    default=[(128, 128, 64, 4, 2, 0), (256, 256, 64, 8, 2, 0), (64, 64, 64, 4, 2, 0)])
    a = ap.parse_args(argv)
    if a.cmd == "ablate":
        res = cmd_ablate(a)
    else:
        import torch

        res = {"sweep": cmd_sweep, "wave": cmd_wave, "stream": cmd_stream, "shapes": cmd_shapes, "large": cmd_large, "grouped": cmd_grouped, "persistent": cmd_persistent, "vendor": cmd_vendor, "attn": cmd_attn, "attn_varlen": cmd_attn_varlen}[a.cmd](a, torch)
    txt = json.dumps(res)
    if a.out:
        os.makedirs(os.path.dirname(os.path.abspath(a.out)), exist_ok=True)
        open(a.out, "w").write(txt)
    summ = res.get("summary") or {k: v for k, v in res.items() if k != "rows"}
    print(json.dumps(summ if a.cmd in ("sweep", "stream", "shapes", "attn", "attn_varlen") else {"workload": res["workload"]}))


if __name__ == "__main__":
    main()
