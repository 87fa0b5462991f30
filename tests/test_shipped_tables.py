"""The dual tables shipped with the package match the compiled registry, their profiling records are consistent
with them, and the GEMM tables select exactly like the oracle's selector on the same file (no GPU)."""
import os

import numpy as np
import pytest

import paper_2604_10187_amd as wt
import wt_synth
from oracle import fit as ofit
from oracle import select as osel
from _pins import lib_limits, split_limits

SPLIT_LIMITS = split_limits()                 # the library's split-K workspace limits, from include/wt.h
MAX_ANCHORS = lib_limits()["max_anchors"]     # anchor slots per bucket of its table format

TABLES = os.path.join(os.path.dirname(wt.LIB_PATH), "tables")
CASES = [(wt.WT_BF16, "mi355x_in0_out1"), (wt.WT_FP8_E4M3, "mi355x_in1_out1"), (wt.WT_ATTN_BF16, "mi355x_attn")]


@pytest.mark.parametrize("in_type,stem", CASES)
def test_table_loads_into_the_registry_and_records_match(in_type, stem):
    ctx = wt.wt_create(-1, in_type, wt.WT_OUT_BF16)
    try:
        wt.wt_load(ctx, os.path.join(TABLES, stem + ".wt"))       # refuses a table whose keys differ from the registry
        nk = wt.wt_key_count(ctx)
        table, _ = osel.read_table(os.path.join(TABLES, stem + ".wt"), **SPLIT_LIMITS)
        assert len(table.keys) == nk
        for k, kd in enumerate(table.keys):
            c, _ = wt.wt_config_get(ctx, 3 * k)
            assert (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, kd.split) == (c.bm, c.bn, c.bk, c.nwave, c.stages, c.split)
        z = np.load(os.path.join(TABLES, stem + "_samples.npz"))
        recs, occ = z["samples"], z["occ"]
        assert len(occ) == nk and int(recs["key_id"].max()) < nk and int(recs["key_id"].min()) == 0
        assert (recs["mean_us"] > 0).all() and (recs["micro_id"] < 3).all() and (recs["w"] >= 1).all()
        # every key has records of the paper's sampler (family 0)
        f0 = recs[recs["family"] == 0]
        assert set(int(k) for k in np.unique(f0["key_id"])) == set(range(nk))
    finally:
        wt.wt_destroy(ctx)


@pytest.mark.parametrize("in_type,stem", CASES[:2])
def test_shipped_gemm_tables_select_like_the_oracle(in_type, stem):
    ctx = wt.wt_create(-1, in_type, wt.WT_OUT_BF16)
    try:
        path = os.path.join(TABLES, stem + ".wt")
        wt.wt_load(ctx, path)
        table, _ = osel.read_table(path, **SPLIT_LIMITS)
        for (M, N, K) in wt_synth.sweep_shapes() + wt_synth.stream_shapes(400):
            if in_type == wt.WT_FP8_E4M3 and K % 16:
                continue
            key, micro, t = osel.select(table, M, N, K)
            c = wt.wt_select(ctx, M, N, K)
            kd = table.keys[key]
            assert (c.bm, c.bn, c.bk, c.nwave, c.stages, c.swizzle, c.split) == \
                (kd.bm, kd.bn, kd.bk, kd.nwave, kd.stages, micro, kd.split)
            assert wt.wt_predict_us(ctx, M, N, K, c) == t
    finally:
        wt.wt_destroy(ctx)


@pytest.mark.parametrize("in_type,stem", CASES)
def test_shipped_tables_are_the_oracles_fit_of_the_shipped_records(in_type, stem):
    """The table files were written by the library's wt_fit from the profiling records stored beside them.  The
    oracle's fit of the same records (its own grouping, shared-micro choice, least squares and anchor thinning) must
    give the same table: every bucket's status and (L, micro) anchors identical, every coefficient equal to within
    the rounding of two different least-squares routines."""
    table, meta = osel.read_table(os.path.join(TABLES, stem + ".wt"), **SPLIT_LIMITS)
    recs = np.load(os.path.join(TABLES, stem + "_samples.npz"))["samples"]
    samples = [(int(r["key_id"]), int(r["micro_id"]), int(r["G"]), int(r["L"]), int(r["w"]), float(r["mean_us"]),
                int(r["family"])) for r in recs]
    mine = ofit.fit_tables(samples, table.keys, table.W, meta["p"], max_anchors=MAX_ANCHORS,
                           relative=bool(meta["weighting"]),      # the objective the file says it was fitted with
                           W_row=table.W_row, row_fams=max(table.row_fams, 1), row_mode=table.row_mode)
    assert (mine.W_row, mine.row_fams, mine.row_mode) == (table.W_row, table.row_fams, table.row_mode)
    n_fitted = 0

    def same(a, b, where):
        nonlocal n_fitted
        assert a.status == b.status and a.anchors == b.anchors, where
        n_fitted += a.status != 0
        for x, y in zip(a.theta, b.theta):
            assert abs(x - y) <= 1e-8 * max(abs(x), abs(y)) + 1e-12, (where, a.theta, b.theta)

    for k in range(len(table.keys)):
        for w in range(table.W + 1):
            same(table.local[k][w] if w < table.W else table.ext[k], mine.local[k][w] if w < table.W else mine.ext[k], (k, w))
        for f in range(table.row_fams):         # the few-row families, where the table has them
            for w in range(table.W_row + 1):
                same(table.row_local[f][k][w] if w < table.W_row else table.row_ext[f][k],
                     mine.row_local[f][k][w] if w < table.W_row else mine.row_ext[f][k], (f + 1, k, w))
    assert n_fitted >= len(table.keys) * (1 + table.row_fams)


def test_shipped_bf16_table_serves_the_decode_regime_from_its_16_row_family():
    """The bf16 table carries one row-band family (matrices of 16 rows under every key): shapes with M <= 16 are priced
    from it under every key alike, everything else from the paper's near-square buckets."""
    table, meta = osel.read_table(os.path.join(TABLES, "mi355x_in0_out1.wt"), **SPLIT_LIMITS)
    assert (table.W_row, table.row_fams, table.row_mode) == (8, 1, 1)
    recs = np.load(os.path.join(TABLES, "mi355x_in0_out1_samples.npz"))["samples"]
    f1 = recs[recs["family"] == 1]
    assert set(int(k) for k in np.unique(f1["key_id"])) == set(range(len(table.keys))) and int(f1["w"].max()) <= 8
    for k, kd in enumerate(table.keys):
        assert osel.family_of(table, 16, kd.bm) == 1 and osel.family_of(table, 17, kd.bm) in (0, 2)
        assert osel.bucket_for(table, k, 1, osel.family_of(table, 17, kd.bm)) is table.local[k][0]
        assert osel.bucket_for(table, k, 1, 1) is table.row_local[0][k][0]
