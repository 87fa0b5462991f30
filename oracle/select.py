"""Oracle two-stage runtime selection (Sec. 4.4) with the extrapolation rule (Sec. 4.5), and a
reader for the binary dual-table file written by the product library, so that lookups can be
compared bit-for-bit on the very same table.

TEST INFRASTRUCTURE: see the package docstring.
"""
from __future__ import annotations

import math
import struct

import numpy as np

from .fit import Bucket, DualTable, KeyDesc
from .geometry import ceil_div, phi_gemm, phi_grouped, split_fits, uniform_rows, wave_count
from .sampler import band_family, row_family


def predict(theta, G: int, L: int) -> float:
    """T-hat = alpha*G*L + beta*G + gamma*L + delta (Sec. 4.3 bucket model), evaluated in IEEE
    binary64 as ((alpha*(G*L) + beta*G) + gamma*L) + delta with G*L formed exactly in integers.
    Python floats never fuse multiply-add, so each product and sum rounds once."""
    a, b, c, d = theta
    return ((a * float(G * L) + b * float(G)) + c * float(L)) + d


def bucket_for(table: DualTable, key: int, w: int, fam: int = 0):
    """Sec. 4.5 rule: wave-local coefficients when w <= W (and that bucket was fitted), the
    extrapolation tuple otherwise.  Returns the Bucket or None when the key has no model.
    fam = 1, 2, 3 looks in that few-row family first (extension) and falls back to the paper's
    near-square buckets when the table lacks the family or it has nothing for the key."""
    if 1 <= fam <= table.row_fams and table.W_row > 0:
        if 1 <= w <= table.W_row and table.row_local[fam - 1][key][w - 1].status:
            return table.row_local[fam - 1][key][w - 1]
        if table.row_ext[fam - 1][key].status:
            return table.row_ext[fam - 1][key]
    if 1 <= w <= table.W:
        b = table.local[key][w - 1]
        if b.status:
            return b
    b = table.ext[key]
    return b if b.status else None


def family_of(table: DualTable, M: int, BM: int) -> int:
    """Which few-row family a shape of M rows consults under a key of tile height BM: by its tile-row count (row_mode 0,
    per key) or by the row band M falls in (row_mode 1, the same for every key); 0 without families."""
    if table.W_row <= 0:
        return 0
    return band_family(M) if table.row_mode == 1 else row_family(ceil_div(M, BM))


def nearest_anchor(anchors, L: int):
    """Sec. 4.4 Stage II: anchor minimising |L* - L_i|; equal distances go to the smaller anchor."""
    best = None
    for (La, micro) in anchors:
        d = abs(L - La)
        if best is None or d < best[0]:
            best = (d, La, micro)
    return best[1], best[2]


def select(table: DualTable, M: int, N: int, K: int):
    """Stage I: argmin over keys of T-hat (strict '<', so ties keep the lowest key id);
    Stage II: nearest loop anchor in the chosen bucket.  Returns (key, micro, T-hat) or None."""
    best = None
    for k, kd in enumerate(table.keys):
        if not split_fits(M, N, kd.bm, kd.bn, kd.split, table.ws_elems, table.max_split_tiles):
            continue     # its partial tiles would not fit the workspace: not a candidate
        G, L = phi_gemm(M, N, K, kd.bm, kd.bn, kd.bk, kd.split)
        w = wave_count(G, kd.cap)
        b = bucket_for(table, k, w, family_of(table, M, kd.bm))
        if b is None:
            continue
        t = predict(b.theta, G, L)
        if math.isnan(t):
            continue
        if best is None or t < best[0]:
            best = (t, k, b, L)
    if best is None:
        return None
    t, k, b, L = best
    _, micro = nearest_anchor(b.anchors, L) if b.anchors else (0, 0)
    return k, micro, t


def select_attn(table: DualTable, n_heads: int, S_q: int, S_kv: int):
    """Runtime selection for an attention launch on a table of attention keys <T_Q, T_KV, wavefronts> (stored in
    the key descriptor as bm = T_Q, bk = T_KV): Stage I prices every key at Phi of Table 2's FlashAttention row,
    Stage II takes the micro of the nearest loop anchor.  Returns (key, micro, T-hat) or None."""
    from .attention import phi_attn

    best = None
    for k, kd in enumerate(table.keys):
        G, L = phi_attn(n_heads, S_q, S_kv, kd.bm, kd.bk)
        b = bucket_for(table, k, wave_count(G, kd.cap), 0)
        if b is None:
            continue
        t = predict(b.theta, G, L)
        if math.isnan(t):
            continue
        if best is None or t < best[0]:
            best = (t, k, b, L)
    if best is None:
        return None
    t, k, b, L = best
    _, micro = nearest_anchor(b.anchors, L) if b.anchors else (0, 0)
    return k, micro, t


def select_grouped(table: DualTable, E: int, M_total: int, N: int, K: int):
    """Grouped GEMM at run time: the dense table serves (Sec. 4.2 samples grouped GEMM as the single-group
    case); G comes from Table 2's grouped row evaluated on the uniform approximation of the routing
    (Sec. 5.2).  Configurations that split K do not run grouped launches and are left out.  Otherwise the
    two stages are those of select().  Returns (key, micro, T-hat) or None."""
    rows = uniform_rows(M_total, E)
    best = None
    for k, kd in enumerate(table.keys):
        if kd.split != 1:
            continue
        G, L = phi_grouped(rows, N, K, kd.bm, kd.bn, kd.bk)
        b = bucket_for(table, k, wave_count(G, kd.cap), family_of(table, rows[0], kd.bm))
        if b is None:
            continue
        t = predict(b.theta, G, L)
        if math.isnan(t):
            continue
        if best is None or t < best[0]:
            best = (t, k, b, L)
    if best is None:
        return None
    t, k, b, L = best
    _, micro = nearest_anchor(b.anchors, L) if b.anchors else (0, 0)
    return k, micro, t


def select_attn_varlen(table: DualTable, n_heads: int, lens_q, lens_kv):
    """Runtime selection for a ragged attention batch whose per-sequence lengths the host knows: the two stages of
    select_attn() with every key priced at phi_attn_varlen of the real lengths.  Returns (key, micro, T-hat) or None."""
    from .attention import phi_attn_varlen

    best = None
    for k, kd in enumerate(table.keys):
        G, L = phi_attn_varlen(n_heads, lens_q, lens_kv, kd.bm, kd.bk)
        b = bucket_for(table, k, wave_count(G, kd.cap), 0)
        if b is None:
            continue
        t = predict(b.theta, G, L)
        if math.isnan(t):
            continue
        if best is None or t < best[0]:
            best = (t, k, b, L)
    if best is None:
        return None
    t, k, b, L = best
    _, micro = nearest_anchor(b.anchors, L) if b.anchors else (0, 0)
    return k, micro, t


def select_grouped_rows(table: DualTable, rows, N: int, K: int):
    """Grouped GEMM whose per-group row counts the host knows (a router that has synchronised, or a fixed split):
    select_grouped() with G from Table 2's grouped row on the real counts instead of the uniform approximation.  The
    few-row family is that of the mean group, ceil(sum / E) rows, which is the uniform reading when the groups are
    equal.  Returns (key, micro, T-hat) or None."""
    rows = list(rows)
    if not rows:
        raise ValueError("at least one group")
    mean_rows = ceil_div(sum(rows), len(rows))
    best = None
    for k, kd in enumerate(table.keys):
        if kd.split != 1:
            continue
        G, L = phi_grouped(rows, N, K, kd.bm, kd.bn, kd.bk)
        b = bucket_for(table, k, wave_count(G, kd.cap), family_of(table, mean_rows, kd.bm))
        if b is None:
            continue
        t = predict(b.theta, G, L)
        if math.isnan(t):
            continue
        if best is None or t < best[0]:
            best = (t, k, b, L)
    if best is None:
        return None
    t, k, b, L = best
    _, micro = nearest_anchor(b.anchors, L) if b.anchors else (0, 0)
    return k, micro, t


# ---- reader for the product's table file ------------------------------------------------------
MAGIC = b"WTDT"


def read_table(path: str, ws_elems=None, max_split_tiles=None) -> tuple[DualTable, dict]:
    """Parse the flat little-endian dual-table file.  ws_elems / max_split_tiles: the split-K feasibility
    limits of the library that will run the table's keys (they are not in the file; None = unlimited).

    Header, 16 uint32: magic 'WTDT', version (1 to 4), n_keys, W, I, p, tau_num, tau_den, n_cu,
    A (anchor slots per bucket), in_type, out_type, key_mode, W_row (version >= 2, else 0), number of
    few-row families (versions 3 and 4; version 2 has one; version 4: row-band families, row_mode 1), the least-squares objective the buckets were fitted with
    (0 absolute, 1 relative; informational, returned in the meta dict).
    Then per key: 8 int32 (bm, bn, bk, nwave, stages, occ, n_micro, split [0 = 1]), int64 cap, and a
    bucket block of R = W+1 rows (w = 1..W, then ext): R*4 float64 theta, R int32 status, R int32
    n_anchor, R*A int32 anchor L, R*A int32 anchor micro.  Versions 2 to 4 append, per key, one further
    block of W_row+1 rows for every few-row family.
    """
    raw = open(path, "rb").read()
    hdr = struct.unpack_from("<4s15I", raw, 0)
    if hdr[0] != MAGIC or hdr[1] not in (1, 2, 3, 4):
        raise ValueError("not a version-1..4 dual table")
    n_keys, W, I, p, tnum, tden, n_cu, A, in_t, out_t, mode = hdr[2:13]
    W_row = hdr[13] if hdr[1] >= 2 else 0
    n_fams = 0 if W_row == 0 else (hdr[14] if hdr[1] >= 3 else 1)
    off = 64

    def block(R):
        nonlocal off
        theta = np.frombuffer(raw, dtype="<f8", count=R * 4, offset=off).reshape(R, 4); off += R * 32
        status = np.frombuffer(raw, dtype="<i4", count=R, offset=off); off += R * 4
        n_anchor = np.frombuffer(raw, dtype="<i4", count=R, offset=off); off += R * 4
        aL = np.frombuffer(raw, dtype="<i4", count=R * A, offset=off).reshape(R, A); off += R * A * 4
        aM = np.frombuffer(raw, dtype="<i4", count=R * A, offset=off).reshape(R, A); off += R * A * 4
        out = []
        for r in range(R):
            anchors = [(int(aL[r, j]), int(aM[r, j])) for j in range(int(n_anchor[r]))]
            out.append(Bucket(theta=tuple(float(x) for x in theta[r]), status=int(status[r]), anchors=anchors))
        return out

    keys, local, ext = [], [], []
    row_local, row_ext = [[] for _ in range(n_fams)], [[] for _ in range(n_fams)]
    for _ in range(n_keys):
        bm, bn, bk, nwave, stages, occ, n_micro, _r = struct.unpack_from("<8i", raw, off); off += 32
        (cap,) = struct.unpack_from("<q", raw, off); off += 8
        keys.append(KeyDesc(bm, bn, bk, nwave, stages, occ, cap, max(1, _r)))
        buckets = block(W + 1)
        local.append(buckets[:W])
        ext.append(buckets[W])
        for f in range(n_fams):
            buckets = block(W_row + 1)
            row_local[f].append(buckets[:W_row])
            row_ext[f].append(buckets[W_row])
    if off != len(raw):
        raise ValueError("trailing bytes in dual table")
    meta = dict(I=I, p=p, tau_num=tnum, tau_den=tden, n_cu=n_cu, A=A, in_type=in_t, out_type=out_t, key_mode=mode,
                W_row=W_row, weighting=hdr[15], row_mode=int(hdr[1] == 4))
    return DualTable(W=W, keys=keys, local=local, ext=ext, W_row=W_row, row_local=row_local, row_ext=row_ext,
                     row_mode=int(hdr[1] == 4), ws_elems=ws_elems, max_split_tiles=max_split_tiles), meta
