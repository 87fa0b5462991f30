// Host half of libwt: config registry, Phi / wave geometry, sparse sampler, bilinear fitter,
// dual table, two-stage selection, table file.  No GPU calls in this file.
//
// Paper sections: Sec. 4.1 (Phi, macro/micro split), Sec. 4.2 (sampling), Sec. 4.3 (bucketed
// bilinear model, dual table), Sec. 4.4 (two-stage selection), Sec. 4.5 (extrapolation).
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <new>
#include <stdexcept>
#include <utility>
#include <vector>

#include "wt_internal.hpp"

namespace wt {

// ---- compiled kernel lists (one function per instantiation unit) -----------------------------
#define WT_DECL(in, out, list) const KernelEntry* wt_kernels_in##in##_out##out##_list##list(int* n);
WT_DECL(0, 0, 0) WT_DECL(0, 0, 1) WT_DECL(0, 0, 2)
WT_DECL(0, 1, 0) WT_DECL(0, 1, 1) WT_DECL(0, 1, 2)
WT_DECL(1, 0, 0) WT_DECL(1, 0, 1) WT_DECL(1, 0, 2)
WT_DECL(1, 1, 0) WT_DECL(1, 1, 1) WT_DECL(1, 1, 2)
#undef WT_DECL
const KernelEntry* wt_kernels_attn(int* n);

const KernelEntry* kernel_list(int in, int out, int list, int* n) {
    if (in == WT_ATTN_BF16) {
        if (out == WT_OUT_BF16 && list == 0) return wt_kernels_attn(n);
        *n = 0;
        return nullptr;
    }
#define WT_CASE(i, o, l) \
    if (in == i && out == o && list == l) return wt_kernels_in##i##_out##o##_list##l(n);
    WT_CASE(0, 0, 0) WT_CASE(0, 0, 1) WT_CASE(0, 0, 2)
    WT_CASE(0, 1, 0) WT_CASE(0, 1, 1) WT_CASE(0, 1, 2)
    WT_CASE(1, 0, 0) WT_CASE(1, 0, 1) WT_CASE(1, 0, 2)
    WT_CASE(1, 1, 0) WT_CASE(1, 1, 1) WT_CASE(1, 1, 2)
#undef WT_CASE
    *n = 0;
    return nullptr;
}

static int ilog2(int v) {
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

// Resident blocks per compute unit from static resources: LDS bytes, wave slots (4 SIMDs x up to 8
// waves, fewer when the per-lane register count exceeds 64), 32 blocks at most.  Used on host-only
// contexts; a device context replaces it with the HIP runtime's answer.
int static_occupancy(int lds_bytes, int nwave, int vgprs) {
    const int regs = ((vgprs + 7) / 8) * 8;
    int wps = 512 / (regs > 0 ? regs : 8);
    if (wps > 8) wps = 8;
    int occ = (4 * wps) / nwave;
    if (lds_bytes > 0) occ = std::min(occ, kLdsPerCU / (((lds_bytes + 511) / 512) * 512));
    return std::max(0, std::min(occ, 32));
}

struct SplitEntry {
    int bm, bn, bk, wm, wn, st, split;
};
#define WT_SPLIT(BM, BN, BK, WM, WN, ST, S) {BM, BN, BK, WM, WN, ST, S},
static const SplitEntry kSplitBf16[] = {
#define WT_LIST_SPLIT_BF16
#include "configs.def"
#undef WT_LIST_SPLIT_BF16
};
static const SplitEntry kSplitFp8[] = {
#define WT_LIST_SPLIT_FP8
#include "configs.def"
#undef WT_LIST_SPLIT_FP8
};
#undef WT_SPLIT

static void add_key(wt_ctx* ctx, const KernelEntry& e, int split) {
    Key k{};
    k.bm = e.bm; k.bn = e.bn; k.bk = e.bk;
    k.nwave = e.wm * e.wn * e.wk;
    k.stages = e.st;
    k.split = split;
    k.sh_m = ilog2(k.bm); k.sh_n = ilog2(k.bn); k.sh_k = ilog2(k.bk * split);
    k.sh_s = ilog2(split);
    k.lds_bytes = e.lds_bytes;
    k.vgprs = (k.bm * k.bn) / (k.nwave * 64) + 64;  // accumulators + working set (estimate)
    k.occ = std::max(1, static_occupancy(k.lds_bytes, k.nwave, k.vgprs));
    k.cap = key_capacity(ctx->cap_mode, k.occ);
    k.n_micro = kNumSwizzle;
    k.first_cfg = static_cast<int>(ctx->cfgs.size());
    const int key_id = static_cast<int>(ctx->keys.size());
    for (int sw = 0; sw < kNumSwizzle; ++sw) {
        Config c{};
        c.cfg = wt_cfg{k.bm, k.bn, k.bk, k.nwave, k.stages, sw, split, static_cast<int32_t>(ctx->cfgs.size())};
        c.res = wt_cfg_res{k.lds_bytes, k.vgprs, k.nwave, k.occ, key_id, sw};
        c.wm = e.wm; c.wn = e.wn;
        c.fn = e.fn;
        c.fn_persistent = e.fn_persistent;
        c.lds_persistent = e.lds_bytes_persistent;
        ctx->cfgs.push_back(c);
    }
    ctx->keys.push_back(k);
}

int build_registry(wt_ctx* ctx) {
    ctx->cfgs.clear();
    ctx->keys.clear();
    std::vector<KernelEntry> base;
    for (int list = 0; list < 3; ++list) {
        int n = 0;
        const KernelEntry* e = kernel_list(ctx->in_type, ctx->out_type, list, &n);
        for (int i = 0; e && i < n; ++i) {
            add_key(ctx, e[i], 1);
            base.push_back(e[i]);
        }
    }
    if (ctx->in_type == WT_ATTN_BF16) return ctx->cfgs.empty() ? WT_ERR_UNSUPPORTED_CFG : WT_OK;
    // split-K keys reuse the kernel of their base entry
    const SplitEntry* sp = ctx->in_type == WT_BF16 ? kSplitBf16 : kSplitFp8;
    const size_t nsp = ctx->in_type == WT_BF16 ? sizeof(kSplitBf16) / sizeof(kSplitBf16[0])
                                               : sizeof(kSplitFp8) / sizeof(kSplitFp8[0]);
    for (size_t i = 0; i < nsp; ++i) {
        if (sp[i].split != 2 && sp[i].split != 4 && sp[i].split != 8) return WT_ERR_UNSUPPORTED_CFG;  // the kernel reduces 2, 4 or 8 slabs
        bool found = false;
        for (const KernelEntry& e : base)
            if (e.bm == sp[i].bm && e.bn == sp[i].bn && e.bk == sp[i].bk && e.wm == sp[i].wm && e.wn == sp[i].wn &&
                e.wk == 1 && e.st == sp[i].st) {
                add_key(ctx, e, sp[i].split);
                found = true;
                break;
            }
        if (!found) return WT_ERR_UNSUPPORTED_CFG;
    }
    return ctx->cfgs.empty() ? WT_ERR_UNSUPPORTED_CFG : WT_OK;
}

static inline bool same_fields(const wt_cfg& r, const wt_cfg& c) {
    return r.bm == c.bm && r.bn == c.bn && r.bk == c.bk && r.nwave == c.nwave && r.stages == c.stages &&
           r.swizzle == c.swizzle && r.split == c.split;
}

int find_config(const wt_ctx* ctx, const wt_cfg& c) {
    const int n = static_cast<int>(ctx->cfgs.size());
    if (c.id >= 0 && c.id < n && same_fields(ctx->cfgs[c.id].cfg, c)) return c.id;
    for (int i = 0; i < n; ++i)
        if (same_fields(ctx->cfgs[i].cfg, c)) return i;
    return -1;
}

// ---- sparse sampler (Sec. 4.2) -------------------------------------------------------------------
static int64_t isqrt64(int64_t v) {
    int64_t r = static_cast<int64_t>(sqrt(static_cast<double>(v)));
    while (r * r > v) --r;
    while ((r + 1) * (r + 1) <= v) ++r;
    return r;
}

// Largest g in [a,b] that is a product m*n with m <= n and n*tau_den <= m*tau_num.  Walks the
// candidate row counts m and takes, for each, the widest admissible n that keeps m*n <= b.
static int64_t best_grid_in(int64_t a, int64_t b, int tau_num, int tau_den) {
    int64_t best = 0;
    const int64_t m_hi = isqrt64(b);
    for (int64_t m = m_hi; m >= 1; --m) {
        const int64_t n_ratio = (m * tau_num) / tau_den;  // floor(tau * m)
        const int64_t n = std::min(b / m, n_ratio);
        if (n < m) continue;
        const int64_t g = m * n;
        if (g < a) {
            // for smaller m the reachable product m*floor(tau*m) only shrinks
            if (m * n_ratio < a) break;
            continue;
        }
        if (g > best) best = g;
    }
    return best;
}

// Grid samples of a key with S blocks per output tile: G = S * tiles, so the sub-interval [a,b] of
// task counts holds the tile counts ceil(a/S)..floor(b/S); the representative is the largest of those
// with a near-square factorisation m x n.  S = 1 is the paper's rule verbatim.
void sample_grid(int64_t cap, int W, int I, int tau_num, int tau_den, int split, std::vector<GridPoint>& out) {
    out.clear();
    for (int w = 1; w <= W; ++w) {
        const int64_t lo = static_cast<int64_t>(w - 1) * cap + 1;  // region R_w = [lo, w*cap]
        for (int i = 1; i <= I; ++i) {
            const int64_t a = ceil_div64(lo + (static_cast<int64_t>(i - 1) * cap) / I, split);
            const int64_t b = (lo - 1 + (static_cast<int64_t>(i) * cap) / I) / split;
            GridPoint gp{0, 0, 0};
            if (b >= a) {
                const int64_t t = best_grid_in(a, b, tau_num, tau_den);
                if (t > 0) {
                    int64_t m = isqrt64(t);  // most-square factorisation of the chosen tile count
                    while (t % m) --m;
                    gp = GridPoint{t * split, m, t / m};
                }
            }
            out.push_back(gp);
        }
    }
}

// Attention grid samples (Sec. 4.2): the head-aligned value floor(b / N_h) * N_h of each sub-interval [a, b],
// kept only if it is still inside; m = query tiles per head, n = N_h.
void sample_grid_heads(int64_t cap, int W, int I, int n_heads, std::vector<GridPoint>& out) {
    out.clear();
    for (int w = 1; w <= W; ++w) {
        const int64_t lo = static_cast<int64_t>(w - 1) * cap + 1;
        for (int i = 1; i <= I; ++i) {
            const int64_t a = lo + (static_cast<int64_t>(i - 1) * cap) / I;
            const int64_t b = lo - 1 + (static_cast<int64_t>(i) * cap) / I;
            const int64_t g = (b / n_heads) * n_heads;
            out.push_back(g >= a && g >= 1 ? GridPoint{g, g / n_heads, n_heads} : GridPoint{0, 0, 0});
        }
    }
}

// Loop counts of an attention grid point: KV length = floor(S_q * percent / 100) for every multiplier.
void kv_loop_anchors(const wt_grid* grid, int64_t S_q, int t_kv, std::vector<int64_t>& out) {
    out.clear();
    for (int j = 0; j < grid->n_k_anchors; ++j) out.push_back(ceil_div64((S_q * grid->k_anchors[j]) / 100, t_kv));
    std::sort(out.begin(), out.end());
    out.erase(std::unique(out.begin(), out.end()), out.end());
}

void loop_anchors(const wt_grid* grid, int bk_eff, std::vector<int64_t>& out) {
    out.clear();
    for (int j = 0; j < grid->n_k_anchors; ++j) out.push_back(ceil_div64(grid->k_anchors[j], bk_eff));
    std::sort(out.begin(), out.end());
    out.erase(std::unique(out.begin(), out.end()), out.end());
}

// ---- bilinear least squares (Sec. 4.3 bucket model) ---------------------------------------------
struct Row {
    double G, L, T;
};

// Solve the n x n system a*x = b by Gaussian elimination with partial pivoting.
static bool solve_small(int n, double a[4][4], double b[4], double x[4]) {
    for (int c = 0; c < n; ++c) {
        int piv = c;
        for (int r = c + 1; r < n; ++r)
            if (fabs(a[r][c]) > fabs(a[piv][c])) piv = r;
        if (a[piv][c] == 0.0) return false;
        if (piv != c) {
            for (int k = 0; k < n; ++k) std::swap(a[c][k], a[piv][k]);
            std::swap(b[c], b[piv]);
        }
        for (int r = c + 1; r < n; ++r) {
            const double f = a[r][c] / a[c][c];
            for (int k = c; k < n; ++k) a[r][k] -= f * a[c][k];
            b[r] -= f * b[c];
        }
    }
    for (int r = n - 1; r >= 0; --r) {
        double s = b[r];
        for (int k = r + 1; k < n; ++k) s -= a[r][k] * x[k];
        x[r] = s / a[r][r];
    }
    return true;
}

// Least squares of T ~ alpha*G*L + beta*G + gamma*L + delta through the normal equations in
// centred variables scaled to unit spread (on a product grid those columns are orthogonal, so the
// system is nearly diagonal).  Terms that a single distinct G (or L) cannot identify are dropped.
// relative = false: ordinary least squares, sum of (That - T)^2 (Sec. 4.3 / Sec. 5.1 as written);
// relative = true: sum of ((That - T) / T)^2 -- every record weighs 1/T^2, so that a bucket whose loop anchors span
// latencies two orders of magnitude apart is fitted to the same relative accuracy at both ends.
static int fit_rows(const std::vector<Row>& rows, double th[4], bool relative) {
    th[0] = th[1] = th[2] = th[3] = 0.0;
    const size_t n = rows.size();
    if (n == 0) return 0;
    double gm = 0, lm = 0;
    for (const Row& r : rows) { gm += r.G; lm += r.L; }
    gm /= static_cast<double>(n);
    lm /= static_cast<double>(n);
    double gs = 0, ls = 0;
    bool many_g = false, many_l = false;
    for (const Row& r : rows) {
        gs += (r.G - gm) * (r.G - gm);
        ls += (r.L - lm) * (r.L - lm);
        many_g |= (r.G != rows[0].G);
        many_l |= (r.L != rows[0].L);
    }
    gs = many_g ? sqrt(gs / static_cast<double>(n)) : 1.0;
    ls = many_l ? sqrt(ls / static_cast<double>(n)) : 1.0;
    // active columns in the order uv, u, v, 1
    int cols[4], nc = 0, status = 0;
    if (many_g && many_l) { cols[nc++] = 0; status |= 1; }
    if (many_g) { cols[nc++] = 1; status |= 2; }
    if (many_l) { cols[nc++] = 2; status |= 4; }
    cols[nc++] = 3; status |= 8;
    double ata[4][4] = {{0}}, atb[4] = {0}, x[4] = {0};
    for (const Row& r : rows) {
        const double u = (r.G - gm) / gs, v = (r.L - lm) / ls;
        const double f[4] = {u * v, u, v, 1.0};
        const double wgt = relative ? 1.0 / (r.T * r.T) : 1.0;
        for (int i = 0; i < nc; ++i) {
            for (int j = 0; j < nc; ++j) ata[i][j] += wgt * (f[cols[i]] * f[cols[j]]);
            atb[i] += wgt * (f[cols[i]] * r.T);
        }
    }
    if (!solve_small(nc, ata, atb, x)) return 0;
    double c[4] = {0, 0, 0, 0};  // coefficients of uv, u, v, 1
    for (int i = 0; i < nc; ++i) c[cols[i]] = x[i];
    const double a = c[0] / (gs * ls);
    th[0] = a;
    th[1] = c[1] / gs - a * lm;
    th[2] = c[2] / ls - a * gm;
    th[3] = c[3] - c[1] * gm / gs - c[2] * lm / ls + a * gm * lm;
    return status;
}

// One bucket: records of a single <key, wave set>.  For every loop count pick the micro whose mean
// latency over the bucket's grid sizes is smallest (it must have a record at each of them; ties go
// to the lower id), keep it as the anchor for that loop count, and fit on those records only.
static void fit_bucket(std::vector<const wt_sample*>& recs, Bucket& out, bool relative) {
    memset(&out, 0, sizeof(out));
    std::sort(recs.begin(), recs.end(), [](const wt_sample* x, const wt_sample* y) {
        if (x->L != y->L) return x->L < y->L;
        if (x->micro_id != y->micro_id) return x->micro_id < y->micro_id;
        return x->G < y->G;
    });
    std::vector<Row> rows;
    std::vector<std::pair<int32_t, int32_t>> anchors;  // (L, micro) of every loop count, ascending L
    size_t i = 0;
    while (i < recs.size()) {
        size_t j = i;
        while (j < recs.size() && recs[j]->L == recs[i]->L) ++j;
        // distinct grid sizes of this loop count
        std::vector<int64_t> grid;
        for (size_t t = i; t < j; ++t) grid.push_back(recs[t]->G);
        std::sort(grid.begin(), grid.end());
        grid.erase(std::unique(grid.begin(), grid.end()), grid.end());
        double best_mean = 0;
        size_t best_lo = 0, best_hi = 0;
        bool have = false;
        size_t t = i;
        while (t < j) {
            size_t u = t;
            double sum = 0;
            std::vector<int64_t> seen;
            while (u < j && recs[u]->micro_id == recs[t]->micro_id) {
                sum += recs[u]->mean_us;
                if (seen.empty() || seen.back() != recs[u]->G) seen.push_back(recs[u]->G);
                ++u;
            }
            if (seen == grid) {
                const double mean = sum / static_cast<double>(u - t);
                if (!have || mean < best_mean) { have = true; best_mean = mean; best_lo = t; best_hi = u; }
            }
            t = u;
        }
        if (have) {
            anchors.emplace_back(static_cast<int32_t>(recs[best_lo]->L), recs[best_lo]->micro_id);
            for (size_t r = best_lo; r < best_hi; ++r)
                rows.push_back(Row{static_cast<double>(recs[r]->G), static_cast<double>(recs[r]->L), recs[r]->mean_us});
        }
        i = j;
    }
    // A bucket stores kMaxAnchors anchors.  With more loop counts than that (attention: every grid size brings
    // its own KV lengths) the ones at ranks floor(i * (n - 1) / (kMaxAnchors - 1)) are kept: first, last and an
    // even spread between them.
    const int n = static_cast<int>(anchors.size());
    out.n_anchor = n < kMaxAnchors ? n : kMaxAnchors;
    for (int a = 0; a < out.n_anchor; ++a) {
        const int src = n <= kMaxAnchors ? a : (a * (n - 1)) / (kMaxAnchors - 1);
        out.anchor_L[a] = anchors[src].first;
        out.anchor_micro[a] = anchors[src].second;
    }
    out.status = fit_rows(rows, out.th, relative);
}

// Ablation "Step": T = w*(a*L + b) with w = ceil(G/cap).  Shared micro per loop count over all of the
// key's records, then the 2x2 normal equations on the columns (w*L, w), each scaled by its largest
// magnitude.  With a single distinct L only b is identified.
static void fit_step(std::vector<const wt_sample*>& recs, int64_t cap, double* a_out, double* b_out, Bucket& anchors) {
    Bucket tmp;
    fit_bucket(recs, tmp, false);  // sorts recs by (L, micro, G) and yields the anchors (shared micro per L)
    anchors = tmp;
    double sxx = 0, sxz = 0, szz = 0, sxy = 0, szy = 0, xmax = 0, zmax = 0;
    bool many = false;
    double first_ratio = -1;
    std::vector<Row> rows;
    size_t i = 0;
    int ai = 0;
    while (i < recs.size()) {
        size_t j = i;
        while (j < recs.size() && recs[j]->L == recs[i]->L) ++j;
        if (ai < tmp.n_anchor && tmp.anchor_L[ai] == recs[i]->L) {
            for (size_t t = i; t < j; ++t)
                if (recs[t]->micro_id == tmp.anchor_micro[ai]) {
                    const double w = static_cast<double>(ceil_div64(recs[t]->G, cap));
                    rows.push_back(Row{w * static_cast<double>(recs[t]->L), w, recs[t]->mean_us});
                }
            ++ai;
        }
        i = j;
    }
    for (const Row& r : rows) {
        xmax = std::max(xmax, fabs(r.G));
        zmax = std::max(zmax, fabs(r.L));
        const double ratio = r.G / r.L;
        if (first_ratio < 0) first_ratio = ratio; else many |= (ratio != first_ratio);
    }
    *a_out = *b_out = 0.0;
    if (rows.empty()) return;
    for (const Row& r : rows) {
        const double x = r.G / xmax, z = r.L / zmax;
        sxx += x * x; sxz += x * z; szz += z * z; sxy += x * r.T; szy += z * r.T;
    }
    if (many) {
        const double det = sxx * szz - sxz * sxz;
        *a_out = ((sxy * szz - szy * sxz) / det) / xmax;
        *b_out = ((szy * sxx - sxy * sxz) / det) / zmax;
    } else {
        *b_out = (szy / szz) / zmax;
    }
}

// Buckets of one sample family: wave buckets 1..W plus the extrapolation entry from the last p waves,
// laid out as out[key * (W + 1) + (w - 1)] with the extrapolation entry last.
static int fit_family(const wt_ctx* ctx, int family, int model, int W, int p, bool relative, const wt_sample* s, size_t n,
                      std::vector<Bucket>& out) {
    const int nk = static_cast<int>(ctx->keys.size());
    out.assign(static_cast<size_t>(nk) * (W + 1), Bucket{});
    std::vector<std::vector<const wt_sample*>> by(static_cast<size_t>(nk) * W);
    for (size_t i = 0; i < n; ++i) {
        if (s[i].key_id < 0 || s[i].key_id >= nk) return WT_ERR_INVALID_ARG;
        if (s[i].family != family || s[i].w < 1 || s[i].w > W) continue;
        if (relative && !(s[i].mean_us > 0.0)) return WT_ERR_INVALID_ARG;   // a relative residual needs T > 0
        by[static_cast<size_t>(s[i].key_id) * W + (s[i].w - 1)].push_back(&s[i]);
    }
    const int first_ext = model == WT_MODEL_LINEAR ? 1 : std::max(1, W - p + 1);
    for (int k = 0; k < nk; ++k) {
        Bucket* kb = &out[static_cast<size_t>(k) * (W + 1)];
        std::vector<const wt_sample*> merged;
        if (model == WT_MODEL_STEP) {
            for (int w = 1; w <= W; ++w) {
                std::vector<const wt_sample*>& recs = by[static_cast<size_t>(k) * W + (w - 1)];
                merged.insert(merged.end(), recs.begin(), recs.end());
            }
            double a = 0, b = 0;
            Bucket anchors;
            const bool ok = !merged.empty();
            fit_step(merged, ctx->keys[k].cap, &a, &b, anchors);
            for (int w = 1; w <= W; ++w) {
                Bucket& bk = kb[w - 1];
                bk = anchors;
                bk.th[0] = 0; bk.th[1] = 0; bk.th[2] = a * w; bk.th[3] = b * w;
                bk.status = ok ? 0xC : 0;
            }
            Bucket& ex = kb[W];
            ex = anchors;
            const double cap = static_cast<double>(ctx->keys[k].cap);
            ex.th[0] = a / cap; ex.th[1] = b / cap; ex.th[2] = 0; ex.th[3] = 0;
            ex.status = ok ? 0x3 : 0;
            continue;
        }
        for (int w = 1; w <= W; ++w) {
            std::vector<const wt_sample*>& recs = by[static_cast<size_t>(k) * W + (w - 1)];
            if (w >= first_ext) merged.insert(merged.end(), recs.begin(), recs.end());
            if (model == WT_MODEL_WAVE_BILINEAR) fit_bucket(recs, kb[w - 1], relative);
        }
        fit_bucket(merged, kb[W], relative);
    }
    return WT_OK;
}

static int fit_table(wt_ctx* ctx, const wt_grid* grid, const wt_sample* s, size_t n) {
    const int W = grid->W;
    // the same bounds wt_load applies, so that every table that can be fitted and saved can be loaded again
    if (W < 1 || W > kMaxWaves || grid->I < 1 || grid->p < 1 || grid->W_row < 0 || grid->W_row > kMaxWaves) return WT_ERR_INVALID_ARG;
    if (grid->model < WT_MODEL_WAVE_BILINEAR || grid->model > WT_MODEL_STEP) return WT_ERR_INVALID_ARG;
    if (grid->weighting != WT_FIT_ABSOLUTE && grid->weighting != WT_FIT_RELATIVE) return WT_ERR_INVALID_ARG;
    const bool relative = grid->weighting == WT_FIT_RELATIVE;
    Table t;
    t.W = W; t.I = grid->I; t.p = grid->p; t.tau_num = grid->tau_num; t.tau_den = grid->tau_den;
    t.weighting = grid->weighting;
    int rc = fit_family(ctx, 0, grid->model, W, grid->p, relative, s, n, t.buckets);
    if (rc != WT_OK) return rc;
    if (grid->W_row > 0) {  // the few-row families always use the wave-bucketed bilinear model
        if (grid->row_mode != WT_ROWS_TILES && grid->row_mode != WT_ROWS_BAND) return WT_ERR_INVALID_ARG;
        if (grid->row_fams < 0 || grid->row_fams > (grid->row_mode == WT_ROWS_BAND ? 4 : 3)) return WT_ERR_INVALID_ARG;
        t.row_mode = grid->row_mode;
        t.W_row = grid->W_row;
        t.row_fams = grid->row_fams > 0 ? grid->row_fams : 1;
        for (int f = 1; f <= t.row_fams; ++f) {
            rc = fit_family(ctx, f, WT_MODEL_WAVE_BILINEAR, t.W_row, std::min(grid->p, t.W_row), relative, s, n, t.row_buckets[f - 1]);
            if (rc != WT_OK) return rc;
        }
    }
    t.fitted = true;
    ctx->table = std::move(t);
    return WT_OK;
}

// ---- two-stage selection (Sec. 4.4, 4.5) -------------------------------------------------------
// rows: the shape's row count M (one group's rows for a grouped launch).  Tile-row families are consulted per key by
// ceil(rows/bm); row-band families by the band rows falls in, the same under every key.
static inline const Bucket* pick_bucket(const Table& t, int key, int bm, int64_t w, int64_t rows) {
    const int fam = t.W_row <= 0 ? 0 : t.row_mode == WT_ROWS_BAND ? band_family(rows) : row_family(ceil_div64(rows, bm));
    if (fam >= 1 && fam <= t.row_fams) {  // few tile rows: that family's buckets first, the paper's as fallback
        const Bucket* rb = &t.row_buckets[fam - 1][static_cast<size_t>(key) * (t.W_row + 1)];
        if (w >= 1 && w <= t.W_row && rb[w - 1].status) return &rb[w - 1];
        if (rb[t.W_row].status) return &rb[t.W_row];
    }
    const Bucket* base = &t.buckets[static_cast<size_t>(key) * (t.W + 1)];
    if (w >= 1 && w <= t.W && base[w - 1].status) return &base[w - 1];
    return base[t.W].status ? &base[t.W] : nullptr;
}

// ((alpha*(G*L) + beta*G) + gamma*L) + delta, each operation rounded once (this file is compiled
// with -ffp-contract=off so no multiply-add is fused).
static inline double predict(const double th[4], int64_t G, int64_t L) {
    const double gl = static_cast<double>(G * L);
    const double g = static_cast<double>(G), l = static_cast<double>(L);
    double t = th[0] * gl;
    t = t + th[1] * g;
    t = t + th[2] * l;
    t = t + th[3];
    return t;
}

// Limits of the selectors that take per-part sizes: the part count the launches accept, totals that fit the int32
// offsets those launches read, and a G*L that cannot leave int64 (tiles <= rows, column tiles <= N, loops <= K).
static constexpr int kMaxSelectParts = 1024;
static constexpr int64_t kMaxSelectTokens = 0x7FFFFFFF;
static inline bool product_fits(int64_t a, int64_t b, int64_t c) {
    if (a <= 0 || b <= 0 || c <= 0) return true;
    return a <= ((int64_t{1} << 62) / b) / c;
}
// Every shape the selectors price must keep G*L inside int64 for every key: tiles <= M*N, at most 16 splits, L <= K.
static inline bool shape_fits(int64_t M, int64_t N, int64_t K) { return product_fits(M, N, K < 16 ? 16 : K); }

// The two stages over a pricing rule: phi(k, key, &G, &L, &rows) says whether key k is a candidate and, if so,
// gives its <G, L> and the row count that names its few-row family.  Stage I: strict '<', so ties keep the
// lowest key id.  Stage II: nearest loop anchor of the chosen bucket.
template <class Phi>
static int select_by(const wt_ctx* ctx, Phi&& phi, int* key_out, int* micro_out, double* t_out) {
    const Table& t = ctx->table;
    const int nk = static_cast<int>(ctx->keys.size());
    const Bucket* best_b = nullptr;
    double best_t = 0;
    int best_k = -1;
    int64_t best_L = 0;
    for (int k = 0; k < nk; ++k) {
        const Key& key = ctx->keys[k];
        int64_t G, L, rows;
        if (!phi(k, key, &G, &L, &rows)) continue;
        const int64_t w = (G + key.cap - 1) / key.cap;
        const Bucket* b = pick_bucket(t, k, key.bm, w, rows);
        if (!b) continue;
        const double th = predict(b->th, G, L);
        if (th != th) continue;
        if (best_k < 0 || th < best_t) { best_k = k; best_t = th; best_b = b; best_L = L; }
    }
    if (best_k < 0) return WT_ERR_NOT_FITTED;
    int micro = 0;
    if (best_b->n_anchor > 0) {
        // anchors ascend in L: binary search for the first anchor >= L*, then compare with its
        // left neighbour; equal distances keep the smaller anchor
        int lo = 0, hi = best_b->n_anchor;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (best_b->anchor_L[mid] < best_L) lo = mid + 1; else hi = mid;
        }
        int pick = lo;
        if (lo == best_b->n_anchor) pick = lo - 1;
        else if (lo > 0 && (best_L - best_b->anchor_L[lo - 1]) <= (best_b->anchor_L[lo] - best_L)) pick = lo - 1;
        micro = best_b->anchor_micro[pick];
    }
    *key_out = best_k;
    *micro_out = micro;
    if (t_out) *t_out = best_t;
    return WT_OK;
}

// groups = 0: dense GEMM of M rows.  groups > 0: grouped GEMM of M rows in total under the uniform
// approximation (Sec. 5.2, grouped-GEMM discussion: per-expert counts are not known on the host without
// a synchronisation): every group is taken to hold ceil(M/groups) rows, so G = groups * tiles of one
// group (Table 2, grouped row), looked up in the dense table (Sec. 4.2 reduces grouped sampling to the
// dense case).  Split-K keys do not run grouped launches and are skipped.
static int select_impl(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, int groups, int* key_out, int* micro_out,
                       double* t_out) {
    const int64_t Mg = groups > 0 ? ceil_div64(M, groups) : M;
    return select_by(ctx, [&](int, const Key& key, int64_t* G, int64_t* L, int64_t* rows) {
        int64_t tiles;
        key_phi(key, Mg, N, K, &tiles, G, L);
        if (groups > 0) {
            if (key.split != 1) return false;
            *G *= groups;
        } else if (!key_fits(key, tiles)) {
            return false;
        }
        *rows = Mg;
        return true;
    }, key_out, micro_out, t_out);
}

// Grouped GEMM with the real per-group row counts: G of Table 2's grouped row summed over the groups; the few-row
// family is that of the mean group, ceil(sum / groups) rows (the uniform reading when the groups are equal).
static int select_rows_impl(const wt_ctx* ctx, int groups, const int64_t* group_rows, int64_t N, int64_t K,
                            int* key_out, int* micro_out) {
    int64_t total = 0;
    for (int e = 0; e < groups; ++e) total += group_rows[e];
    const int64_t mean_rows = ceil_div64(total, groups);
    return select_by(ctx, [&](int, const Key& key, int64_t* G, int64_t* L, int64_t* rows) {
        if (key.split != 1) return false;
        int64_t g = 0, tiles, ge;
        for (int e = 0; e < groups; ++e) {
            key_phi(key, group_rows[e], N, K, &tiles, &ge, L);
            g += ge;
        }
        *G = g;
        *rows = mean_rows;
        return true;
    }, key_out, micro_out, nullptr);
}

// A ragged attention batch with the real per-sequence lengths (Table 2's attention row per sequence): G counts every
// block, L is the mean loop count over the blocks rounded half up, so G*L is the launch's number of key-tile
// iterations to within rounding.  No block at all: G = L = 0.
static int select_varlen_impl(const wt_ctx* ctx, int batch, const int64_t* len_q, const int64_t* len_kv,
                              int64_t n_heads, int* key_out, int* micro_out) {
    return select_by(ctx, [&](int, const Key& key, int64_t* G, int64_t* L, int64_t* rows) {
        int64_t t = 0, iters = 0;
        for (int b = 0; b < batch; ++b) {
            const int64_t tiles = (len_q[b] + key.bm - 1) >> key.sh_m;
            const int64_t loops = (len_kv[b] + (int64_t{1} << key.sh_k) - 1) >> key.sh_k;
            t += tiles;
            iters += tiles * loops;
        }
        *G = n_heads * t;
        *L = t ? (2 * iters + t) / (2 * t) : 0;
        *rows = 0;  // attention tables carry no few-row families
        return true;
    }, key_out, micro_out, nullptr);
}

// ---- table file ------------------------------------------------------------------------------------
// Little-endian.  Header: 16 uint32 = 'WTDT', version (1; 2 with the single-tile-row family; 3 with several
// tile-row families; 4 with row-band families), n_keys, W, I, p, tau_num, tau_den, n_cu, anchor slots A, in_type, out_type, key_mode
// (capacity mode), W_row (version >= 2), row_fams (versions 3, 4), fit objective.  Per key: 8 int32 (bm, bn, bk, nwave, stages, occ,
// n_micro, split [0 in older files = 1]), int64 cap (256, or 256*occ when key_mode = 0), then a bucket block of R = W+1 rows
// (w = 1..W then ext): R*4 float64 theta, R int32 status, R int32 n_anchor, R*A int32 anchor L,
// R*A int32 anchor micro; versions 2 to 4 append one block of W_row+1 rows per few-row family.
static const uint32_t kMagic = 0x54445457u;  // "WTDT"

static bool write_block(FILE* f, const Bucket* b, int R) {
    bool ok = true;
    for (int r = 0; ok && r < R; ++r) ok = fwrite(b[r].th, sizeof(double), 4, f) == 4;
    for (int r = 0; ok && r < R; ++r) ok = fwrite(&b[r].status, sizeof(int32_t), 1, f) == 1;
    for (int r = 0; ok && r < R; ++r) ok = fwrite(&b[r].n_anchor, sizeof(int32_t), 1, f) == 1;
    for (int r = 0; ok && r < R; ++r) ok = fwrite(b[r].anchor_L, sizeof(int32_t), kMaxAnchors, f) == kMaxAnchors;
    for (int r = 0; ok && r < R; ++r) ok = fwrite(b[r].anchor_micro, sizeof(int32_t), kMaxAnchors, f) == kMaxAnchors;
    return ok;
}

static bool read_block(FILE* f, Bucket* b, int R) {
    bool ok = true;
    for (int r = 0; ok && r < R; ++r) ok = fread(b[r].th, sizeof(double), 4, f) == 4;
    for (int r = 0; ok && r < R; ++r) ok = fread(&b[r].status, sizeof(int32_t), 1, f) == 1;
    for (int r = 0; ok && r < R; ++r) ok = fread(&b[r].n_anchor, sizeof(int32_t), 1, f) == 1;
    for (int r = 0; ok && r < R; ++r) ok = fread(b[r].anchor_L, sizeof(int32_t), kMaxAnchors, f) == kMaxAnchors;
    for (int r = 0; ok && r < R; ++r) ok = fread(b[r].anchor_micro, sizeof(int32_t), kMaxAnchors, f) == kMaxAnchors;
    for (int r = 0; ok && r < R; ++r) ok = b[r].n_anchor >= 0 && b[r].n_anchor <= kMaxAnchors;
    return ok;
}

static int save_table(const wt_ctx* ctx, const char* path) {
    const Table& t = ctx->table;
    if (!t.fitted) return WT_ERR_NOT_FITTED;
    FILE* f = fopen(path, "wb");
    if (!f) return WT_ERR_IO;
    const uint32_t nk = static_cast<uint32_t>(ctx->keys.size());
    const uint32_t hdr[16] = {kMagic, t.W_row > 0 ? (t.row_mode == WT_ROWS_BAND ? 4u : t.row_fams > 1 ? 3u : 2u) : 1u, nk, static_cast<uint32_t>(t.W), static_cast<uint32_t>(t.I),
                              static_cast<uint32_t>(t.p), static_cast<uint32_t>(t.tau_num),
                              static_cast<uint32_t>(t.tau_den), static_cast<uint32_t>(kNumCU),
                              static_cast<uint32_t>(kMaxAnchors), static_cast<uint32_t>(ctx->in_type),
                              static_cast<uint32_t>(ctx->out_type), static_cast<uint32_t>(ctx->cap_mode),
                              static_cast<uint32_t>(t.W_row), static_cast<uint32_t>(t.row_fams), static_cast<uint32_t>(t.weighting)};
    bool ok = fwrite(hdr, sizeof(hdr), 1, f) == 1;
    const int R = t.W + 1;
    for (uint32_t k = 0; ok && k < nk; ++k) {
        const Key& key = ctx->keys[k];
        const int32_t kd[8] = {key.bm, key.bn, key.bk, key.nwave, key.stages, key.occ, key.n_micro, key.split};
        ok = ok && fwrite(kd, sizeof(kd), 1, f) == 1;
        ok = ok && fwrite(&key.cap, sizeof(int64_t), 1, f) == 1;
        ok = ok && write_block(f, &t.buckets[static_cast<size_t>(k) * R], R);
        for (int fam = 0; fam < t.row_fams; ++fam)
            ok = ok && write_block(f, &t.row_buckets[fam][static_cast<size_t>(k) * (t.W_row + 1)], t.W_row + 1);
    }
    ok = (fclose(f) == 0) && ok;
    return ok ? WT_OK : WT_ERR_IO;
}

static int load_table(wt_ctx* ctx, const char* path) {
    FILE* f = fopen(path, "rb");
    if (!f) return WT_ERR_IO;
    uint32_t hdr[16];
    int rc = WT_OK;
    Table t;
    std::vector<int> occs;
    if (fread(hdr, sizeof(hdr), 1, f) != 1 || hdr[0] != kMagic || hdr[1] < 1u || hdr[1] > 4u) rc = WT_ERR_IO;
    if (rc == WT_OK && hdr[1] == 1u) hdr[13] = 0;
    if (rc == WT_OK) hdr[14] = hdr[13] == 0 ? 0u : (hdr[1] >= 3u ? hdr[14] : 1u);
    if (rc == WT_OK && hdr[14] > (hdr[1] == 4u ? 4u : 3u)) rc = WT_ERR_INVALID_ARG;
    if (rc == WT_OK && hdr[1] == 4u && hdr[14] == 0) rc = WT_ERR_INVALID_ARG;  // version 4 means row-band families are present
    if (rc == WT_OK && hdr[13] > static_cast<uint32_t>(kMaxWaves)) rc = WT_ERR_INVALID_ARG;
    if (rc == WT_OK && (hdr[2] != ctx->keys.size() || hdr[9] != static_cast<uint32_t>(kMaxAnchors) ||
                        hdr[8] != static_cast<uint32_t>(kNumCU) || hdr[10] != static_cast<uint32_t>(ctx->in_type) ||
                        hdr[11] != static_cast<uint32_t>(ctx->out_type) || hdr[3] < 1 ||
                        hdr[3] > static_cast<uint32_t>(kMaxWaves) || hdr[12] > 1u || hdr[15] > 1u))
        rc = WT_ERR_INVALID_ARG;  // table was built for another registry, device size or storage type
    if (rc == WT_OK) {
        t.W = static_cast<int>(hdr[3]); t.I = static_cast<int>(hdr[4]); t.p = static_cast<int>(hdr[5]);
        t.tau_num = static_cast<int>(hdr[6]); t.tau_den = static_cast<int>(hdr[7]);
        const int R = t.W + 1;
        t.W_row = static_cast<int>(hdr[13]);
        t.weighting = static_cast<int>(hdr[15]);
        t.row_fams = static_cast<int>(hdr[14]);
        t.row_mode = hdr[1] == 4u ? WT_ROWS_BAND : WT_ROWS_TILES;
        t.buckets.assign(ctx->keys.size() * R, Bucket{});
        for (int fam = 0; fam < t.row_fams; ++fam) t.row_buckets[fam].assign(ctx->keys.size() * (t.W_row + 1), Bucket{});
        for (size_t k = 0; rc == WT_OK && k < ctx->keys.size(); ++k) {
            int32_t kd[8];
            int64_t cap;
            if (fread(kd, sizeof(kd), 1, f) != 1 || fread(&cap, sizeof(cap), 1, f) != 1) { rc = WT_ERR_IO; break; }
            const Key& key = ctx->keys[k];
            if (kd[0] != key.bm || kd[1] != key.bn || kd[2] != key.bk || kd[3] != key.nwave || kd[4] != key.stages ||
                (kd[7] < 1 ? 1 : kd[7]) != key.split || kd[5] < 1 || cap != key_capacity(static_cast<int>(hdr[12]), kd[5])) { rc = WT_ERR_INVALID_ARG; break; }
            occs.push_back(kd[5]);
            bool ok = read_block(f, &t.buckets[k * R], R);
            for (int fam = 0; ok && fam < t.row_fams; ++fam) ok = read_block(f, &t.row_buckets[fam][k * (t.W_row + 1)], t.W_row + 1);
            if (!ok) rc = WT_ERR_IO;
        }
        // the header's sizes must account for every byte: a file longer than they say was written under other ones
        if (rc == WT_OK && fgetc(f) != EOF) rc = WT_ERR_IO;
    }
    fclose(f);
    if (rc != WT_OK) return rc;
    // the table's wave boundaries are those of the occupancy it was profiled with
    ctx->cap_mode = static_cast<int>(hdr[12]);
    for (size_t k = 0; k < ctx->keys.size(); ++k) {
        ctx->keys[k].occ = occs[k];
        ctx->keys[k].cap = key_capacity(ctx->cap_mode, occs[k]);
        for (int m = 0; m < ctx->keys[k].n_micro; ++m) ctx->cfgs[ctx->keys[k].first_cfg + m].res.occ = occs[k];
    }
    t.fitted = true;
    ctx->table = std::move(t);
    return WT_OK;
}

}  // namespace wt

// ===== C ABI (host-only entry points) ==================================================================
using namespace wt;

extern "C" {

const char* wt_status_string(int s) {
    switch (s) {
        case WT_OK: return "ok";
        case WT_ERR_INVALID_ARG: return "invalid argument";
        case WT_ERR_UNSUPPORTED_CFG: return "configuration not in the registry";
        case WT_ERR_INFEASIBLE: return "configuration does not fit the device or the split-K workspace";
        case WT_ERR_NOT_FITTED: return "no dual table (call wt_fit or wt_load)";
        case WT_ERR_HIP: return "HIP call failed";
        case WT_ERR_BUFFER_TOO_SMALL: return "buffer too small";
        case WT_ERR_IO: return "file error";
        case WT_ERR_NO_DEVICE: return "host-only context";
        case WT_ERR_NO_MEMORY: return "out of host memory";
        default: return "unknown status";
    }
}

int wt_last_hip_error(const wt_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int wt_config_count(const wt_ctx* ctx, int* n) {
    if (!ctx || !n) return WT_ERR_INVALID_ARG;
    *n = static_cast<int>(ctx->cfgs.size());
    return WT_OK;
}

int wt_key_count(const wt_ctx* ctx, int* n) {
    if (!ctx || !n) return WT_ERR_INVALID_ARG;
    *n = static_cast<int>(ctx->keys.size());
    return WT_OK;
}

int wt_config_get(const wt_ctx* ctx, int i, wt_cfg* cfg, wt_cfg_res* res) {
    if (!ctx || i < 0 || i >= static_cast<int>(ctx->cfgs.size())) return WT_ERR_INVALID_ARG;
    if (cfg) *cfg = ctx->cfgs[i].cfg;
    if (res) *res = ctx->cfgs[i].res;
    return WT_OK;
}

int wt_config_find(const wt_ctx* ctx, const wt_cfg* fields, int* id) {
    if (!ctx || !fields || !id) return WT_ERR_INVALID_ARG;
    wt_cfg c = *fields;
    c.id = -1;
    const int i = find_config(ctx, c);
    if (i < 0) return WT_ERR_UNSUPPORTED_CFG;
    *id = i;
    return WT_OK;
}

int wt_key_set_occ(wt_ctx* ctx, int key_id, int occ) {
    if (!ctx || key_id < 0 || key_id >= static_cast<int>(ctx->keys.size()) || occ < 1) return WT_ERR_INVALID_ARG;
    Key& k = ctx->keys[key_id];
    k.occ = occ;
    k.cap = key_capacity(ctx->cap_mode, occ);
    for (int m = 0; m < k.n_micro; ++m) ctx->cfgs[k.first_cfg + m].res.occ = occ;
    return WT_OK;
}

int wt_set_capacity_mode(wt_ctx* ctx, int mode) {
    if (!ctx || (mode != WT_CAP_CU_TIMES_OCC && mode != WT_CAP_CU_ONLY)) return WT_ERR_INVALID_ARG;
    ctx->cap_mode = mode;
    for (Key& k : ctx->keys) k.cap = key_capacity(mode, k.occ);
    ctx->table = Table();
    return WT_OK;
}

int wt_wave_count(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, wt_cfg cfg, int64_t* G, int64_t* L,
                  int32_t* w) {
    if (!ctx || M < 0 || N < 0 || K < 0 || !shape_fits(M, N, K)) return WT_ERR_INVALID_ARG;
    const int id = find_config(ctx, cfg);
    if (id < 0) return WT_ERR_UNSUPPORTED_CFG;
    const Key& k = ctx->keys[ctx->cfgs[id].res.key_id];
    int64_t tiles, g, l;
    key_phi(k, M, N, K, &tiles, &g, &l);
    if (G) *G = g;
    if (L) *L = l;
    if (w) *w = static_cast<int32_t>(ceil_div64(g, k.cap));
    return WT_OK;
}

int wt_sample_grid(int64_t capacity, int32_t W, int32_t I, int32_t tau_num, int32_t tau_den, int32_t split,
                   int64_t* g, int64_t* m, int64_t* n, size_t cap_out, size_t* n_out) {
    if (capacity < 1 || W < 1 || W > kMaxWaves || I < 1 || I > kMaxSubIntervals || tau_num < tau_den || tau_den < 1 ||
        split < 1 || !n_out)
        return WT_ERR_INVALID_ARG;
    WT_GUARD([&]() -> int {
        std::vector<GridPoint> pts;
        sample_grid(capacity, W, I, tau_num, tau_den, split, pts);
        *n_out = pts.size();
        if (pts.size() > cap_out) return WT_ERR_BUFFER_TOO_SMALL;
        for (size_t i = 0; i < pts.size(); ++i) {
            if (g) g[i] = pts[i].g;
            if (m) m[i] = pts[i].m;
            if (n) n[i] = pts[i].n;
        }
        return WT_OK;
    }());
}

int wt_sample_grid_heads(int64_t capacity, int32_t W, int32_t I, int32_t n_heads, int64_t* g, int64_t* q_tiles,
                         size_t cap_out, size_t* n_out) {
    if (capacity < 1 || W < 1 || W > kMaxWaves || I < 1 || I > kMaxSubIntervals || n_heads < 1 || !n_out)
        return WT_ERR_INVALID_ARG;
    WT_GUARD([&]() -> int {
        std::vector<GridPoint> pts;
        sample_grid_heads(capacity, W, I, n_heads, pts);
        *n_out = pts.size();
        if (pts.size() > cap_out) return WT_ERR_BUFFER_TOO_SMALL;
        for (size_t i = 0; i < pts.size(); ++i) {
            if (g) g[i] = pts[i].g;
            if (q_tiles) q_tiles[i] = pts[i].m;
        }
        return WT_OK;
    }());
}

int wt_fit(wt_ctx* ctx, const wt_grid* grid, const wt_sample* samples, size_t n) {
    if (!ctx || !grid || (!samples && n)) return WT_ERR_INVALID_ARG;
    WT_GUARD(fit_table(ctx, grid, samples, n));
}

int wt_select(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, wt_cfg* out) {
    if (!ctx || !out || M < 0 || N < 0 || K < 0 || !shape_fits(M, N, K)) return WT_ERR_INVALID_ARG;
    if (!ctx->table.fitted) return WT_ERR_NOT_FITTED;
    int key, micro;
    const int rc = select_impl(ctx, M, N, K, 0, &key, &micro, nullptr);
    if (rc != WT_OK) return rc;
    const Key& k = ctx->keys[key];
    if (micro < 0 || micro >= k.n_micro) micro = 0;
    *out = ctx->cfgs[k.first_cfg + micro].cfg;
    return WT_OK;
}

int wt_select_grouped(const wt_ctx* ctx, int32_t groups, int64_t M_total, int64_t N, int64_t K, wt_cfg* out) {
    if (!ctx || !out || groups < 1 || M_total < 0 || N < 0 || K < 0 || !shape_fits(M_total + groups, N, K))
        return WT_ERR_INVALID_ARG;
    if (!ctx->table.fitted) return WT_ERR_NOT_FITTED;
    int key, micro;
    const int rc = select_impl(ctx, M_total, N, K, groups, &key, &micro, nullptr);
    if (rc != WT_OK) return rc;
    const Key& k = ctx->keys[key];
    if (micro < 0 || micro >= k.n_micro) micro = 0;
    *out = ctx->cfgs[k.first_cfg + micro].cfg;
    return WT_OK;
}

int wt_select_grouped_rows(const wt_ctx* ctx, int32_t groups, const int64_t* group_rows, int64_t N, int64_t K,
                           wt_cfg* out) {
    if (!ctx || !out || groups < 1 || groups > kMaxSelectParts || !group_rows || N < 0 || K < 0 ||
        ctx->in_type == WT_ATTN_BF16)
        return WT_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int e = 0; e < groups; ++e) {
        if (group_rows[e] < 0 || group_rows[e] > kMaxSelectTokens - total) return WT_ERR_INVALID_ARG;
        total += group_rows[e];
    }
    if (!shape_fits(total + groups, N, K)) return WT_ERR_INVALID_ARG;
    if (!ctx->table.fitted) return WT_ERR_NOT_FITTED;
    int key, micro;
    const int rc = select_rows_impl(ctx, groups, group_rows, N, K, &key, &micro);
    if (rc != WT_OK) return rc;
    const Key& k = ctx->keys[key];
    if (micro < 0 || micro >= k.n_micro) micro = 0;
    *out = ctx->cfgs[k.first_cfg + micro].cfg;
    return WT_OK;
}

int wt_select_attn_varlen(const wt_ctx* ctx, int32_t batch, const int64_t* len_q, const int64_t* len_kv,
                          int64_t n_heads, wt_cfg* out) {
    if (!ctx || !out || batch < 1 || batch > kMaxSelectParts || !len_q || !len_kv || n_heads < 1 || n_heads > 65536 ||
        ctx->in_type != WT_ATTN_BF16)
        return WT_ERR_INVALID_ARG;
    int64_t tq = 0, tkv = 0;
    for (int b = 0; b < batch; ++b) {
        if (len_q[b] < 0 || len_kv[b] < 0 || len_q[b] > kMaxSelectTokens - tq || len_kv[b] > kMaxSelectTokens - tkv)
            return WT_ERR_INVALID_ARG;
        tq += len_q[b];
        tkv += len_kv[b];
    }
    if (!product_fits(n_heads, tq, tkv)) return WT_ERR_INVALID_ARG;
    if (!ctx->table.fitted) return WT_ERR_NOT_FITTED;
    int key, micro;
    const int rc = select_varlen_impl(ctx, batch, len_q, len_kv, n_heads, &key, &micro);
    if (rc != WT_OK) return rc;
    const Key& k = ctx->keys[key];
    if (micro < 0 || micro >= k.n_micro) micro = 0;
    *out = ctx->cfgs[k.first_cfg + micro].cfg;
    return WT_OK;
}

int wt_wave_count_grouped(const wt_ctx* ctx, int32_t groups, const int64_t* group_rows, int64_t N, int64_t K,
                          wt_cfg cfg, int64_t* G, int64_t* L, int32_t* w) {
    if (!ctx || groups < 1 || !group_rows || N < 0 || K < 0) return WT_ERR_INVALID_ARG;
    const int id = find_config(ctx, cfg);
    if (id < 0) return WT_ERR_UNSUPPORTED_CFG;
    const Key& k = ctx->keys[ctx->cfgs[id].res.key_id];
    if (k.split != 1) return WT_ERR_UNSUPPORTED_CFG;
    int64_t g = 0, l = 0, total = 0;
    for (int e = 0; e < groups; ++e) {
        if (group_rows[e] < 0 || group_rows[e] > kMaxSelectTokens - total) return WT_ERR_INVALID_ARG;
        total += group_rows[e];
    }
    if (!shape_fits(total + groups, N, K)) return WT_ERR_INVALID_ARG;
    for (int e = 0; e < groups; ++e) {
        int64_t tiles, ge;
        key_phi(k, group_rows[e], N, K, &tiles, &ge, &l);
        g += ge;
    }
    if (G) *G = g;
    if (L) *L = l;
    if (w) *w = static_cast<int32_t>(ceil_div64(g, k.cap));
    return WT_OK;
}

int wt_predict_us(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, wt_cfg cfg, double* us) {
    if (!ctx || !us || M < 0 || N < 0 || K < 0 || !shape_fits(M, N, K)) return WT_ERR_INVALID_ARG;
    if (!ctx->table.fitted) return WT_ERR_NOT_FITTED;
    const int id = find_config(ctx, cfg);
    if (id < 0) return WT_ERR_UNSUPPORTED_CFG;
    const int kid = ctx->cfgs[id].res.key_id;
    const Key& k = ctx->keys[kid];
    int64_t tiles, G, L;
    key_phi(k, M, N, K, &tiles, &G, &L);
    if (!key_fits(k, tiles)) return WT_ERR_INFEASIBLE;
    const Bucket* b = pick_bucket(ctx->table, kid, k.bm, ceil_div64(G, k.cap), M);
    if (!b) return WT_ERR_NOT_FITTED;
    *us = predict(b->th, G, L);
    return WT_OK;
}

int wt_select_bench(const wt_ctx* ctx, const int64_t* shapes, size_t n, int repeats, double* mean_ns,
                    double* p99_ns) {
    if (!ctx || !shapes || n == 0 || repeats < 1) return WT_ERR_INVALID_ARG;
    if (!ctx->table.fitted) return WT_ERR_NOT_FITTED;
    std::vector<double> per;
    try {
        per.assign(n, 0.0);
    } catch (...) {
        return WT_ERR_NO_MEMORY;
    }
    volatile int sink = 0;
    double total = 0;
    for (int r = 0; r < repeats; ++r) {
        for (size_t i = 0; i < n; ++i) {
            wt_cfg c;
            const auto t0 = std::chrono::steady_clock::now();
            const int rc = wt_select(ctx, shapes[3 * i], shapes[3 * i + 1], shapes[3 * i + 2], &c);
            const auto t1 = std::chrono::steady_clock::now();
            if (rc != WT_OK) return rc;
            sink = sink + c.id;
            const double ns = std::chrono::duration<double, std::nano>(t1 - t0).count();
            per[i] = (r == 0) ? ns : std::min(per[i], ns);
            total += ns;
        }
    }
    // mean over every timed call; p99 over shapes of each shape's best repeat (removes scheduler noise)
    if (mean_ns) *mean_ns = total / (static_cast<double>(n) * repeats);
    if (p99_ns) {
        std::sort(per.begin(), per.end());
        *p99_ns = per[std::min(n - 1, static_cast<size_t>(0.99 * static_cast<double>(n)))];
    }
    return WT_OK;
}

int wt_save(const wt_ctx* ctx, const char* path) {
    if (!ctx || !path) return WT_ERR_INVALID_ARG;
    WT_GUARD(save_table(ctx, path));
}

int wt_load(wt_ctx* ctx, const char* path) {
    if (!ctx || !path) return WT_ERR_INVALID_ARG;
    WT_GUARD(load_table(ctx, path));
}

}  // extern "C"
