// Internal data model of libwt (host side).  Not part of the ABI.
#pragma once

#include <stdint.h>

#include <new>
#include <stdexcept>
#include <vector>

#include "../../include/wt.h"
#include "registry.hpp"

namespace wt {

constexpr int kNumCU = 256;            // compute units of one MI355X
constexpr int kLdsPerCU = 160 * 1024;  // bytes
constexpr int kNumSwizzle = 3;         // micro parameter values 0..2
constexpr int kMaxAnchors = WT_MAX_ANCHORS;  // loop anchors stored per bucket
constexpr int kMaxWaves = 4096;         // largest W (and W_row) of a table or a sample grid
constexpr int kMaxSubIntervals = 4096;  // largest I of a sample grid
constexpr int kMaxRowFams = 4;         // few-row sample families: 1, 2, 4 tile rows (three), or 16, 32, 64, 128 rows (four)
constexpr int kRowBand0 = 16;          // rows of the first row-band family; each further family doubles them
// Family consulted for a shape with `rows` = ceil(M/bm) tile rows: 1 -> 1, 2..3 -> 2, 4..7 -> 3, else 0.
inline int row_family(int64_t rows) { return rows <= 1 ? 1 : rows <= 3 ? 2 : rows <= 7 ? 3 : 0; }
// Row-band families: the family of the smallest band (16, 32, 64, 128 rows) that holds M; 0 above the last band.
inline int band_family(int64_t M) {
    for (int f = 1; f <= 4; ++f)
        if (M <= (int64_t{kRowBand0} << (f - 1))) return f;
    return 0;
}
// Split-K workspace owned by a context: fp32 partial tiles and one arrival counter per output tile.
constexpr int64_t kWsElems = WT_SPLITK_WS_FLOATS;        // 256 MiB of floats
constexpr int64_t kMaxSplitTiles = WT_SPLITK_MAX_TILES;  // arrival counters

struct Config {
    wt_cfg cfg;
    wt_cfg_res res;
    int wm, wn;
    const void* fn;
    const void* fn_persistent;
    int occ_persistent = 1;  // resident blocks per CU of the persistent kernel (its grid is 256 x this)
    int lds_persistent = 0;  // its dynamic LDS bytes
};

struct Key {
    int bm, bn, bk, nwave, stages;
    int split;             // S: blocks per output tile along K (1 = no split); a power of two
    int sh_m, sh_n, sh_k;  // log2 of bm, bn and of split*bk (all powers of two)
    int sh_s;              // log2 of split
    int occ;
    int64_t cap;  // kNumCU * occ
    int n_micro;
    int first_cfg;
    int lds_bytes;
    int vgprs;
};

struct Bucket {
    double th[4];  // alpha, beta, gamma, delta
    int32_t status;  // 0 = no model; else bit0..3 = alpha..delta identified
    int32_t n_anchor;
    int32_t anchor_L[kMaxAnchors];
    int32_t anchor_micro[kMaxAnchors];
};

struct Table {
    bool fitted = false;
    int W = 0, I = 0, p = 0, tau_num = 11, tau_den = 10;
    int weighting = 0;   // wt_weighting the buckets were fitted with (recorded in the table file; lookups do not use it)
    int row_mode = 0;    // wt_row_mode of the few-row families (meaningful when W_row > 0)
    // buckets[key * (W + 1) + (w - 1)] for w = 1..W; index W is the extrapolation entry
    std::vector<Bucket> buckets;
    // few-row families (extension) f = 1..row_fams, grids of 1, 2, 4 tile rows:
    // row_buckets[f - 1][key * (W_row + 1) + (w - 1)], last = extrapolation
    int W_row = 0;
    int row_fams = 0;
    std::vector<Bucket> row_buckets[kMaxRowFams];
};

}  // namespace wt

// No exception crosses the ABI: entry points that allocate host memory evaluate their body inside this guard.
#define WT_GUARD(expr)                    \
    try {                                 \
        return (expr);                    \
    } catch (const std::bad_alloc&) {     \
        return WT_ERR_NO_MEMORY;          \
    } catch (const std::length_error&) {  \
        return WT_ERR_NO_MEMORY;          \
    } catch (...) {                       \
        return WT_ERR_INVALID_ARG;        \
    }

struct wt_ctx {
    int device = -1;
    int in_type = 0, out_type = 0;
    int last_hip = 0;
    int cap_mode = WT_CAP_CU_ONLY;  // wt_cap_mode
    int persistent = 0;             // 1, 2: launches clamp the grid to the resident block count (2: tasks from a queue)
    int* queue = nullptr;           // two ints behind the split-K counters: the persistent kernels' task queue
    std::vector<wt::Config> cfgs;
    std::vector<wt::Key> keys;
    wt::Table table;
    void* ev_start = nullptr;  // hipEvent_t pair used by the timing calls
    void* ev_stop = nullptr;
    float* ws = nullptr;       // device: split-K partial tiles (kWsElems floats), then the counters
    int* counters = nullptr;   // device: kMaxSplitTiles ints, zero between launches
    void* static_scratch = nullptr;  // device: this GPU's copy of the library's static scratch array (wt_gemm_noalloc)
};

namespace wt {

// host-side pieces (wt_host.cpp)
int build_registry(wt_ctx* ctx);  // fills cfgs/keys from the compiled kernel lists; static occupancy
int static_occupancy(int lds_bytes, int nwave, int acc_vgprs);
inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t key_capacity(int cap_mode, int occ) {
    return cap_mode == WT_CAP_CU_ONLY ? kNumCU : static_cast<int64_t>(kNumCU) * (occ > 0 ? occ : 1);
}
int find_config(const wt_ctx* ctx, const wt_cfg& c);
// Phi of a structural key (Table 2, dense GEMM row; split-K makes S tasks per output tile, each
// walking ceil(K / (S*bk)) k-tiles).
inline void key_phi(const Key& k, int64_t M, int64_t N, int64_t K, int64_t* tiles, int64_t* G, int64_t* L) {
    const int64_t t = ((M + k.bm - 1) >> k.sh_m) * ((N + k.bn - 1) >> k.sh_n);
    *tiles = t;
    *G = t << k.sh_s;
    *L = (K + (int64_t{1} << k.sh_k) - 1) >> k.sh_k;
}
// A split-K key can run a shape only if its partial tiles fit the context's workspace.
inline bool key_fits(const Key& k, int64_t tiles) {
    return k.split == 1 || (tiles <= kMaxSplitTiles && ((tiles << k.sh_s) << (k.sh_m + k.sh_n)) <= kWsElems);
}

struct GridPoint {
    int64_t g, m, n;
};
void sample_grid(int64_t cap, int W, int I, int tau_num, int tau_den, int split, std::vector<GridPoint>& out);
void loop_anchors(const wt_grid* grid, int bk_eff, std::vector<int64_t>& out);
void sample_grid_heads(int64_t cap, int W, int I, int n_heads, std::vector<GridPoint>& out);
void kv_loop_anchors(const wt_grid* grid, int64_t S_q, int t_kv, std::vector<int64_t>& out);

}  // namespace wt
