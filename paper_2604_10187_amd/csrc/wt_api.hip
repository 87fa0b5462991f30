// Device half of the C ABI: context creation, GEMM launch, event timing, sparse profiling.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "attn_kernel.hpp"
#include "gemm_kernel.hpp"
#include "wt_internal.hpp"

using namespace wt;

// Device memory for callers that cannot allocate (wt_gemm_noalloc): split-K partial tiles, then the arrival
// counters.  Every GPU the library runs on holds its own copy until the process ends.  In host code the name
// `scratch` is only a handle for hipGetSymbolAddress; the address each device uses is in g_scratch_ptr[device].
constexpr size_t kStaticWsFloats = WT_NOALLOC_WS_FLOATS;
constexpr size_t kStaticTiles = WT_NOALLOC_MAX_TILES;
constexpr size_t kStaticBytes = kStaticWsFloats * sizeof(float) + kStaticTiles * sizeof(int);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // per device: address of that device's copy of `scratch`

// Called with `device` current (wt_create).  Returns the device's address of the static array, or NULL with the
// HIP error in *err.
void* static_scratch_for(int device, hipError_t* err) {
    *err = hipSuccess;
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            *err = e != hipSuccess ? e : hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}

// Arrival counters of the tiles a launch is about to use, set to zero on the launch's stream (a kernel, not a
// memset node: the call may be under graph capture).
__global__ void zero_ints(int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Where a launch keeps its split-K partial tiles and counters, and how much room there is.
struct Workspace {
    float* ws;
    int* counters;
    int64_t ws_elems, max_tiles;
};

#define WT_HIP(ctx, call)                     \
    do {                                      \
        hipError_t e_ = (call);               \
        if (e_ != hipSuccess) {               \
            (ctx)->last_hip = (int)e_;        \
            return WT_ERR_HIP;                \
        }                                     \
    } while (0)

// Largest K for which BM*K*esize stays below the buffer-offset sentinel for every tile height.
constexpr int64_t kMaxK = 1 << 21;
constexpr int64_t kMaxDim = 1 << 30;
constexpr double kMinTimedUs = 300.0;  // shortest event-timed batch that is trusted

int validate_shape(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return WT_ERR_INVALID_ARG;
    const int vec = ctx->in_type == WT_BF16 ? 8 : 16;
    if (K % vec) return WT_ERR_INVALID_ARG;
    return WT_OK;
}

// One GEMM problem as the launch code sees it; groups == 0 is the dense case.
struct Problem {
    int64_t M, N, K;
    const void* A;
    const void* B;
    void* C;
    const float* sA;
    const float* sB;
    int groups = 0;
    const int32_t* offsets = nullptr;  // device, groups + 1 entries
    // attention contexts: (M, N, K) = (S_q, H_q, S_kv), A = Q, B = K, C = O
    const void* V = nullptr;
    int64_t H_kv = 0;
    float scale = 0.0f;
    int causal = 0;
    int64_t batch = 1;   // sequences per attention launch
    const int32_t* cu_q = nullptr;    // variable-length batch: device, batch + 1 token offsets into Q / O (M = total)
    const int32_t* cu_kv = nullptr;   //                        ... into K / V (K = total)
};

constexpr int64_t kMaxSeq = 1 << 22;  // S_q, S_kv: row offsets times heads times 128 stay far below 2^63, block ids below 2^31

int launch_attn(wt_ctx* ctx, const Config& c, const Problem& p, hipStream_t stream) {
    if (p.M == 0 || p.N == 0) return WT_OK;
    // variable-length batch: every sequence may end in a partial query tile, so the grid is sized for
    // ceil(total / T_Q) + batch tiles per head and the blocks past the last real tile exit at once
    const int64_t q_tiles = ceil_div64(p.M, c.cfg.bm) + (p.cu_q ? p.batch : 0);
    const int64_t G = q_tiles * p.N * (p.cu_q ? 1 : p.batch);
    if (G > 0x7FFFFFFF || p.batch * p.N > 0x7FFFFFFF) return WT_ERR_INVALID_ARG;
    AttnArgs a;
    a.batch = (int)p.batch;
    a.cu_q = p.cu_q; a.cu_kv = p.cu_kv;
    a.Q = static_cast<const __bf16*>(p.A); a.K = static_cast<const __bf16*>(p.B);
    a.V = static_cast<const __bf16*>(p.V); a.O = static_cast<__bf16*>(p.C);
    a.S_q = (int)p.M; a.S_kv = (int)p.K; a.H_q = (int)p.N; a.H_kv = (int)p.H_kv;
    a.q_tiles = (int)q_tiles;
    // Causal launches: blocks differ in length, and starting every head's longest query tiles first (order 1 on
    // the reversed tile index) balances the tail; measured best or within 0.5 % of best on every test shape, so
    // the order cached from unmasked profiling is not consulted.
    a.order = p.causal ? 1 : c.cfg.swizzle;
    a.causal = p.causal;
    a.scale_log2 = p.scale * 1.4426950408889634f;
    void* params[] = {&a};
    WT_HIP(ctx, hipLaunchKernel(c.fn, dim3((unsigned)G), dim3((unsigned)(c.cfg.nwave * 64)), params,
                                (size_t)c.res.lds_bytes, stream));
    return WT_OK;
}

constexpr int kMaxGroups = 1024;
constexpr int64_t kStreamCBytes = 128ll << 20;

int launch(wt_ctx* ctx, const Config& c, const Problem& p, hipStream_t stream, const Workspace* alt = nullptr) {
    if (ctx->in_type == WT_ATTN_BF16) return launch_attn(ctx, c, p, stream);
    const Workspace own{ctx->ws, ctx->counters, kWsElems, kMaxSplitTiles};
    const Workspace& W = alt ? *alt : own;
    const Key& key = ctx->keys[c.res.key_id];
    int64_t tiles_m = ceil_div64(p.M, c.cfg.bm);
    const int64_t tiles_n = ceil_div64(p.N, c.cfg.bn);
    if (p.M == 0 || p.N == 0) return WT_OK;
    if (p.groups > 0) {
        if (key.split != 1) return WT_ERR_UNSUPPORTED_CFG;  // grouped launches do not split K
        tiles_m += p.groups;  // every group may end in a partial row tile; surplus blocks exit at once
    }
    const int64_t tiles = tiles_m * tiles_n, G = tiles << key.sh_s;
    if (G > 0x7FFFFFFF) return WT_ERR_INVALID_ARG;
    if (key.split > 1 && (tiles > W.max_tiles || ((tiles << key.sh_s) << (key.sh_m + key.sh_n)) > W.ws_elems))
        return WT_ERR_INFEASIBLE;
    GemmArgs args;
    args.A = p.A; args.B = p.B; args.C = p.C; args.scaleA = p.sA; args.scaleB = p.sB;
    args.M = (int)p.M; args.N = (int)p.N; args.K = (int)p.K;
    args.tiles_m = (int)tiles_m; args.tiles_n = (int)tiles_n;
    args.swizzle = c.cfg.swizzle;
    args.splits = key.split;
    // each block of a split tile walks L = ceil(K / (S*bk)) k-tiles
    args.k_per_split = (int)(ceil_div64(p.K, (int64_t)key.bk * key.split) * key.bk);
    args.ws = W.ws;
    args.counters = W.counters;
    args.group_offsets = p.groups > 0 ? p.offsets : nullptr;
    args.groups = p.groups;
    args.vgrid = (int)G;
    args.queue = (ctx->persistent == 2 && !alt) ? ctx->queue : nullptr;
    // an output larger than half the 256 MB memory-side cache is written with the non-temporal hint
    const int64_t c_bytes = p.M * p.N * (ctx->out_type == WT_OUT_BF16 ? 2 : 4);
    args.stream_c = c_bytes > kStreamCBytes ? 1 : 0;
    // persistent launch: as many blocks as the device holds at once, each walking the task list with that stride
    const int64_t resident = (int64_t)kNumCU * std::max(1, c.occ_persistent);
    const int64_t grid = ctx->persistent ? std::min(G, resident) : G;
    if (key.split > 1 && (!W.ws || !W.counters)) return WT_ERR_NO_DEVICE;
    if (alt && key.split > 1) {
        // the static array keeps whatever the last call left: this launch's counters start at zero
        const int n = (int)tiles;
        hipLaunchKernelGGL(zero_ints, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, W.counters, n);
        WT_HIP(ctx, hipGetLastError());
    }
    void* params[] = {&args};
    WT_HIP(ctx, hipLaunchKernel(ctx->persistent ? c.fn_persistent : c.fn, dim3((unsigned)grid), dim3((unsigned)(c.cfg.nwave * 64)), params,
                                (size_t)(ctx->persistent ? c.lds_persistent : c.res.lds_bytes), stream));
    return WT_OK;
}

int check_gemm_args(const wt_ctx* ctx, const Problem& p, const wt_cfg& cfg, int* id) {
    if (!ctx || ctx->in_type == WT_ATTN_BF16) return WT_ERR_INVALID_ARG;
    if (ctx->device < 0) return WT_ERR_NO_DEVICE;
    const int rc = validate_shape(ctx, p.M, p.N, p.K);
    if (rc != WT_OK) return rc;
    if (p.groups < 0 || p.groups > kMaxGroups) return WT_ERR_INVALID_ARG;
    if (p.groups > 0 && p.M > 0 && !p.offsets) return WT_ERR_INVALID_ARG;
    if (p.M * p.N > 0 && (!p.C || (p.K > 0 && (!p.A || !p.B)))) return WT_ERR_INVALID_ARG;
    if (ctx->in_type == WT_FP8_E4M3 && p.M * p.N > 0 && (!p.sA || !p.sB)) return WT_ERR_INVALID_ARG;
    *id = find_config(ctx, cfg);
    if (*id < 0) return WT_ERR_UNSUPPORTED_CFG;
    if (ctx->cfgs[*id].res.occ < 1) return WT_ERR_INFEASIBLE;
    return WT_OK;
}

int time_config(wt_ctx* ctx, const Config& c, const Problem& p, int warmup, int iters, hipStream_t stream,
                double* mean_us) {
    hipEvent_t e0 = (hipEvent_t)ctx->ev_start, e1 = (hipEvent_t)ctx->ev_stop;
    for (int i = 0; i < warmup; ++i) {
        const int rc = launch(ctx, c, p, stream);
        if (rc != WT_OK) return rc;
    }
    // Timed batch: `iters` back-to-back launches between one event pair.  A batch shorter than
    // kMinTimedUs is too close to the event resolution and to launch jitter, so it is repeated with
    // proportionally more launches (at most 64x); the mean is over the launches of the last batch.
    float ms = 0;
    for (int pass = 0; pass < 2; ++pass) {
        WT_HIP(ctx, hipEventRecord(e0, stream));
        for (int i = 0; i < iters; ++i) {
            const int rc = launch(ctx, c, p, stream);
            if (rc != WT_OK) return rc;
        }
        WT_HIP(ctx, hipEventRecord(e1, stream));
        WT_HIP(ctx, hipEventSynchronize(e1));
        WT_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
        const double total_us = (double)ms * 1000.0;
        if (pass == 1 || total_us >= kMinTimedUs) break;
        const double per = total_us > 0.5 ? total_us / iters : 0.5;
        const int more = (int)(kMinTimedUs / per) + 1;
        iters = std::min(std::max(more, iters), iters * 64);
    }
    *mean_us = (double)ms * 1000.0 / (double)iters;
    return WT_OK;
}

struct Plan {
    size_t n_samples = 0;
    size_t bytesA = 0, bytesB = 0, bytesC = 0;
};

bool key_in_slice(const wt_grid* g, int k, int nk) {
    if (g->key_count <= 0) return k < nk;
    return k >= g->key_first && k < g->key_first + g->key_count;
}

int check_grid(const wt_grid* g) {
    if (!g || g->W < 1 || g->W > kMaxWaves || g->I < 1 || g->I > kMaxSubIntervals || g->W_row > kMaxWaves || g->tau_den < 1 || g->tau_num < g->tau_den || g->p < 1 || g->n_k_anchors < 1 ||
        !g->k_anchors || g->warmup < 0 || g->iters < 1 || g->W_row < 0 || g->W_split < 0 || g->row_fams < 0 ||
        (g->row_mode != WT_ROWS_TILES && g->row_mode != WT_ROWS_BAND) || g->row_fams > (g->row_mode == WT_ROWS_BAND ? 4 : 3))
        return WT_ERR_INVALID_ARG;
    for (int j = 0; j < g->n_k_anchors; ++j)
        if (g->k_anchors[j] < 1) return WT_ERR_INVALID_ARG;
    if (g->n_heads < 0) return WT_ERR_INVALID_ARG;
    return WT_OK;
}

// Attention contexts (Sec. 4.2, attention rules): head-aligned grid sizes, S_q = (g / N_h) * T_Q, KV lengths from
// the multipliers; fn gets (M, N, K) = (S_q, N_h, L * T_KV).
template <typename F>
int walk_plan_attn(const wt_ctx* ctx, const wt_grid* grid, F&& fn) {
    if (grid->n_heads < 1) return WT_ERR_INVALID_ARG;
    const int nk = (int)ctx->keys.size();
    std::vector<GridPoint> pts;
    std::vector<int64_t> anchors;
    for (int k = 0; k < nk; ++k) {
        if (!key_in_slice(grid, k, nk)) continue;
        const Key& key = ctx->keys[k];
        sample_grid_heads(key.cap, grid->W, grid->I, grid->n_heads, pts);
        for (size_t s = 0; s < pts.size(); ++s) {
            if (pts[s].g == 0) continue;
            const int64_t S_q = pts[s].m * key.bm;
            if (grid->max_out_elems > 0 && S_q * grid->n_heads * kHeadDim > grid->max_out_elems) continue;
            const int w = (int)(s / (size_t)grid->I) + 1;
            kv_loop_anchors(grid, S_q, key.bk, anchors);
            for (int64_t L : anchors) {
                if (L < 1 || L * key.bk > kMaxSeq || S_q > kMaxSeq) continue;
                const int rc = fn(k, pts[s], w, 0, L, S_q, (int64_t)grid->n_heads, L * key.bk);
                if (rc != WT_OK) return rc;
            }
        }
    }
    return WT_OK;
}

// Walk the sampling plan; fn(key, point, w, family, L, M, N, K) is called for every workload that will be
// timed: the paper's near-square grids (family 0), then, when grid->W_row > 0, the few-row grids m x n
// (m = 1, 2, 4 tile rows: families 1, 2, 3) with n the widest that keeps the task count in the sub-interval.
template <typename F>
int walk_plan(const wt_ctx* ctx, const wt_grid* grid, F&& fn) {
    if (ctx->in_type == WT_ATTN_BF16) return walk_plan_attn(ctx, grid, fn);
    const int nk = (int)ctx->keys.size();
    std::vector<GridPoint> pts;
    std::vector<int64_t> anchors;
    for (int k = 0; k < nk; ++k) {
        if (!key_in_slice(grid, k, nk)) continue;
        const Key& key = ctx->keys[k];
        // split-K keys: only the first W_split waves are worth profiling (0 = all W)
        const int W = (key.split > 1 && grid->W_split > 0) ? std::min(grid->W, grid->W_split) : grid->W;
        sample_grid(key.cap, W, grid->I, grid->tau_num, grid->tau_den, key.split, pts);
        loop_anchors(grid, key.bk * key.split, anchors);
        for (size_t s = 0; s < pts.size() && !grid->skip_near; ++s) {
            if (pts[s].g == 0) continue;
            const int64_t M = pts[s].m * key.bm, N = pts[s].n * key.bn;
            if (grid->max_out_elems > 0 && M * N > grid->max_out_elems) continue;
            if (!key_fits(key, pts[s].m * pts[s].n)) continue;
            const int w = (int)(s / (size_t)grid->I) + 1;
            for (int64_t L : anchors) {
                const int rc = fn(k, pts[s], w, 0, L, M, N, L * key.bk * key.split);
                if (rc != WT_OK) return rc;
            }
        }
        // few-row families: m rows of tiles, the widest n that keeps the task count S*m*n inside the sub-interval
        const int n_fams = grid->W_row > 0 ? (grid->row_fams > 0 ? grid->row_fams : 1) : 0;
        const int W_row = (key.split > 1 && grid->W_split > 0) ? std::min(grid->W_row, grid->W_split) : grid->W_row;
        for (int fam = 1; fam <= n_fams; ++fam) {
            // tile-row families: m = 1, 2, 4 full tile rows; row-band families: 16, 32, 64, 128 rows whatever the
            // key's tile height, so that every key of a band is profiled on the same matrices
            const int64_t band_rows = int64_t{kRowBand0} << (fam - 1);
            const int64_t m = grid->row_mode == WT_ROWS_BAND ? ceil_div64(band_rows, key.bm) : int64_t{1} << (fam - 1);
            for (int w = 1; w <= W_row; ++w) {
                for (int i = 1; i <= grid->I; ++i) {
                    const int64_t lo = (int64_t)(w - 1) * key.cap + 1;
                    const int64_t a = lo + ((int64_t)(i - 1) * key.cap) / grid->I;
                    const int64_t b = lo - 1 + ((int64_t)i * key.cap) / grid->I;
                    const int64_t n = b / (m * key.split);
                    const GridPoint pt{n * m * key.split, m, n};
                    if (n < 1 || pt.g < a) continue;
                    const int64_t M = grid->row_mode == WT_ROWS_BAND ? band_rows : m * key.bm, N = n * key.bn;
                    if (grid->max_out_elems > 0 && M * N > grid->max_out_elems) continue;
                    if (!key_fits(key, m * n)) continue;
                    for (int64_t L : anchors) {
                        const int rc = fn(k, pt, w, fam, L, M, N, L * key.bk * key.split);
                        if (rc != WT_OK) return rc;
                    }
                }
            }
        }
    }
    return WT_OK;
}

int sample_plan_impl(const wt_ctx* ctx, const wt_grid* grid, size_t* n_samples, size_t* bytesA, size_t* bytesB,
                            size_t* bytesC) {
    int rc = WT_OK;
    Plan p;
    const size_t esz = ctx->in_type == WT_BF16 ? 2 : 1, osz = ctx->out_type == WT_OUT_F32 ? 4 : 2;
    const bool attn = ctx->in_type == WT_ATTN_BF16;
    rc = walk_plan(ctx, grid, [&](int k, const GridPoint&, int, int, int64_t, int64_t M, int64_t N, int64_t K) {
        p.n_samples += (size_t)ctx->keys[k].n_micro;
        if (attn) {  // Q, K followed by V, O; bf16
            p.bytesA = std::max(p.bytesA, (size_t)(M * N * kHeadDim) * 2);
            p.bytesB = std::max(p.bytesB, (size_t)(K * N * kHeadDim) * 4);
            p.bytesC = std::max(p.bytesC, (size_t)(M * N * kHeadDim) * 2);
            return (int)WT_OK;
        }
        p.bytesA = std::max(p.bytesA, (size_t)(M * K) * esz);
        p.bytesB = std::max(p.bytesB, (size_t)(N * K) * esz);
        p.bytesC = std::max(p.bytesC, (size_t)(M * N) * osz);
        return (int)WT_OK;
    });
    if (rc != WT_OK) return rc;
    if (n_samples) *n_samples = p.n_samples;
    if (bytesA) *bytesA = p.bytesA;
    if (bytesB) *bytesB = p.bytesB;
    if (bytesC) *bytesC = p.bytesC;
    return WT_OK;
}

}  // namespace

static int profile_sparse_impl(wt_ctx* ctx, const wt_grid* grid, void* scrA, void* scrB, void* scrC, size_t bytesA,
                               size_t bytesB, size_t bytesC, void* hip_stream, wt_sample* out, size_t cap, size_t* n_out);

extern "C" {

int wt_create(wt_ctx** out, int device, int in_type, int out_type) {
    if (!out || (in_type != WT_BF16 && in_type != WT_FP8_E4M3 && in_type != WT_ATTN_BF16) ||
        (out_type != WT_OUT_F32 && out_type != WT_OUT_BF16) || (in_type == WT_ATTN_BF16 && out_type != WT_OUT_BF16))
        return WT_ERR_INVALID_ARG;
    *out = nullptr;
    wt_ctx* ctx = new (std::nothrow) wt_ctx();
    if (!ctx) return WT_ERR_INVALID_ARG;
    ctx->device = device;
    ctx->in_type = in_type;
    ctx->out_type = out_type;
    int rc = WT_ERR_NO_MEMORY;
    try {
        rc = build_registry(ctx);
    } catch (...) {
    }
    if (rc != WT_OK) { delete ctx; return rc; }
    if (device >= 0) {
        hipError_t e = hipSetDevice(device);
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (e == hipSuccess) e = hipEventCreate(&e0);
        if (e == hipSuccess) e = hipEventCreate(&e1);
        if (e != hipSuccess) { delete ctx; return WT_ERR_HIP; }
        ctx->ev_start = e0; ctx->ev_stop = e1;
        {   // this device's copy of the static scratch array (wt_gemm_noalloc); a failure is reported by that call
            hipError_t es = hipSuccess;
            ctx->static_scratch = static_scratch_for(device, &es);
            if (!ctx->static_scratch) ctx->last_hip = (int)es;
        }
        // split-K workspace: partial tiles, then the arrival counters (zero now; every launch leaves them zero)
        if (in_type != WT_ATTN_BF16) {  // attention kernels use no workspace
            void* ws = nullptr;
            // (two more ints behind the counters: the persistent kernels' task queue, zero between launches as well)
            const size_t ws_bytes = (size_t)kWsElems * sizeof(float), cnt_bytes = (size_t)(kMaxSplitTiles + 2) * sizeof(int);
            e = hipMalloc(&ws, ws_bytes + cnt_bytes);
            if (e == hipSuccess) e = hipMemset((char*)ws + ws_bytes, 0, cnt_bytes);
            if (e == hipSuccess) e = hipDeviceSynchronize();
            if (e != hipSuccess) {
                if (ws) (void)hipFree(ws);
                (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
                delete ctx;
                return WT_ERR_HIP;
            }
            ctx->ws = (float*)ws;
            ctx->counters = (int*)((char*)ws + ws_bytes);
            ctx->queue = ctx->counters + kMaxSplitTiles;
        }
        // per-key resources from the runtime: LDS opt-in, register count, resident blocks per CU
        for (size_t k = 0; k < ctx->keys.size(); ++k) {
            Key& key = ctx->keys[k];
            const Config& c0 = ctx->cfgs[key.first_cfg];
            int occ = 0;
            hipFuncAttributes fa;
            memset(&fa, 0, sizeof(fa));
            e = hipFuncSetAttribute(c0.fn, hipFuncAttributeMaxDynamicSharedMemorySize, key.lds_bytes);
            if (e == hipSuccess && c0.fn_persistent)
                e = hipFuncSetAttribute(c0.fn_persistent, hipFuncAttributeMaxDynamicSharedMemorySize, c0.lds_persistent);
            if (e == hipSuccess) e = hipFuncGetAttributes(&fa, c0.fn);
            if (e == hipSuccess)
                e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, c0.fn, key.nwave * 64, (size_t)key.lds_bytes);
            if (e != hipSuccess) { (void)hipGetLastError(); occ = 0; }
            key.vgprs = fa.numRegs;
            key.occ = occ;
            key.cap = key_capacity(ctx->cap_mode, occ);
            int occ_p = 0;
            if (!c0.fn_persistent) {
                occ_p = 1;
            } else if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ_p, c0.fn_persistent, key.nwave * 64,
                                                                    (size_t)c0.lds_persistent) != hipSuccess) {
                (void)hipGetLastError();
                occ_p = 1;
            }
            for (int m = 0; m < key.n_micro; ++m) {
                ctx->cfgs[key.first_cfg + m].res.occ = occ;
                ctx->cfgs[key.first_cfg + m].res.vgprs = fa.numRegs;
                ctx->cfgs[key.first_cfg + m].occ_persistent = std::max(1, occ_p);
            }
        }
    }
    *out = ctx;
    return WT_OK;
}

int wt_destroy(wt_ctx* ctx) {
    if (!ctx) return WT_ERR_INVALID_ARG;
    if (ctx->ev_start) (void)hipEventDestroy((hipEvent_t)ctx->ev_start);
    if (ctx->ev_stop) (void)hipEventDestroy((hipEvent_t)ctx->ev_stop);
    if (ctx->ws) (void)hipFree(ctx->ws);
    delete ctx;
    return WT_OK;
}

int wt_set_persistent(wt_ctx* ctx, int on) {
    if (!ctx || on < 0 || on > 2 || (on && ctx->in_type == WT_ATTN_BF16)) return WT_ERR_INVALID_ARG;
    if (on == 2 && !ctx->queue) return WT_ERR_NO_DEVICE;
    ctx->persistent = on;
    return WT_OK;
}

int wt_tile_coords(int tiles_m, int tiles_n, int swizzle, int block, int* tm, int* tn) {
    if (tiles_m < 1 || tiles_n < 1 || swizzle < 0 || swizzle >= kNumSwizzle || block < 0 ||
        (int64_t)block >= (int64_t)tiles_m * tiles_n || !tm || !tn)
        return WT_ERR_INVALID_ARG;
    tile_coords(block, tiles_m, tiles_n, swizzle, *tm, *tn);  // the kernel's own mapping, run on the host
    return WT_OK;
}

int wt_gemm(wt_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C, const float* scaleA,
            const float* scaleB, wt_cfg cfg, void* hip_stream) {
    int id = -1;
    const Problem p{M, N, K, A, B, C, scaleA, scaleB};
    const int rc = check_gemm_args(ctx, p, cfg, &id);
    if (rc != WT_OK) return rc;
    return launch(ctx, ctx->cfgs[id], p, (hipStream_t)hip_stream);
}

int wt_gemm_noalloc(wt_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
                    const float* scaleA, const float* scaleB, wt_cfg cfg, void* hip_stream) {
    int id = -1;
    const Problem p{M, N, K, A, B, C, scaleA, scaleB};
    const int rc = check_gemm_args(ctx, p, cfg, &id);
    if (rc != WT_OK) return rc;
    if (!ctx->static_scratch) return WT_ERR_HIP;   // hipGetSymbolAddress failed at wt_create (wt_last_hip_error)
    float* base = static_cast<float*>(ctx->static_scratch);
    const Workspace w{base, reinterpret_cast<int*>(base + kStaticWsFloats), (int64_t)kStaticWsFloats, (int64_t)kStaticTiles};
    return launch(ctx, ctx->cfgs[id], p, (hipStream_t)hip_stream, &w);
}

int wt_time_gemm(wt_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
                 const float* scaleA, const float* scaleB, wt_cfg cfg, int warmup, int iters, void* hip_stream,
                 double* mean_us) {
    int id = -1;
    if (!mean_us || warmup < 0 || iters < 1) return WT_ERR_INVALID_ARG;
    const Problem p{M, N, K, A, B, C, scaleA, scaleB};
    const int rc = check_gemm_args(ctx, p, cfg, &id);
    if (rc != WT_OK) return rc;
    return time_config(ctx, ctx->cfgs[id], p, warmup, iters, (hipStream_t)hip_stream, mean_us);
}

int wt_gemm_grouped(wt_ctx* ctx, int32_t groups, const int32_t* group_offsets, int64_t M_total, int64_t N, int64_t K,
                    const void* A, const void* B, void* C, const float* scaleA, const float* scaleB, wt_cfg cfg,
                    void* hip_stream) {
    int id = -1;
    if (groups < 1) return WT_ERR_INVALID_ARG;
    const Problem p{M_total, N, K, A, B, C, scaleA, scaleB, groups, group_offsets};
    const int rc = check_gemm_args(ctx, p, cfg, &id);
    if (rc != WT_OK) return rc;
    return launch(ctx, ctx->cfgs[id], p, (hipStream_t)hip_stream);
}

int wt_time_gemm_grouped(wt_ctx* ctx, int32_t groups, const int32_t* group_offsets, int64_t M_total, int64_t N,
                         int64_t K, const void* A, const void* B, void* C, const float* scaleA, const float* scaleB,
                         wt_cfg cfg, int warmup, int iters, void* hip_stream, double* mean_us) {
    int id = -1;
    if (!mean_us || warmup < 0 || iters < 1 || groups < 1) return WT_ERR_INVALID_ARG;
    const Problem p{M_total, N, K, A, B, C, scaleA, scaleB, groups, group_offsets};
    const int rc = check_gemm_args(ctx, p, cfg, &id);
    if (rc != WT_OK) return rc;
    return time_config(ctx, ctx->cfgs[id], p, warmup, iters, (hipStream_t)hip_stream, mean_us);
}

static int check_attn_args(const wt_ctx* ctx, int64_t H_q, int64_t H_kv, int64_t S_q, int64_t S_kv, const void* Q,
                           const void* K, const void* V, void* O, float scale, int causal, const wt_cfg& cfg, int* id) {
    if (!ctx || ctx->in_type != WT_ATTN_BF16) return WT_ERR_INVALID_ARG;
    if (ctx->device < 0) return WT_ERR_NO_DEVICE;
    if (H_q < 1 || H_kv < 1 || H_q % H_kv || H_q > 65536 || S_q < 0 || S_kv < 0 || S_q > kMaxSeq || S_kv > kMaxSeq ||
        (causal != 0 && causal != 1) || (causal && S_kv < S_q) || !(scale > 0.0f) || !(scale < 1e30f))
        return WT_ERR_INVALID_ARG;
    if (S_q > 0 && (!Q || !O || (S_kv > 0 && (!K || !V)))) return WT_ERR_INVALID_ARG;
    *id = find_config(ctx, cfg);
    if (*id < 0) return WT_ERR_UNSUPPORTED_CFG;
    if (ctx->cfgs[*id].res.occ < 1) return WT_ERR_INFEASIBLE;
    return WT_OK;
}

int wt_attn_batched(wt_ctx* ctx, int64_t batch, int64_t n_heads, int64_t n_kv_heads, int64_t S_q, int64_t S_kv,
                    const void* Q, const void* K, const void* V, void* O, float scale, int causal, wt_cfg cfg,
                    void* hip_stream) {
    int id = -1;
    if (batch < 0 || batch > 65536) return WT_ERR_INVALID_ARG;
    const int rc = check_attn_args(ctx, n_heads, n_kv_heads, S_q, S_kv, Q, K, V, O, scale, causal, cfg, &id);
    if (rc != WT_OK) return rc;
    if (batch == 0) return WT_OK;
    Problem p{S_q, n_heads, S_kv, Q, K, O, nullptr, nullptr};
    p.V = V; p.H_kv = n_kv_heads; p.scale = scale; p.causal = causal; p.batch = batch;
    return launch(ctx, ctx->cfgs[id], p, (hipStream_t)hip_stream);
}

int wt_attn_varlen(wt_ctx* ctx, int64_t batch, int64_t n_heads, int64_t n_kv_heads, int64_t total_q, int64_t total_kv,
                   const int32_t* cu_q, const int32_t* cu_kv, const void* Q, const void* K, const void* V, void* O,
                   float scale, int causal, wt_cfg cfg, void* hip_stream) {
    int id = -1;
    if (batch < 0 || batch > kMaxGroups || total_q > 0x7FFFFFFF || total_kv > 0x7FFFFFFF) return WT_ERR_INVALID_ARG;
    // (a causal sequence with fewer keys than queries is not an error here: the host does not see the lengths;
    //  its queries that see no key come out as zeros)
    const int rc = check_attn_args(ctx, n_heads, n_kv_heads, total_q, causal ? std::max(total_q, total_kv) : total_kv,
                                   Q, K, V, O, scale, causal, cfg, &id);
    if (rc != WT_OK) return rc;
    if (batch == 0 || total_q == 0) return WT_OK;
    if (!cu_q || !cu_kv) return WT_ERR_INVALID_ARG;
    Problem p{total_q, n_heads, total_kv, Q, K, O, nullptr, nullptr};
    p.V = V; p.H_kv = n_kv_heads; p.scale = scale; p.causal = causal; p.batch = batch; p.cu_q = cu_q; p.cu_kv = cu_kv;
    return launch(ctx, ctx->cfgs[id], p, (hipStream_t)hip_stream);
}

int wt_attn(wt_ctx* ctx, int64_t n_heads, int64_t n_kv_heads, int64_t S_q, int64_t S_kv, const void* Q,
            const void* K, const void* V, void* O, float scale, int causal, wt_cfg cfg, void* hip_stream) {
    return wt_attn_batched(ctx, 1, n_heads, n_kv_heads, S_q, S_kv, Q, K, V, O, scale, causal, cfg, hip_stream);
}

int wt_time_attn(wt_ctx* ctx, int64_t n_heads, int64_t n_kv_heads, int64_t S_q, int64_t S_kv, const void* Q,
                 const void* K, const void* V, void* O, float scale, int causal, wt_cfg cfg, int warmup, int iters,
                 void* hip_stream, double* mean_us) {
    int id = -1;
    if (!mean_us || warmup < 0 || iters < 1) return WT_ERR_INVALID_ARG;
    const int rc = check_attn_args(ctx, n_heads, n_kv_heads, S_q, S_kv, Q, K, V, O, scale, causal, cfg, &id);
    if (rc != WT_OK) return rc;
    Problem p{S_q, n_heads, S_kv, Q, K, O, nullptr, nullptr};
    p.V = V; p.H_kv = n_kv_heads; p.scale = scale; p.causal = causal;
    return time_config(ctx, ctx->cfgs[id], p, warmup, iters, (hipStream_t)hip_stream, mean_us);
}

int wt_attn_block_coords(int n_heads, int q_tiles, int order, int block, int* head, int* q_tile) {
    if (n_heads < 1 || q_tiles < 1 || order < 0 || order >= kAttnOrders || block < 0 ||
        (int64_t)block >= (int64_t)n_heads * q_tiles || !head || !q_tile)
        return WT_ERR_INVALID_ARG;
    attn_block_coords(block, n_heads, q_tiles, order, *head, *q_tile);
    return WT_OK;
}

int wt_sample_plan(const wt_ctx* ctx, const wt_grid* grid, size_t* n_samples, size_t* bytesA, size_t* bytesB,
                   size_t* bytesC) {
    if (!ctx) return WT_ERR_INVALID_ARG;
    int rc = check_grid(grid);
    if (rc != WT_OK) return rc;
    WT_GUARD(sample_plan_impl(ctx, grid, n_samples, bytesA, bytesB, bytesC));
}

int wt_profile_sparse(wt_ctx* ctx, const wt_grid* grid, void* scrA, void* scrB, void* scrC, size_t bytesA,
                      size_t bytesB, size_t bytesC, void* hip_stream, wt_sample* out, size_t cap, size_t* n_out) {
    if (!ctx || !out || !n_out || !scrA || !scrB || !scrC) return WT_ERR_INVALID_ARG;
    if (ctx->device < 0) return WT_ERR_NO_DEVICE;
    WT_GUARD(profile_sparse_impl(ctx, grid, scrA, scrB, scrC, bytesA, bytesB, bytesC, hip_stream, out, cap, n_out));
}

}  // extern "C"

static int profile_sparse_impl(wt_ctx* ctx, const wt_grid* grid, void* scrA, void* scrB, void* scrC, size_t bytesA,
                               size_t bytesB, size_t bytesC, void* hip_stream, wt_sample* out, size_t cap, size_t* n_out) {
    size_t need = 0, nA = 0, nB = 0, nC = 0;
    int rc = wt_sample_plan(ctx, grid, &need, &nA, &nB, &nC);
    if (rc != WT_OK) return rc;
    if (need > cap || nA > bytesA || nB > bytesB || nC > bytesC) return WT_ERR_BUFFER_TOO_SMALL;
    hipStream_t stream = (hipStream_t)hip_stream;
    // fp8 kernels read two fp32 scales; their values do not affect timing, so the head of scrB
    // (any bit pattern) stands in for both.
    const float* sA = (const float*)scrB;
    const float* sB = (const float*)scrB;
    size_t n = 0;
    rc = walk_plan(ctx, grid, [&](int k, const GridPoint& pt, int w, int family, int64_t L, int64_t M, int64_t N, int64_t K) {
        const Key& key = ctx->keys[k];
        for (int m = 0; m < key.n_micro; ++m) {
            const Config& c = ctx->cfgs[key.first_cfg + m];
            double us = 0;
            if (c.res.occ < 1) return (int)WT_ERR_INFEASIBLE;
            Problem p{M, N, K, scrA, scrB, scrC, sA, sB};
            if (ctx->in_type == WT_ATTN_BF16) {  // multi-head, full attention; V sits behind K in scrB
                p.V = (const char*)scrB + (size_t)(K * N * kHeadDim) * 2;
                p.H_kv = N;
                p.scale = 0.08838834764831845f;  // 1 / sqrt(128)
            }
            const int r = time_config(ctx, c, p, grid->warmup, grid->iters, stream, &us);
            if (r != WT_OK) return r;
            wt_sample s;
            memset(&s, 0, sizeof(s));
            s.key_id = k; s.micro_id = m; s.G = pt.g; s.L = L; s.w = w; s.family = family; s.mean_us = us;
            out[n++] = s;
        }
        return (int)WT_OK;
    });
    *n_out = n;
    return rc;
}
