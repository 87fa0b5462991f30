/* wt.h -- C ABI of libwt: a tile-parameterised MFMA GEMM for AMD MI355X (gfx950) and the
 * WaveTune selector that chooses its runtime configuration.
 *
 * Paper: "WaveTune: Wave-aware Bilinear Modeling for Efficient GPU Kernel Auto-tuning".
 * Section / equation references below are to that paper.
 *
 * Conventions
 *   - Every function returns WT_OK (0) or a negative wt_status.  Nothing throws across the ABI.
 *   - "device pointer" = address in the HBM of the context's GPU; "host pointer" = ordinary memory.
 *   - The caller owns every buffer and the HIP stream.  wt_gemm and wt_select never allocate.
 *   - Matrices: A is [M,K] row-major, B is stored K-contiguous as [N,K] row-major (the weight
 *     layout of a linear layer, so C = A * B^T in storage terms), C is [M,N] row-major.
 *     K must be a multiple of 8 (bf16) or 16 (fp8): rows are moved in 16-byte pieces.
 *   - A configuration c = (bm, bn, bk, nwave, stages, swizzle, split): block tile BM x BN x BK,
 *     wavefronts per block, LDS pipeline stages, block-rasterisation mode, and the number S of
 *     blocks that share one output tile along K (split-K; 1 = none).  All but swizzle form the
 *     structural ("macro") key: they fix G, L and how many blocks fit on a compute unit.  With
 *     split S the kernel launches G = S * tiles tasks of L = ceil(K / (S*bk)) loop iterations
 *     (Table 2's mapping applied to the kernel's own task list); partial tiles meet in a workspace
 *     owned by the context and the last block to arrive adds them in split order.
 *     swizzle is the micro parameter (Sec. 4.1: macro governs partitioning, wave dynamics
 *     and dominant occupancy; micro tunes execution efficiency, e.g. rasterisation for L2 reuse).
 *     swizzle 0: tiles in row-major order (XCD x of the 8 walks tile columns x, x+8, ...);
 *     swizzle 1 / 2: each XCD gets a contiguous range of a grouped order (groups of 4 / 8 tile rows
 *     walked column by column), so that tiles sharing a B panel run on the same XCD's L2.  A grid of
 *     at most 8 tile rows is walked as one such group under every mode (row-major never pays there).
 */
#ifndef WT_H
#define WT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WT_OK = 0,
    WT_ERR_INVALID_ARG = -1,     /* null pointer, negative size, K not a multiple of the vector width */
    WT_ERR_UNSUPPORTED_CFG = -2, /* (bm,bn,bk,nwave,stages,swizzle,split) is not in the registry */
    WT_ERR_INFEASIBLE = -3,      /* config exists but does not fit the device (LDS / registers), or a split-K
                                  * config's partial tiles for this shape exceed the context's workspace */
    WT_ERR_NOT_FITTED = -4,      /* wt_select / wt_predict_us before wt_fit or wt_load */
    WT_ERR_HIP = -5,             /* a HIP call failed; see wt_last_hip_error() */
    WT_ERR_BUFFER_TOO_SMALL = -6,
    WT_ERR_IO = -7,
    WT_ERR_NO_DEVICE = -8,       /* device work requested from a host-only context */
    WT_ERR_NO_MEMORY = -9        /* a host allocation failed */
} wt_status;

/* Storage type of A and B.  WT_ATTN_BF16 makes an attention context instead of a GEMM one: its registry holds
 * the FlashAttention-style kernels (see wt_attn), out_type must be WT_OUT_BF16, and the shape triple of
 * wt_select / wt_wave_count / wt_predict_us reads (M, N, K) = (S_q, N_h, S_kv). */
typedef enum { WT_BF16 = 0, WT_FP8_E4M3 = 1, WT_ATTN_BF16 = 2 } wt_in_t;
typedef enum { WT_OUT_F32 = 0, WT_OUT_BF16 = 1 } wt_out_t; /* storage type of C */

typedef struct wt_ctx wt_ctx; /* opaque: config registry, per-config resources, dual table */

/* Feasibility limits of this library (properties of the build, not of the method):
 *   a context's split-K workspace holds WT_SPLITK_WS_FLOATS fp32 partial-tile elements and one arrival counter
 *   for each of at most WT_SPLITK_MAX_TILES output tiles per launch; a split-K configuration whose partial tiles
 *   for a shape exceed either is not a candidate of wt_select and wt_gemm returns WT_ERR_INFEASIBLE for it;
 *   a dual-table bucket stores at most WT_MAX_ANCHORS <loop count, micro> anchors (Sec. 4.3 anchor table) --
 *   with more distinct loop counts in a bucket, those at ranks floor(i*(n-1)/(WT_MAX_ANCHORS-1)) are kept. */
#define WT_SPLITK_WS_FLOATS (1 << 26)
#define WT_SPLITK_MAX_TILES (1 << 16)
#define WT_MAX_ANCHORS 8

/* One kernel configuration.  id is the registry index (or -1: look the fields up). */
typedef struct {
    int32_t bm, bn, bk, nwave, stages, swizzle;
    int32_t split; /* S >= 1 */
    int32_t id;
} wt_cfg;

/* Resources of a configuration.  occ = blocks resident per compute unit: the HIP runtime's answer
 * on a device context, a static LDS/wave-slot estimate on a host-only context.  key_id groups
 * configs that differ only in swizzle; micro_id is the position inside the group. */
typedef struct {
    int32_t lds_bytes, vgprs, nwave, occ;
    int32_t key_id, micro_id;
} wt_cfg_res;

/* One profiling record <G, L, w, c_macro, c_micro, mean latency> (Sec. 4.2, profiling output). */
typedef struct {
    int32_t key_id, micro_id;
    int64_t G, L;
    int32_t w;
    int32_t family; /* 0: near-square grid (the paper's sampler); 1..: a few-row family of wt_grid.W_row -- grids of 1, 2,
                     * 4 tile rows (WT_ROWS_TILES) or matrices of 16, 32, 64, 128 rows (WT_ROWS_BAND) */
    double mean_us;
} wt_sample;

/* Sampling / fitting parameters (Sec. 4.2, 4.5; Sec. 5.1 uses W=40, I=4, tau=11/10, p=10, five K
 * anchors in [1024,5120], 3 warm-up + 5 measured runs).  key_first/key_count restrict
 * wt_profile_sparse to a slice of structural keys (0,0 = all) so that profiling can be split
 * over several calls.  max_out_elems caps M*N of an instantiated workload (0 = no cap): grid
 * points whose output would exceed it are skipped. */
typedef struct {
    int32_t W, I, tau_num, tau_den, p; /* 1 <= W <= 4096, 1 <= I <= 4096, tau_num >= tau_den >= 1, p >= 1 */
    int32_t n_k_anchors;
    const int32_t* k_anchors; /* host pointer, n_k_anchors entries */
    int32_t warmup, iters;
    int32_t key_first, key_count;
    int64_t max_out_elems;
    int32_t model;    /* wt_model: which latency model wt_fit builds (0 = the paper's) */
    int32_t W_split;  /* split-K keys are profiled for waves 1..min(W, W_split) only (0 = all W); beyond their
                       * profiled waves they have no model and wt_select does not consider them */
    int32_t W_row;    /* extension, 0 = off (the paper's method): also profile and fit W_row waves of few-row
                       * grids -- families 1..row_fams, each, per sub-interval, with the widest n_G that keeps the
                       * task count inside it -- kept in their own bucket sets, which wt_select consults for shapes
                       * of few rows, falling back to the paper's buckets.  What a family holds and which shapes
                       * consult it is row_mode's (wt_row_mode, below).  The paper's sampler stays near-square (tau)
                       * and its test shapes have M >= 64; these grids cover the serving shapes (few rows, very
                       * wide) whose B operand streams from HBM with little reuse, which near-square samples of the
                       * same G do not show. */
    int32_t row_fams; /* number of few-row families: 1..3 under WT_ROWS_TILES, 1..4 under WT_ROWS_BAND (0 is read as
                       * 1); used only when W_row > 0 */
    int32_t skip_near; /* 1: wt_sample_plan / wt_profile_sparse leave out the near-square family (to add few-row
                        * records to an existing set); wt_fit ignores it */
    int32_t n_heads;   /* attention contexts only (must be >= 1 there): head count N_h of the profiled workloads.
                        * Grid sizes are head-aligned, g = floor(b / N_h) * N_h >= a (Sec. 4.2), a grid point is
                        * S_q = (g / N_h) * T_Q (Eq. 6), and k_anchors holds KV-length multipliers in percent of
                        * S_q (Sec. 5.1: 1.0 to 3.0): L = ceil(floor(S_q * pct / 100) / T_KV), S_kv = L * T_KV.
                        * tau, W_row, W_split are unused; max_out_elems caps S_q * N_h * 128. */
    int32_t weighting; /* wt_weighting: what the least squares of wt_fit's bilinear buckets minimise (below) */
    int32_t row_mode;  /* which grids the few-row families hold when W_row > 0 (wt_row_mode, below) */
} wt_grid;

/* Objective of the per-bucket least squares (Sec. 4.3 bucket model; Sec. 5.1 "least-squares regression").
 *   WT_FIT_ABSOLUTE  sum of (That - T)^2, ordinary least squares: the paper as written, and the default;
 *   WT_FIT_RELATIVE  sum of ((That - T) / T)^2: every record weighs 1 / T^2.  A deviation made for loop-anchor sets
 *                    wider than the paper's [1024, 5120]: with anchors from K = 256 to 28672 a bucket's latencies span
 *                    two orders of magnitude and ordinary least squares spends its accuracy on the long-K records,
 *                    leaving short-K predictions off by their own size (even negative).  Every record must then have
 *                    mean_us > 0 (WT_ERR_INVALID_ARG otherwise).  The Step ablation is always fitted absolutely. */
typedef enum { WT_FIT_ABSOLUTE = 0, WT_FIT_RELATIVE = 1 } wt_weighting;

/* What the few-row families of wt_grid.W_row hold (extension; the paper's sampler has no such grids).
 *   WT_ROWS_TILES  families 1..3 are grids of 1, 2, 4 full tile rows of the key at hand (M = m_G * bm), and a shape
 *                  consults, per key, the family of its own tile-row count ceil(M/bm): family 1 for one, 2 for two
 *                  or three, 3 for four to seven tile rows.  Keys of different tile heights are then priced from
 *                  different matrices.
 *   WT_ROWS_BAND   families 1..4 are grids of exactly 16, 32, 64, 128 rows under EVERY key (ceil(rows/bm) tile rows,
 *                  the last one partial), and a shape with M <= 128 consults the family of the smallest band that
 *                  holds M under every key alike, so that Stage I compares predictions made from the same matrices. */
typedef enum { WT_ROWS_TILES = 0, WT_ROWS_BAND = 1 } wt_row_mode;

/* Latency models wt_fit can build into the dual table.  WAVE_BILINEAR is the method (Sec. 4.3);
 * the other two are its ablations (Sec. 5.4) expressed in the same table form:
 *   LINEAR  no wave buckets: one bilinear tuple per key fitted over all profiled waves;
 *   STEP    T = w*(a*L + b), w = ceil(G/capacity): latency as a function of the wave count only
 *           (the classical T_wave*ceil(G/N) model of Sec. 3.2), continued linearly beyond W. */
typedef enum { WT_MODEL_WAVE_BILINEAR = 0, WT_MODEL_LINEAR = 1, WT_MODEL_STEP = 2 } wt_model;

/* ---- context ------------------------------------------------------------------------------ */
/* device >= 0: bind to that GPU, query kernel resources.  device = -1: host-only context (Phi,
 * sampler, fit, select, save/load work; wt_gemm and wt_profile_sparse return WT_ERR_NO_DEVICE). */
int wt_create(wt_ctx** out, int device, int in_type, int out_type);
int wt_destroy(wt_ctx* ctx);
int wt_last_hip_error(const wt_ctx* ctx);          /* hipError_t of the last failing HIP call */
const char* wt_status_string(int status);

/* ---- config registry ---------------------------------------------------------------------- */
int wt_config_count(const wt_ctx* ctx, int* n);
int wt_config_get(const wt_ctx* ctx, int i, wt_cfg* cfg, wt_cfg_res* res);
int wt_config_find(const wt_ctx* ctx, const wt_cfg* fields, int* id); /* match the seven fields */
int wt_key_count(const wt_ctx* ctx, int* n);
/* Override the recorded occupancy of structural key key_id (e.g. with a measured value). */
int wt_key_set_occ(wt_ctx* ctx, int key_id, int occ);
/* Wave capacity used by the wave count, the sampler and the table buckets:
 *   WT_CAP_CU_ONLY (default)  capacity = 256 compute units: the paper's w = ceil(G / N_SM) (Sec. 3.2, 3.3);
 *   WT_CAP_CU_TIMES_OCC       capacity = 256 x resident blocks per CU of the key (a "wave" = everything
 *                             that can be resident at once).
 * Changing the mode discards a fitted table; wt_load sets the mode the table was built with. */
typedef enum { WT_CAP_CU_TIMES_OCC = 0, WT_CAP_CU_ONLY = 1 } wt_cap_mode;
int wt_set_capacity_mode(wt_ctx* ctx, int mode);

/* ---- the GEMM (Sec. 3.2, tiled-GEMM paragraph) ------------------------------------------- */
/* C[M,N] = A[M,K] * B[N,K]^T under configuration cfg.  A, B, C: device pointers (types per
 * the context).  scaleA/scaleB: device pointers to one fp32 each, fp8 only (C = sA*sB*sum),
 * NULL for bf16.  Asynchronous on hip_stream (a hipStream_t, NULL = default stream); never
 * synchronises, never allocates.  M, N may be any non-negative size (edge tiles are masked);
 * M*N == 0 is a no-op; K == 0 writes zeros.
 * Split-K configurations (cfg.split > 1) stage partial tiles in the context's workspace (256 MiB,
 * allocated by wt_create): WT_ERR_INFEASIBLE when ceil(M/bm)*ceil(N/bn)*split*bm*bn exceeds 2^26
 * floats or there are more than 65536 tiles.  Launches that use the workspace must be ordered on
 * one stream per context: two of them running concurrently race on it. */
int wt_gemm(wt_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
            const float* scaleA, const float* scaleB, wt_cfg cfg, void* hip_stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc: wt_gemm with the split-K partial tiles and arrival counters kept in a static device array
 * of the library (WT_NOALLOC_WS_FLOATS fp32 elements + WT_NOALLOC_MAX_TILES counters, 64 MiB + 128 KiB, held by
 * every GPU the library runs on until the process ends) instead of the context's workspace.  Same arguments, same
 * results bit for bit as wt_gemm.  The call itself allocates nothing on host or device and does not synchronise;
 * the array's address on the context's GPU is looked up once, by wt_create (WT_ERR_HIP here if that failed).
 * WT_ERR_INFEASIBLE when a split-K configuration's partial tiles exceed the array: ceil(M/bm)*ceil(N/bn)*split*bm*bn
 * > WT_NOALLOC_WS_FLOATS or more than WT_NOALLOC_MAX_TILES output tiles.  Unsplit configurations use no scratch and
 * have no such limit.  All calls on one GPU -- from any context, on any stream -- share that GPU's array: a
 * split-K launch first zeroes its tiles' counters (a small kernel on hip_stream), and two split-K launches that
 * overlap in time on one GPU race on the array; order them on one stream. */
#define WT_NOALLOC_WS_FLOATS (1 << 24)
#define WT_NOALLOC_MAX_TILES (1 << 15)
int wt_gemm_noalloc(wt_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
                    const float* scaleA, const float* scaleB, wt_cfg cfg, void* hip_stream);

/* Launch policy (Sec. 3.2, note on persistent kernels: the launched grid is clamped to what the device holds
 * at once while G remains the logical task count).  on = 1: every later launch of this context starts
 * min(G, 256 x resident blocks per CU) blocks and block b runs tasks b, b + grid, b + 2*grid, ... of the same
 * task list (same rasterisation, same split-K protocol, same results); on = 2: the same grid, but a block draws its
 * further tasks from a device-side queue as it gets to them (the queue lives beside the context's split-K counters:
 * launches of one context that overlap in time race on it, as they do on the split-K workspace); on = 0 (default):
 * one block per task.  Where a kernel's LDS has room, a persistent block requests its next task's first k-tiles
 * before it writes the current tile out.  Phi, wave counts, tables and selection are unaffected.  wt_gemm_noalloc
 * launches treat 2 as 1 (the queue is context memory).  Errors: WT_ERR_INVALID_ARG (on outside 0..2, attention
 * context), WT_ERR_NO_DEVICE (on = 2 on a host-only context). */
int wt_set_persistent(wt_ctx* ctx, int on);

/* ---- grouped GEMM (Table 2, grouped-GEMM row: G = sum_e ceil(M_e/bm) * ceil(N/bn), L = ceil(K/bk)) ---- */
/* For every group e in [0, groups): C[r0:r1, :] = A[r0:r1, :] * B[e]^T with r0 = offsets[e], r1 = offsets[e+1].
 * A: [M_total, K] rows of all groups back to back; B: [groups, N, K]; C: [M_total, N]; all device pointers.
 * group_offsets: DEVICE pointer to groups+1 ascending int32 row offsets (offsets[0] = 0, offsets[groups] =
 * M_total), read by the kernel -- the host never needs the routing result, so no synchronisation is needed
 * between the router and this call.  Entries are clipped to [0, M_total] on the device, so wrong contents give
 * wrong results but never an access outside A, B or C.  The grid is sized for the worst case
 * (ceil(M_total/bm) + groups row tiles); surplus blocks exit at once.  groups <= 1024; cfg.split must be 1
 * (WT_ERR_UNSUPPORTED_CFG otherwise).  Asynchronous, never allocates. */
int wt_gemm_grouped(wt_ctx* ctx, int32_t groups, const int32_t* group_offsets, int64_t M_total, int64_t N,
                    int64_t K, const void* A, const void* B, void* C, const float* scaleA, const float* scaleB,
                    wt_cfg cfg, void* hip_stream);
/* wt_time_gemm's protocol for a grouped launch. */
int wt_time_gemm_grouped(wt_ctx* ctx, int32_t groups, const int32_t* group_offsets, int64_t M_total, int64_t N,
                         int64_t K, const void* A, const void* B, void* C, const float* scaleA,
                         const float* scaleB, wt_cfg cfg, int warmup, int iters, void* hip_stream,
                         double* mean_us);
/* Exact Phi of a grouped launch whose per-group row counts are known (host pointer, groups entries). */
int wt_wave_count_grouped(const wt_ctx* ctx, int32_t groups, const int64_t* group_rows, int64_t N, int64_t K,
                          wt_cfg cfg, int64_t* G, int64_t* L, int32_t* w);
/* Runtime selection for a grouped launch from the dense dual table (Sec. 4.2: grouped GEMM is sampled as the
 * single-group case) under the uniform approximation of Sec. 5.2: per-group counts are unknown on the host, so
 * each group is taken to hold ceil(M_total/groups) rows.  Split-K keys are not candidates.  Host only. */
int wt_select_grouped(const wt_ctx* ctx, int32_t groups, int64_t M_total, int64_t N, int64_t K, wt_cfg* out);
/* The same when the host does know the per-group row counts (a router that has synchronised, a fixed split):
 * group_rows is a HOST pointer to `groups` counts >= 0, and G is Table 2's grouped row on them, sum_e ceil(M_e/bm) *
 * ceil(N/bn), instead of the uniform approximation; an empty group adds no tile.  The few-row family, where the table
 * has them, is that of the mean group, ceil(sum/groups) rows, so equal groups give wt_select_grouped's answer.
 * 1 <= groups <= 1024 and the counts' sum must fit an int32 (WT_ERR_INVALID_ARG otherwise, and for an attention
 * context).  WT_ERR_NOT_FITTED without a table.  Host only. */
int wt_select_grouped_rows(const wt_ctx* ctx, int32_t groups, const int64_t* group_rows, int64_t N, int64_t K,
                           wt_cfg* out);

/* ---- attention (Table 2, FlashAttention row: G = N_h * ceil(S_q/T_Q), L = ceil(S_kv/T_KV)) ---------------- */
/* O = softmax(scale * Q K^T [+ causal mask]) V per head, one sequence, bf16 in and out, head dimension 128, on a
 * WT_ATTN_BF16 context.  Device pointers: Q and O are [S_q, n_heads, 128], K and V are [S_kv, n_kv_heads, 128]
 * (token-major, head dimension contiguous).  n_kv_heads divides n_heads: query head h reads KV head
 * h / (n_heads / n_kv_heads) (grouped-query attention; equal counts = multi-head attention).  causal = 1: query i
 * sees keys j <= i + (S_kv - S_q), which needs S_kv >= S_q.  scale must be positive and finite (the kernel
 * tracks the running maximum in unscaled units).  S_kv = 0 writes zeros; S_q = 0 is a no-op.
 * A configuration is <bm, bn, bk, nwave, stages, swizzle, split> = <T_Q, 1, T_KV, wavefronts, 1, order, 1>: a block
 * owns T_Q query rows of one head and loops over the KV tiles; `order` is the micro parameter (0: the query tiles
 * of a head are consecutive blocks; 1: the heads of a query tile are consecutive blocks; 2: as 0, with every one
 * of the 8 XCDs given a contiguous range so that a head's K/V stay in one L2).  Causal launches ignore `order`:
 * their blocks differ in length, so they are always started longest first with the heads of a query tile
 * consecutive (order 1 on the reversed query-tile index).  Scores and softmax are fp32, the
 * probabilities are rounded to bf16 before they multiply V.  Asynchronous on hip_stream, never allocates or
 * synchronises.  The persistent launch policy does not apply. */
int wt_attn(wt_ctx* ctx, int64_t n_heads, int64_t n_kv_heads, int64_t S_q, int64_t S_kv, const void* Q,
            const void* K, const void* V, void* O, float scale, int causal, wt_cfg cfg, void* hip_stream);
/* The same for `batch` sequences of equal lengths in one launch: Q and O are [batch, S_q, n_heads, 128], K and V
 * [batch, S_kv, n_kv_heads, 128].  The grid holds batch * n_heads * ceil(S_q/T_Q) blocks, mapped by `order` as if the
 * launch had batch * n_heads heads -- Table 2's attention row with the batch folded into N_h -- so the configuration
 * for such a launch is wt_select(ctx, S_q, batch * n_heads, S_kv).  0 <= batch <= 65536 (0 is a no-op); every other
 * argument as for wt_attn, which is this call with batch = 1.  Results per sequence are bit-identical to wt_attn's. */
int wt_attn_batched(wt_ctx* ctx, int64_t batch, int64_t n_heads, int64_t n_kv_heads, int64_t S_q, int64_t S_kv,
                    const void* Q, const void* K, const void* V, void* O, float scale, int causal, wt_cfg cfg,
                    void* hip_stream);
/* A batch of sequences of DIFFERENT lengths in one launch, their tokens packed back to back: Q and O are
 * [total_q, n_heads, 128], K and V [total_kv, n_kv_heads, 128]; cu_q and cu_kv are DEVICE pointers to batch + 1
 * ascending int32 token offsets (sequence b owns query tokens [cu_q[b], cu_q[b+1]) and key tokens [cu_kv[b],
 * cu_kv[b+1])).  As with the grouped GEMM the host never reads them (a serving engine builds them on the device): the
 * grid is sized for the worst case, n_heads * (ceil(total_q/T_Q) + batch) blocks, a block finds its sequence from the
 * offsets, and blocks past the last query tile exit at once.  Offsets are clipped to [0, total] in the kernel, so no
 * content of the arrays can make an access leave the tensors.  causal = 1 aligns every sequence's queries to the end
 * of its own keys; a query that sees no key (a sequence with fewer keys than queries) yields zeros; causal launches walk
 * the batch's query tiles from the last to the first, longest blocks first.  0 <= batch <= 1024.
 * Selection: wt_select_attn_varlen when the host knows the lengths; from the totals alone, under the uniform
 * approximation of Sec. 5.2, wt_select(ctx, ceil(total_q/batch), batch * n_heads, ceil(total_kv/batch)).  Results per sequence are bit-identical
 * to wt_attn's.  Asynchronous, never allocates or synchronises. */
int wt_attn_varlen(wt_ctx* ctx, int64_t batch, int64_t n_heads, int64_t n_kv_heads, int64_t total_q, int64_t total_kv,
                   const int32_t* cu_q, const int32_t* cu_kv, const void* Q, const void* K, const void* V, void* O,
                   float scale, int causal, wt_cfg cfg, void* hip_stream);
/* Runtime selection for a wt_attn_varlen launch when the host knows the sequence lengths (HOST pointers len_q and
 * len_kv, `batch` entries >= 0 each; a serving engine that schedules the batch has them).  Table 2's attention row is
 * read per sequence: sequence b contributes ceil(len_q[b]/T_Q) blocks per head, each looping ceil(len_kv[b]/T_KV)
 * times; G = n_heads * the number of query tiles, and L is the mean loop count over the blocks, rounded half up, so
 * that G*L is the launch's number of key-tile iterations to within rounding -- exactly the row of Table 2 with the
 * batch folded into N_h when the lengths are equal.  The mean length that wt_select on the totals prices understates
 * a ragged batch's work, which its longest sequences carry.  1 <= batch <= 1024, 1 <= n_heads <= 65536, each sum of
 * lengths must fit an int32 and n_heads * sum(len_q) * sum(len_kv) must stay below 2^62 (WT_ERR_INVALID_ARG
 * otherwise, and for a context that is not an attention context).  WT_ERR_NOT_FITTED without a table.  Host only. */
int wt_select_attn_varlen(const wt_ctx* ctx, int32_t batch, const int64_t* len_q, const int64_t* len_kv,
                          int64_t n_heads, wt_cfg* out);
/* wt_time_gemm's protocol for an attention launch. */
int wt_time_attn(wt_ctx* ctx, int64_t n_heads, int64_t n_kv_heads, int64_t S_q, int64_t S_kv, const void* Q,
                 const void* K, const void* V, void* O, float scale, int causal, wt_cfg cfg, int warmup, int iters,
                 void* hip_stream, double* mean_us);
/* Diagnostic: (head, query tile) of workgroup `block` under `order` -- the kernel's own mapping on the host. */
int wt_attn_block_coords(int n_heads, int q_tiles, int order, int block, int* head, int* q_tile);
/* Head-aligned grid samples (Sec. 4.2): up to cap_out pairs (g, q tiles per head) in w-major, i-minor order;
 * g = 0 where the sub-interval holds no multiple of n_heads.  Host only. */
int wt_sample_grid_heads(int64_t capacity, int32_t W, int32_t I, int32_t n_heads, int64_t* g, int64_t* q_tiles,
                         size_t cap_out, size_t* n_out);

/* Diagnostic: the (tile row, tile column) that workgroup `block` of a tiles_m x tiles_n grid computes
 * under rasterisation mode `swizzle` -- the kernel's own mapping evaluated on the host.  Host only. */
int wt_tile_coords(int tiles_m, int tiles_n, int swizzle, int block, int* tm, int* tn);

/* ---- geometry (Table 2 Dense-GEMM row; Sec. 3.2 / 3.3 wave count) ------------------------ */
/* G = split*ceil(M/bm)*ceil(N/bn), L = ceil(K/(split*bk)), w = ceil(G / capacity) (see wt_set_capacity_mode). */
int wt_wave_count(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, wt_cfg cfg,
                  int64_t* G, int64_t* L, int32_t* w);

/* ---- sparse structural sampling (Sec. 4.2) ------------------------------------------------ */
/* Grid samples for a capacity: fills up to cap_out triples (g, m, n) in w-major, i-minor order
 * (g = 0 where a sub-interval holds no value with a near-square factorisation).  split = S >= 1:
 * task counts are multiples of S, g = S*m*n with m x n the near-square tile grid (S = 1: Eq. 3-4). */
int wt_sample_grid(int64_t capacity, int32_t W, int32_t I, int32_t tau_num, int32_t tau_den, int32_t split,
                   int64_t* g, int64_t* m, int64_t* n, size_t cap_out, size_t* n_out);
/* Number of records wt_profile_sparse would produce and the scratch bytes it needs. */
int wt_sample_plan(const wt_ctx* ctx, const wt_grid* grid, size_t* n_samples, size_t* bytesA,
                   size_t* bytesB, size_t* bytesC);
/* Instantiate every sample (M = m*bm, N = n*bn, K = L*split*bk), run every micro with warm-up +
 * measured launches timed by HIP events on hip_stream, write one record per <key, micro, g, L>.
 * scrA/scrB/scrC: device scratch of at least the planned sizes (contents: any finite values).
 * Attention contexts: scrA holds Q, scrB holds K followed by V, scrC holds O; workloads are multi-head
 * (n_kv_heads = n_heads, Sec. 4.2), not causal, scale 1/sqrt(128).
 * Synchronises the stream. */
int wt_profile_sparse(wt_ctx* ctx, const wt_grid* grid, void* scrA, void* scrB, void* scrC,
                      size_t bytesA, size_t bytesB, size_t bytesC, void* hip_stream,
                      wt_sample* out, size_t cap, size_t* n_out);
/* Time one (shape, config): warm-up + iters launches between one HIP event pair, mean microseconds.
 * If the timed batch lasts under 300 us it is repeated with proportionally more launches (at most
 * 64x) so that kernels of a few microseconds are not timed at the resolution of the events.  Same
 * protocol as wt_profile_sparse; used for exhaustive search. */
int wt_time_gemm(wt_ctx* ctx, int64_t M, int64_t N, int64_t K, const void* A, const void* B, void* C,
                 const float* scaleA, const float* scaleB, wt_cfg cfg, int warmup, int iters,
                 void* hip_stream, double* mean_us);

/* Diagnostic: sustained MFMA-only throughput of the device (register operands of magnitude ~1,
 * no memory traffic; 2 blocks of 4 wavefronts per compute unit, iters x 16 MFMAs each).  This is
 * the power- and clock-limited ceiling of a dense contraction, reported beside the nominal peak.
 * For bf16 the loop is run with 32x32x16 and with 16x16x32 MFMAs (same flop count) and the higher rate is returned.
 * sink_dev: device pointer to one float (never written in practice).  Synchronises the stream. */
int wt_mfma_ceiling(wt_ctx* ctx, int in_type, int iters, void* hip_stream, float* sink_dev,
                    double* tflops);

/* ---- modelling (Sec. 4.3, 4.5) ------------------------------------------------------------ */
/* Build the dual table from records (from the GPU or from any synthetic source).  Host only. */
int wt_fit(wt_ctx* ctx, const wt_grid* grid, const wt_sample* samples, size_t n);

/* ---- runtime selection (Sec. 4.4, 4.5) ---------------------------------------------------- */
/* Stage I: argmin over structural keys of the bucket's bilinear prediction (extrapolation tuple
 * when w > W or the bucket is empty); Stage II: nearest loop anchor -> micro.  Host only,
 * read-only, thread-safe, no allocation, no system calls.  WT_ERR_NOT_FITTED without a table.  This call and every
 * other that evaluates Phi or a prediction (wt_wave_count, wt_predict_us, the grouped and variable-length forms)
 * returns WT_ERR_INVALID_ARG for a negative dimension and for a shape so large that G*L could leave int64:
 * M * N * max(K, 16) above 2^62 (grouped: M = rows + groups), far beyond what a launch accepts. */
int wt_select(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, wt_cfg* out);
/* Predicted latency of one configuration's structural key for a shape (microseconds). */
int wt_predict_us(const wt_ctx* ctx, int64_t M, int64_t N, int64_t K, wt_cfg cfg, double* us);
/* Time n calls of wt_select over a shape list inside the library (steady clock): mean and p99
 * nanoseconds per call.  shapes: host pointer to n triples (M,N,K). */
int wt_select_bench(const wt_ctx* ctx, const int64_t* shapes, size_t n, int repeats,
                    double* mean_ns, double* p99_ns);

/* ---- dual-table artifact ------------------------------------------------------------------- */
/* The dual table of Sec. 4.3 / 4.5 (per key and wave: four coefficients, status, loop anchors with their micro; the
 * extrapolation tuple; the few-row families where fitted) as one little-endian file.  wt_save: WT_ERR_NOT_FITTED
 * without a table, WT_ERR_IO if the file cannot be written.  wt_load replaces the context's table, capacity mode and
 * per-key occupancy with the file's, or leaves the context as it was and returns WT_ERR_IO (unreadable, not a table
 * file, unknown version, shorter or longer than its header says) or WT_ERR_INVALID_ARG (written for another registry,
 * storage type or compute-unit count, or a header field out of range). */
int wt_save(const wt_ctx* ctx, const char* path);
int wt_load(wt_ctx* ctx, const char* path);

#ifdef __cplusplus
}
#endif
#endif /* WT_H */
