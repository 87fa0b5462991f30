// Tile-parameterised MFMA GEMM for gfx950 (MI355X): C[M,N] = A[M,K] * B[N,K]^T.
//
// One workgroup computes a BM x BN tile of C and walks K in L = ceil(K/BK) steps, each step
// staging a BM x BK piece of A and a BN x BK piece of B (Sec. 3.2, tiled-GEMM paragraph:
// G = ceil(M/BM)*ceil(N/BN) blocks, L loop iterations per block).
//
// gfx950 mapping
//   * global -> LDS: buffer_load_dwordx4 ... lds (16 bytes per lane straight into LDS, no VGPR
//     round trip).  One wavefront instruction fills 1 KiB of contiguous LDS.  Out-of-range
//     pieces (rows past M/N, k past K) are given an offset beyond the buffer's num_records, for
//     which the hardware returns zeros.
//   * LDS layout: row r of the staged tile holds BK elements; its 16-byte chunks are stored at
//     slot (chunk ^ ((r >> SWZ_SH) & (CPR-1))) so that the 16-byte fragment reads of 16
//     consecutive rows fall into distinct banks.  The XOR is applied on the global side of the
//     copy (each lane picks the source chunk that belongs in its fixed LDS slot).
//   * math: v_mfma_f32_32x32x16_bf16 (or 16x16x32 when a wavefront's sub-tile has a 16-wide
//     side); fp8 uses v_mfma_f32_32x32x64_f8f6f4 / 16x16x128 with both operand formats e4m3 and
//     unit block scales.  fp32 accumulation in registers.
//   * pipeline: ST LDS stages in a ring, one barrier per k-tile, fragments double-buffered in
//     registers; every MFMA is followed by at most one fragment read and its share of the refill
//     loads (spread over the whole k-tile when ST >= 3, over its last k-step when ST = 2) and the
//     scheduler is fenced after each such group.  vmcnt is managed by hand (the direct-to-LDS
//     loads are issued from inline asm so that the compiler does not serialise them against
//     every LDS read).
//     The fp8 256x256x128 kernel on four wavefronts (16x16x128 MFMAs, 256 accumulators per lane) keeps ONE set of A
//     fragments that is replaced row by row and double-buffers only the B fragments (GemmTraits::ROLL): two full
//     sets of 8-register fragments do not fit beside the accumulators.
//   * block rasterisation (the micro parameter).  Workgroups are dealt round-robin to the 8 XCDs,
//     each with its own L2.  0 = row-major (so XCD x walks the tile columns x, x+8, ...);
//     1 and 2 give each XCD a contiguous range of a grouped tile sequence (groups of 4 resp. 8
//     tile rows walked column by column), so tiles that share a B panel meet in one L2.  Grids of
//     at most 8 tile rows are one such group under every mode.
//   * split-K (structural parameter S > 1): the grid holds S blocks per output tile, block
//     (tile, s) walks k-tiles [s*Ls, (s+1)*Ls) with Ls = ceil(K / (S*BK)), stores its fp32
//     accumulators to a workspace slab, four registers per lane per 16-byte piece (fully coalesced), and bumps the tile's
//     arrival counter; the block that arrives last adds the S slabs in split order (so the result
//     does not depend on arrival order), writes C and clears the counter.  Nobody waits for anybody.
//     Slabs travel as agent-scope coherent (sc1) 16-byte buffer accesses, the counter as an agent-scope atomic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace wt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

struct GemmArgs {
    const void* A;
    const void* B;
    void* C;
    const float* scaleA;
    const float* scaleB;
    int M, N, K;
    int tiles_m, tiles_n;
    int swizzle;
    int splits;         // S >= 1
    int k_per_split;    // Ls * BK elements (multiple of BK); unused when S == 1
    float* ws;          // S > 1: tiles * S slabs of BM*BN floats
    int* counters;      // S > 1: one arrival counter per tile, zero before and after every launch
    // Grouped GEMM (Table 2, grouped row): rows [off[e], off[e+1]) of A and C belong to group e and
    // are multiplied by B[e] (N x K each).  group_offsets: device pointer to groups+1 ascending row
    // offsets, NULL for a dense GEMM.  M is then the total row count and tiles_m an upper bound
    // (ceil(M/BM) + groups) on the number of row tiles; surplus blocks exit at once.
    const int* group_offsets;
    int groups;
    int vgrid;          // number of tasks; read by the persistent kernel only
    int* queue;         // persistent kernel: NULL = block b runs tasks b, b + grid, ...; else two ints, zero before and
                        // after every launch: [0] hands out the tasks beyond the first grid-ful, [1] counts finished blocks
    int stream_c;       // 1: C is larger than the caches can usefully keep; its line-wise stores carry the non-temporal hint
};

constexpr int kWave = 64;
constexpr uint32_t kOobOffset = 0x7FFFFFF0u;  // >= any num_records we set: reads as zeros
constexpr int kXcd = 8;
constexpr int kGroupM = 8;

// Block rasterisation.  The modes are defined on a grid that is at least as wide as it is tall (rows <= cols) and
// are mirrored -- rows and columns change roles -- on a taller one.  Every order sweeps the long side once per band of
// the short side, so the operand that is read again for every band is the smaller of A and B (the one more likely to
// stay in the memory-side cache), and a tall grid behaves like the wide grid of the transposed problem, which is the
// kind of grid the near-square sampler (n_G >= m_G) profiles.
//   mode 0      plain short-side-major order (column by column on a wide grid): XCD x takes every eighth tile;
//   mode 1, 2   the sequence "bands of 4 (8) rows, each walked column by column" cut into eight contiguous ranges,
//               XCD x taking the x-th: tiles that share panels run on the same XCD and meet in its L2.
// Grids of at most kGroupM rows are walked the same way under every mode: as one band, each XCD a contiguous range.
__host__ __device__ __forceinline__ void tile_coords_wide(int bid, int rows, int cols, int mode, int& r, int& c) {
    if (mode == 0 && rows > kGroupM) {
        c = bid / rows;
        r = bid - c * rows;
        return;
    }
    // XCD x receives the workgroups with bid % 8 == x; hand it the x-th contiguous chunk of the sequence
    const int total = rows * cols;
    const int per = total / kXcd, rem = total - per * kXcd;
    const int xcd = bid % kXcd, local = bid / kXcd;
    const int id = xcd * per + (xcd < rem ? xcd : rem) + local;
    const int band = (mode == 1 && rows > kGroupM) ? kGroupM / 2 : kGroupM;
    const int group = band * cols;
    const int gid = id / group;
    const int first = gid * band;
    const int gm = (rows - first) < band ? (rows - first) : band;
    const int in_group = id - gid * group;
    r = first + in_group % gm;
    c = in_group / gm;
}

__host__ __device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int mode, int& tm, int& tn) {
    if (tiles_m > tiles_n)
        tile_coords_wide(bid, tiles_n, tiles_m, mode, tn, tm);
    else
        tile_coords_wide(bid, tiles_m, tiles_n, mode, tm, tn);
}

__device__ __forceinline__ i32x4 make_rsrc(const void* base, uint32_t num_records) {
    const uint64_t p = reinterpret_cast<uint64_t>(base);
    i32x4 r;
    r.x = static_cast<int>(static_cast<uint32_t>(p));
    r.y = static_cast<int>(static_cast<uint32_t>(p >> 32) & 0xFFFFu);  // stride 0, no swizzle
    r.z = static_cast<int>(num_records);
    r.w = 0x00020000;  // raw buffer, 32-bit data format
    return r;
}

// 16 bytes per lane, global -> LDS.  lds_base is the wave-uniform LDS byte address of the
// 1 KiB destination; lane l lands at lds_base + 16*l.  Source = rsrc base + voffset + soffset.
__device__ __forceinline__ void load_lds_16B(i32x4 rsrc, uint32_t voffset, uint32_t soffset, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, %3 offen lds"
        :
        : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
        : "memory", "m0");
}

__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// keep the instruction scheduler from moving anything across this point
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void block_barrier() {
    asm volatile("s_barrier" ::: "memory");
}

template <int IN>
struct InTraits;
template <>
struct InTraits<0> {  // bf16
    static constexpr int esize = 2;
    static constexpr int epc = 8;  // elements per 16-byte chunk
};
template <>
struct InTraits<1> {  // fp8 e4m3
    static constexpr int esize = 1;
    static constexpr int epc = 16;
};

template <int BM, int BN, int BK, int WM, int WN, int ST, int IN, int OUT, int WK = 1, int MIF = 0>
struct GemmTraits {
    static constexpr int NW = WM * WN * WK;  // WK wavefronts share a sub-tile and divide each k-tile's k-steps
    static constexpr int NT = NW * kWave;
    static constexpr int esize = InTraits<IN>::esize;
    static constexpr int epc = InTraits<IN>::epc;
    static constexpr int RB = BK * esize;        // bytes per staged row
    static constexpr int CPR = RB / 16;          // 16-byte chunks per row
    static constexpr int TM = BM / WM;           // wavefront sub-tile
    static constexpr int TN = BN / WN;
    // MFMA tile side: 32 when the sub-tile allows it, unless the configuration asks for 16 (MIF = 16): for some
    // kernels, notably 256x256x64 on 8 wavefronts, twice as many half-length MFMAs schedule measurably better
    static constexpr int MI = MIF ? MIF : ((TM % 32 == 0 && TN % 32 == 0) ? 32 : 16);
    static_assert(MIF == 0 || MIF == 16, "MFMA tile side override");
    // k extent of one MFMA: bf16 32x32x16 / 16x16x32; fp8 32x32x64 / 16x16x128
    static constexpr int KS = (IN == 0) ? (MI == 32 ? 16 : 32) : (MI == 32 ? 64 : 128);
    static constexpr int CPK = KS * esize / 16;  // chunks one MFMA consumes along k per row
    static constexpr int CPL = CPK / (kWave / MI);  // chunks per lane per MFMA operand
    static constexpr int STAGE_BYTES = (BM + BN) * RB;
    // with WK > 1 the stages are reused, after the main loop, for the partial sub-tiles of the wavefronts wk > 0
    static constexpr int RED_BYTES = (WK - 1) * BM * BN * 4;
    static constexpr int LDS_BYTES = STAGE_BYTES * ST > RED_BYTES ? STAGE_BYTES * ST : RED_BYTES;
    static constexpr int A_INSTR = BM * CPR / kWave;  // 1 KiB wavefront loads per stage
    static constexpr int B_INSTR = BN * CPR / kWave;
    static constexpr int LPW = (A_INSTR + B_INSTR) / NW;  // loads per wavefront per stage
    // when both counts divide evenly, load t of every wavefront is known at compile time to be A or B
    static constexpr bool SPLIT = (A_INSTR % NW == 0) && (B_INSTR % NW == 0);
    static constexpr int SWZ_SH = (RB >= 256) ? 0 : (RB == 128 ? 1 : 2);
    static constexpr int FM = TM / MI, FN = TN / MI;
    static constexpr int ACC = MI * MI / kWave;  // accumulator floats per lane per MFMA tile
    static constexpr int KSTEPS = BK / KS;
    static constexpr int KSW = KSTEPS / WK;       // k-steps of a k-tile that one wavefront computes
    static constexpr int NMK = FM * FN;           // MFMAs per k-step per wavefront
    // With three or more stages the refill of a freed stage is spread over a whole k-tile (the
    // loads of k-tile t+ST-1 ride along the MFMAs of k-tile t); with two stages it has to follow the
    // barrier inside the last k-step (k-tile t+ST then rides along the last MFMAs of k-tile t).
    static constexpr bool SPREAD = ST >= 3;
    // 256 accumulators per lane (one wavefront per SIMD): the MFMAs are issued from inline asm that accumulates in
    // place in the accumulation registers
    static constexpr bool ASMACC = (IN == 0) && (MI == 16) && (FM * FN == 64) && (WK == 1);
    // fp8, 256 accumulators per lane on 16x16x128 MFMAs (asked for with MIF = 16): one k-step per k-tile, a fragment
    // is 8 registers, so two full fragment sets do not fit beside the accumulators.  The A fragments are kept in ONE
    // set and replaced row by row as the MFMAs of a row are issued; only the B fragments are double-buffered.
    static constexpr bool ROLL = (IN == 1) && (MIF == 16) && (FM == 8) && (FN == 8) && (WK == 1) && (ST == 2) && (BK == KS);
    // Epilogue through LDS (when a sub-tile row of C is at least one 128-byte line and the staging fits the
    // workgroup's LDS): the MFMA operands are swapped so that a lane holds four consecutive columns of one row,
    // each wavefront parks one row of MFMA tiles (MI rows x TN columns, converted to the output type) in its own
    // LDS region and reads it back row-contiguous, 16 bytes per lane, so that C is written in whole lines.
    // Rows are padded to a stride of EPI_Q (mod 64) dwords, which spreads both access patterns over the banks.
    static constexpr int OSIZE = OUT == 0 ? 4 : 2;
    static constexpr int EPI_ROW = TN * OSIZE;                               // bytes of one sub-tile row
    // wanted row stride in dwords, mod 64.  (16x16 tiles, bf16 out: an 8-byte write is served 32 lanes at a time -- 16
    // rows x 2 column groups, 4 dwords a row -- so rows 4 dwords apart touch every bank once; measured 2-3 % on
    // launches of one tile per CU.  The same reasoning gives 2 for 32x32 tiles, which measured 4-6 % slower than 4.)
    static constexpr int EPI_Q = (MI == 16 && OSIZE == 2) ? 4 : (kWave / MI) * OSIZE;
    static constexpr int EPI_STRIDE = EPI_ROW + 4 * ((EPI_Q - EPI_ROW / 4) & 63);   // bytes
    static constexpr int EPI_WAVE_BYTES = MI * EPI_STRIDE;
    static constexpr bool LDS_EPI = (WK == 1) && (EPI_ROW >= 128) && (NW * EPI_WAVE_BYTES <= LDS_BYTES);
    // Persistent kernel: when the C staging fits beside the stages, the next task's first k-tiles are requested before
    // this task's epilogue (the staging then lives behind the stages); 16 more bytes hold the next task's index.
    static constexpr int EPI_BYTES = LDS_EPI ? NW * EPI_WAVE_BYTES : 0;
    static constexpr bool PIPE_OK = (ST >= 2) && (WK == 1) && !ROLL && (LDS_BYTES + EPI_BYTES + 16 <= 160 * 1024);
    // (kernels without that room pass the index through the first bytes of the stages, between tasks)
    static constexpr int SLOT_OFF = PIPE_OK ? LDS_BYTES + EPI_BYTES : 0;
    static constexpr int LDS_BYTES_PERSISTENT = PIPE_OK ? SLOT_OFF + 16 : LDS_BYTES;
    static constexpr int EPI_LPR = EPI_ROW / 16;                             // lanes that cover one row, 16 bytes each
    static constexpr int EPI_READS = MI * EPI_ROW / 1024;                    // 1 KiB wavefront reads per MFMA tile row
    static_assert(BK % KS == 0, "BK must hold whole MFMA k-steps");
    static_assert(KSTEPS % WK == 0, "k-steps divide evenly over the WK wavefronts");
    static_assert((BM * CPR) % kWave == 0 && (BN * CPR) % kWave == 0, "whole 1 KiB loads");
    static_assert((A_INSTR + B_INSTR) % NW == 0, "equal loads per wavefront");
    static_assert(TM % MI == 0 && TN % MI == 0, "sub-tile is a whole number of MFMA tiles");
    static_assert(CPR >= 4 && (CPR & (CPR - 1)) == 0, "row of 64..512 bytes");
    static_assert(LPW * (ST - 1) <= 63, "vmcnt range");
    static_assert(ST == 1 || KSTEPS >= 1, "k-steps");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

template <int IN>
struct FragType;
template <>
struct FragType<0> {
    using type = bf16x8;
};
template <>
struct FragType<1> {
    using type = i32x8;
};

template <int MI>
struct AccType;
template <>
struct AccType<32> {
    using type = f32x16;
};
template <>
struct AccType<16> {
    using type = f32x4;
};

// What a task is, in block-uniform scalars: the tile (and split) it computes and where its operands start.
struct TaskDesc {
    int tile, split;
    int row0, m_end, col0;
    int k0, K;            // this task's k range [k0, k0 + K)
    const char* Bbase;
    bool valid;           // false: a surplus task of a grouped launch (past the last row tile)
};

template <class T, int BM, int BN>
__device__ __forceinline__ TaskDesc task_setup(const GemmArgs& args, const int block_id, const int lane) {
    TaskDesc d;
    d.valid = false;
    d.tile = 0; d.split = 0; d.row0 = 0; d.m_end = 0; d.col0 = 0; d.k0 = 0; d.K = 0; d.Bbase = nullptr;
    {
        // blocks [s*tiles, (s+1)*tiles) form split s; within a split the rasterisation is the usual one
        int tile = block_id, split = 0;
        if (args.splits > 1) {
            const int tiles = args.tiles_m * args.tiles_n;
            split = tile / tiles;
            tile -= split * tiles;
        }
        int tm, tn;
        tile_coords(tile, args.tiles_m, args.tiles_n, args.swizzle, tm, tn);
        int row0 = tm * BM, m_end = args.M;
        const int col0 = tn * BN;
        const char* Bbase = static_cast<const char*>(args.B);
        if (args.group_offsets) {
            // tm counts row tiles over the groups' concatenated tile lists: find the group it falls in.
            // Offsets are read on the device (the host never learns the routing) and clipped to [0, M],
            // so whatever they hold, every access stays inside A, B[0..groups) and C.
            // Every wavefront does the lookup for itself: lane l sums the tiles of groups [l*c, (l+1)*c),
            // a scan over the lanes locates the lane whose range holds tm, and only that lane's <= c groups
            // are walked one by one (a serial walk over all groups costs ~0.2 us per group and block, more
            // than a small tile's arithmetic when there are a hundred experts).
            const int E = args.groups;
            auto bounds = [&](int e, int& lo, int& hi) {
                lo = min(max(args.group_offsets[e], 0), args.M);
                hi = min(max(args.group_offsets[e + 1], lo), args.M);
                return (hi - lo + BM - 1) / BM;
            };
            const int c = (E + kWave - 1) / kWave;
            int mine = 0;
            for (int i = 0; i < c; ++i) {
                const int e = lane * c + i;
                int lo, hi;
                if (e < E) mine += bounds(e, lo, hi);
            }
            int incl = mine;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const int v = __shfl_up(incl, d);
                if (lane >= d) incl += v;
            }
            const int excl = incl - mine;
            const unsigned long long hit = __ballot(tm >= excl && tm < incl);
            if (hit == 0) return d;  // past the last row tile
            const int src = __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(hit)) - 1);
            int first = __builtin_amdgcn_readfirstlane(__shfl(excl, src));
            int e = src * c, lo = 0, hi = 0;
            bool found = false;
            for (int i = 0; i < c && e < E; ++i, ++e) {
                const int t = bounds(e, lo, hi);
                if (tm < first + t) { found = true; break; }
                first += t;
            }
            if (!found) return d;
            row0 = lo + (tm - first) * BM;
            m_end = hi;
            Bbase += static_cast<int64_t>(e) * args.N * (static_cast<int64_t>(args.K) * T::esize);
        }
        // this block's k range [k0, k0 + K): the whole of args.K unless split
        int k0 = 0, K = args.K;
        if (args.splits > 1) {
            k0 = split * args.k_per_split;
            K = args.K - k0;
            K = K < 0 ? 0 : (K > args.k_per_split ? args.k_per_split : K);
            if (K == 0) k0 = 0;  // empty range: every load is sent out of range below
        }

        d.tile = tile; d.split = split; d.row0 = row0; d.m_end = m_end; d.col0 = col0; d.k0 = k0; d.K = K; d.Bbase = Bbase;
        d.valid = true;
    }
    return d;
}

// State a persistent block carries from task to task.
struct PipeState {
    TaskDesc next;        // the task after the current one (valid only if have_next)
    int next_id;          // its index in the task list (>= vgrid: none)
    int my_next;          // thread 0: the index obtained for the next task (static stride or from the queue)
    bool have_next;       // next / next_id are filled in
    bool prefetched;      // the first k-tiles of `next` have been requested into the stages
};

// One task of the launch: task `block_id` of the task list (a tile, or one split of a tile).
template <int BM, int BN, int BK, int WM, int WN, int ST, int IN, int OUT, int WK, int MIF = 0, bool PIPE = false>
__device__ __forceinline__ void gemm_task(const GemmArgs& args, const TaskDesc& d, PipeState* const ps = nullptr) {
    using T = GemmTraits<BM, BN, BK, WM, WN, ST, IN, OUT, WK, MIF>;
    using acc_t = typename AccType<T::MI>::type;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wk = wv / (WM * WN), wmn = wv - wk * (WM * WN);  // k slice, position in the sub-tile grid
    const int wm = wmn / WN, wn = wmn - wm * WN;
    {
        const int tile = d.tile, split = d.split, row0 = d.row0, m_end = d.m_end, col0 = d.col0, k0 = d.k0, K = d.K;
        const char* const Bbase = d.Bbase;
        // ---- global -> LDS plan: this wavefront's LPW loads per stage --------------------------
        const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
            (__attribute__((address_space(3))) char*)smem));
        const int64_t row_bytes = static_cast<int64_t>(args.K) * T::esize;
        const int64_t k0_bytes = static_cast<int64_t>(k0) * T::esize;
        auto records = [&](int rows_left) -> uint32_t {  // bytes from the descriptor base to the end of the matrix
            const int64_t b = static_cast<int64_t>(rows_left) * row_bytes - k0_bytes;
            return b > static_cast<int64_t>(kOobOffset) ? kOobOffset : static_cast<uint32_t>(b);
        };
        const i32x4 rsrcA = make_rsrc(static_cast<const char*>(args.A) + static_cast<int64_t>(row0) * row_bytes + k0_bytes,
                                      records(m_end - row0));
        const i32x4 rsrcB = make_rsrc(Bbase + static_cast<int64_t>(col0) * row_bytes + k0_bytes,
                                      records(args.N - col0));
        // has the previous task of this persistent block already requested this task's first k-tiles?
        bool prefetched = false;
        if constexpr (PIPE) prefetched = ps->prefetched;
        // Load slot t of this wavefront fills the 1 KiB LDS piece j = wv + t*NW of a stage.  The lane's
        // source offset at k-tile 0 stays in a register for the whole kernel; the k advance is a scalar.
        // ld_tail[t] is the same offset for the one partial k-tile (K % BK != 0), already replaced by
        // the out-of-range sentinel where the piece lies at or past K, so that it reads as zeros.
        const int L = (K + BK - 1) / BK;
        const int L_full = K / BK;
        uint32_t ld_voff[T::LPW], ld_tail[T::LPW];
    #pragma unroll
        for (int t = 0; t < T::LPW; ++t) {
            const int j = wv + t * T::NW;
            const int p = j * kWave + lane;               // 16-byte slot index inside the stage
            const int r = p / T::CPR;                     // staged row: [0,BM) = A, [BM,BM+BN) = B
            const int slot = p % T::CPR;
            const int chunk = slot ^ ((r >> T::SWZ_SH) & (T::CPR - 1));
            const int rl = (j < T::A_INSTR) ? r : r - BM; // row inside its own matrix tile
            ld_voff[t] = static_cast<uint32_t>(rl) * static_cast<uint32_t>(row_bytes) + chunk * 16;
            ld_tail[t] = (L_full * BK + chunk * T::epc < K) ? ld_voff[t] : kOobOffset;
        }
        // One load: slot t of k-tile kt into LDS stage `stage`.  TAIL = the k-tile may be the partial one
        // or lie past the end (then every piece is out of range and zero-fills the stage), so every
        // k-tile index issues the same number of loads and the vmcnt bookkeeping stays uniform.
        auto issue_load_rs = [&](const i32x4& rA, const i32x4& rB, int t, int kt, int stage, bool tail) {
            const int j = wv + t * T::NW;
            const uint32_t dst = lds0 + stage * T::STAGE_BYTES + j * 1024;
            // The hardware range-checks the per-lane offset only (the scalar offset is added after the
            // check), so anything that must read as zeros is expressed through voff.
            uint32_t koff = static_cast<uint32_t>(kt) * (BK * T::esize);
            uint32_t voff = ld_voff[t];
            if (tail) {
                if (kt >= L_full) voff = (kt < L) ? ld_tail[t] : kOobOffset;  // uniform conditions
                if (kt >= L) koff = 0;
            }
            if constexpr (T::SPLIT) {
                if (t < T::A_INSTR / T::NW)
                    load_lds_16B(rA, voff, koff, dst);
                else
                    load_lds_16B(rB, voff, koff, dst);
            } else {
                const bool is_a = j < T::A_INSTR;  // wave-uniform
                i32x4 rs;
                rs.x = is_a ? rA.x : rB.x;
                rs.y = is_a ? rA.y : rB.y;
                rs.z = is_a ? rA.z : rB.z;
                rs.w = rA.w;
                load_lds_16B(rs, voff, koff, dst);
            }
        };
        auto issue_load = [&](int t, int kt, int stage, bool tail) { issue_load_rs(rsrcA, rsrcB, t, kt, stage, tail); };
        auto issue_tile = [&](int kt, int stage) {
    #pragma unroll
            for (int t = 0; t < T::LPW; ++t) issue_load(t, kt, stage, true);
        };

        // ---- fragment read plan -------------------------------------------------------------------
        // lane -> (row inside an MFMA tile, first chunk along k)
        const int frow = lane % T::MI;
        const int fchunk = (lane / T::MI) * T::CPL;
        acc_t acc[T::FM][T::FN];
    #pragma unroll
        for (int i = 0; i < T::FM; ++i)
    #pragma unroll
            for (int j = 0; j < T::FN; ++j)
    #pragma unroll
                for (int e = 0; e < T::ACC; ++e) acc[i][j][e] = 0.0f;

        using frag_t = typename FragType<IN>::type;
        auto read_frag = [&](int stage, int r, int ks) -> frag_t {
            const int sw = (r >> T::SWZ_SH) & (T::CPR - 1);
            const char* row = smem + stage * T::STAGE_BYTES + r * T::RB;
            const int c0 = (wk * T::KSW + ks) * T::CPK + fchunk;  // this wavefront's slice of the k-tile
            if constexpr (IN == 0) {
                return *reinterpret_cast<const bf16x8*>(row + ((c0 ^ sw) * 16));
            } else {
                // fp8: each lane feeds 32 consecutive k (two 16-byte chunks) of its row
                const i32x4 lo = *reinterpret_cast<const i32x4*>(row + ((c0 ^ sw) * 16));
                const i32x4 hi = *reinterpret_cast<const i32x4*>(row + (((c0 + 1) ^ sw) * 16));
                return i32x8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            }
        };
        struct Frags {
            frag_t a[T::FM];
            frag_t b[T::FN];
        };
        auto load_frags = [&](Frags& f, int stage, int ks) {
    #pragma unroll
            for (int i = 0; i < T::FM; ++i) f.a[i] = read_frag(stage, wm * T::TM + i * T::MI + frow, ks);
    #pragma unroll
            for (int j = 0; j < T::FN; ++j) f.b[j] = read_frag(stage, BM + wn * T::TN + j * T::MI + frow, ks);
        };
        auto mfma = [&](const Frags& f, int i, int j) {
            // x = the MFMA's row operand, y = its column operand.  As (A, B) a lane holds one column of the C tile
            // and groups of four consecutive rows; swapped, (B, A), it holds one row (lane % MI) and groups of four
            // consecutive columns (16x16: 4*(lane/16) + e; 32x32: 8*(e/4) + 4*(lane/32) + e%4).  Products and
            // summation order are the same either way.
            const frag_t& x = T::LDS_EPI ? f.b[j] : f.a[i];
            const frag_t& y = T::LDS_EPI ? f.a[i] : f.b[j];
            if constexpr (IN == 0) {
                if constexpr (T::MI == 32)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[i][j], 0, 0, 0);
                else if constexpr (T::ASMACC)
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(x), "v"(y));
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, acc[i][j], 0, 0, 0);
            } else {
                // cbsz = blgp = 0 select e4m3 for both operands; unit block scales
                if constexpr (T::MI == 32)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x, y, acc[i][j], 0, 0, 0, 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(x, y, acc[i][j], 0, 0, 0, 0, 0, 0);
            }
        };
        auto mma = [&](const Frags& f) {
    #pragma unroll
            for (int i = 0; i < T::FM; ++i)
    #pragma unroll
                for (int j = 0; j < T::FN; ++j) mfma(f, i, j);
        };

        // ---- main loop --------------------------------------------------------------------------------
        constexpr int KSTEPS = T::KSW;  // k-steps this wavefront runs per k-tile
        constexpr int NMK = T::NMK;
        constexpr int NFR = T::FM + T::FN;  // fragments read per k-step
        if constexpr (ST == 1) {
            Frags f;
            for (int kt = 0; kt < L; ++kt) {
                issue_tile(kt, 0);
                wait_vmcnt<0>();
                block_barrier();
    #pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    load_frags(f, 0, ks);
                    mma(f);
                }
                block_barrier();
            }
        } else if constexpr (T::ROLL) {
            // One k-step per k-tile, 64 MFMAs in row-major order (A fragment i against B fragments 0..7).  Everything
            // k-tile t needs from LDS is read during k-tile t-1: B into the other B set, A fragment i into the single
            // A set as soon as row i of k-tile t-1 has been issued.  So when a wavefront has issued row 0 of k-tile t
            // and waited for its reads, it has nothing left to read from stage t%2: it waits for its share of k-tile
            // t+1, meets the others at the barrier, and over rows 1..7 reads k-tile t+1's fragments and (rows 1..4)
            // issues k-tile t+2 into the freed stage.  Row 0 ahead of the barrier hides the latency of the last reads
            // of the previous k-tile (A fragment 7, issued after its row 7).
            static_assert(T::LPW == 16 && KSTEPS == 1, "shape of the rolling schedule");
            frag_t fa[8], fb[2][8];
            if (!prefetched) {
                issue_tile(0, 0);
                issue_tile(1, 1);
                wait_vmcnt<T::LPW>();
            } else {
                wait_vmcnt<0>();
            }
            block_barrier();
    #pragma unroll
            for (int i = 0; i < 8; ++i) fa[i] = read_frag(0, wm * T::TM + i * T::MI + frow, 0);
    #pragma unroll
            for (int j = 0; j < 8; ++j) fb[0][j] = read_frag(0, BM + wn * T::TN + j * T::MI + frow, 0);
            int stage = 0;
            // (LDS epilogue: the B fragment is the MFMA's row operand, the A fragment its column operand)
            auto mf = [&](int i, int j, const frag_t& bj) {
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(bj), "v"(fa[i]));
            };
            static_assert(T::LDS_EPI, "operand order of the in-place MFMA");
            auto tile_body = [&](int kt, auto tail_tag, auto par_tag) {
                constexpr bool TAIL = decltype(tail_tag)::value;
                constexpr int P = decltype(par_tag)::value;
                const int nxt = stage ^ 1;
    #pragma unroll
                for (int j = 0; j < 8; ++j) {
                    mf(0, j, fb[P][j]);
                    sched_fence();
                }
                wait_lgkmcnt0();     // every fragment of k-tile kt is in registers
                wait_vmcnt<0>();     // this wavefront's share of k-tile kt+1 has landed
                block_barrier();
                sched_fence();
    #pragma unroll
                for (int r = 1; r < 8; ++r) {
    #pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        mf(r, j, fb[P][j]);
                        if (j == 0) fa[r - 1] = read_frag(nxt, wm * T::TM + (r - 1) * T::MI + frow, 0);
                        if (j == 4) fb[P ^ 1][r - 1] = read_frag(nxt, BM + wn * T::TN + (r - 1) * T::MI + frow, 0);
                        if (r == 7 && j == 6) fb[P ^ 1][7] = read_frag(nxt, BM + wn * T::TN + 7 * T::MI + frow, 0);
                        if (r <= 4 && (j & 1) == 0) issue_load((r - 1) * 4 + j / 2, kt + 2, stage, TAIL);
                        sched_fence();
                    }
                }
                fa[7] = read_frag(nxt, wm * T::TM + 7 * T::MI + frow, 0);   // (used last; in by the next barrier)
                sched_fence();
                stage = nxt;
            };
            using P0 = std::integral_constant<int, 0>;
            using P1 = std::integral_constant<int, 1>;
            int kt = 0;
            for (; kt + 3 < L_full; kt += 2) {      // both refill targets, kt+2 and kt+3, lie wholly inside K
                tile_body(kt, std::false_type{}, P0{});
                tile_body(kt + 1, std::false_type{}, P1{});
            }
            for (; kt < L; kt += 2) {
                tile_body(kt, std::true_type{}, P0{});
                if (kt + 1 < L) tile_body(kt + 1, std::true_type{}, P1{});
            }
            wait_vmcnt<0>();
            wait_lgkmcnt0();
            asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
        } else {
            // Software pipeline, one barrier per k-tile.  Every MFMA is followed by at most one fragment
            // read and a share of the global->LDS loads, and the scheduler is fenced after each such
            // group, so address arithmetic and memory issue sit in the shadow of the running MFMA.
            //   * fragments of k-step ks+1 are read during the MFMAs of ks (two register sets);
            //   * at the start of the last k-step the wavefront waits for its reads of k-tile t and for
            //     its share of k-tile t+1, meets the others at the barrier (after which stage t%ST is
            //     free and k-tile t+1 is complete), and reads k-tile t+1's first fragments during the
            //     last MFMAs of k-tile t;
            //   * refill: SPREAD (ST >= 3) issues k-tile t+ST-1 into the stage freed one barrier earlier,
            //     evenly over all MFMAs of k-tile t; otherwise k-tile t+ST goes into the stage just freed,
            //     over the MFMAs of the last k-step.
            constexpr int AHEAD = T::SPREAD ? ST - 1 : ST;     // k-tiles issued by the prologue
            constexpr int NM = KSTEPS * NMK;
            // loads placed before the barrier point of a k-tile (SPREAD only)
            constexpr int N_BEFORE = T::SPREAD ? ((KSTEPS - 1) * NMK * T::LPW + NM - 1) / NM : 0;
            constexpr int WAIT_LOOP = T::SPREAD ? T::LPW * (ST - 3) + N_BEFORE : T::LPW * (ST - 2);
            static_assert(WAIT_LOOP <= 63, "vmcnt range");
            Frags f[2];
            if (!prefetched) {
    #pragma unroll
                for (int s = 0; s < AHEAD; ++s) issue_tile(s, s);
                wait_vmcnt<T::LPW*(AHEAD - 1)>();
            } else {
                // requested before the previous task's epilogue; its C stores are in the same counter and loads and
                // stores do not retire in one order, so wait for everything
                wait_vmcnt<0>();
            }
            block_barrier();
            load_frags(f[0], 0, 0);
            int stage = 0;
            auto read_one = [&](Frags& dst, int q, int stg, int ks) {
                if (q < T::FM)
                    dst.a[q] = read_frag(stg, wm * T::TM + q * T::MI + frow, ks);
                else
                    dst.b[q - T::FM] = read_frag(stg, BM + wn * T::TN + (q - T::FM) * T::MI + frow, ks);
            };
            auto tile_body = [&](int kt, auto tail_tag) {
                constexpr bool TAIL = decltype(tail_tag)::value;
                const int nxt = (stage + 1 == ST) ? 0 : stage + 1;
                int fill = stage + (ST - 1);      // SPREAD: stage of k-tile kt+ST-1
                if (fill >= ST) fill -= ST;
    #pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    const bool last = ks == KSTEPS - 1;
                    Frags& cur = f[ks & 1];
                    Frags& nx = f[(ks + 1) & 1];
                    if (last) {
                        wait_lgkmcnt0();          // this wavefront's reads of k-tile kt are done
                        wait_vmcnt<WAIT_LOOP>();  // its share of k-tile kt+1 has landed
                        block_barrier();
                        sched_fence();
                    }
    #pragma unroll
                    for (int idx = 0; idx < NMK; ++idx) {
                        mfma(cur, idx / T::FN, idx % T::FN);
                        // fragment reads for the next k-step, spaced over this k-step's MFMAs and finished a few
                        // MFMAs before its end so that their latency is covered
    #pragma unroll
                        for (int q = 0; q < NFR; ++q)
                            if ((q * (NMK > 4 ? NMK - 3 : 1)) / NFR == idx) read_one(nx, q, last ? nxt : stage, last ? 0 : ks + 1);
                        // refill loads
                        if constexpr (T::SPREAD) {
                            const int g = ks * NMK + idx;
    #pragma unroll
                            for (int l = 0; l < T::LPW; ++l)
                                if ((l * NM) / T::LPW == g) issue_load(l, kt + ST - 1, fill, TAIL);
                        } else {
                            if (last) {
    #pragma unroll
                                for (int l = 0; l < T::LPW; ++l)
                                    if ((l * NMK) / T::LPW == idx) issue_load(l, kt + ST, stage, TAIL);
                            }
                        }
                        sched_fence();
                    }
                }
                if constexpr ((KSTEPS & 1) != 0) f[0] = f[1];
                stage = nxt;
            };
            int kt = 0;
            // k-tiles whose refill target lies wholly inside K need no range handling
            for (; kt + AHEAD < L_full; ++kt) tile_body(kt, std::false_type{});
            for (; kt < L; ++kt) tile_body(kt, std::true_type{});
            wait_vmcnt<0>();
            if constexpr (T::ASMACC) asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
            // ---- hand-over (persistent kernel): request the next task's first k-tiles before this task's epilogue
            if constexpr (PIPE && T::PIPE_OK) {
                if (args.splits == 1) {
                    int* const slot = reinterpret_cast<int*>(smem + T::SLOT_OFF);
                    if (threadIdx.x == 0) *slot = ps->my_next;
                    __syncthreads();   // every wavefront is past its last read of the stages; the slot is written
                    const int nid = __builtin_amdgcn_readfirstlane(*slot);
                    ps->next_id = nid;
                    ps->have_next = true;
                    ps->prefetched = false;
                    if (nid < args.vgrid) {
                        ps->next = task_setup<T, BM, BN>(args, nid, lane);
                        if (ps->next.valid) {
                            const TaskDesc& n = ps->next;   // (splits == 1: same k range, same k-tile counts)
                            const i32x4 nA = make_rsrc(static_cast<const char*>(args.A) + static_cast<int64_t>(n.row0) * row_bytes,
                                                       records(n.m_end - n.row0));
                            const i32x4 nB = make_rsrc(n.Bbase + static_cast<int64_t>(n.col0) * row_bytes, records(args.N - n.col0));
    #pragma unroll
                            for (int s = 0; s < AHEAD; ++s)
    #pragma unroll
                                for (int t = 0; t < T::LPW; ++t) issue_load_rs(nA, nB, t, s, s, true);
                            ps->prefetched = true;
                        }
                    }
                }
            }
        }

        // ---- reduction over the WK wavefronts of a sub-tile --------------------------------------
        // Wavefronts wk > 0 park their partial sub-tile in LDS (the stages are free now), wavefront
        // wk = 0 of each sub-tile adds them in wk order and alone goes on to write C.
        if constexpr (WK > 1) {
            constexpr int NQ = T::FM * T::FN * T::ACC / 4;   // 16-byte pieces per lane
            constexpr int QPT = T::ACC / 4;
            constexpr int SUB = T::TM * T::TN;               // floats per sub-tile
            __syncthreads();                                 // everybody is past its last fragment read
            f32x4* const red = reinterpret_cast<f32x4*>(smem);
            if (wk > 0) {
                f32x4* dst = red + (static_cast<size_t>(wk - 1) * (WM * WN) + wmn) * (SUB / 4) + lane;
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int ij = q / QPT, e0 = 4 * (q % QPT);
                    const acc_t& a = acc[ij / T::FN][ij % T::FN];
                    dst[q * kWave] = f32x4{a[e0], a[e0 + 1], a[e0 + 2], a[e0 + 3]};
                }
            }
            __syncthreads();
            if (wk > 0) return;
#pragma unroll
            for (int k = 1; k < WK; ++k) {
                const f32x4* src = red + (static_cast<size_t>(k - 1) * (WM * WN) + wmn) * (SUB / 4) + lane;
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int ij = q / QPT, e0 = 4 * (q % QPT);
                    acc_t& a = acc[ij / T::FN][ij % T::FN];
                    const f32x4 v = src[q * kWave];
                    a[e0] += v.x; a[e0 + 1] += v.y; a[e0 + 2] += v.z; a[e0 + 3] += v.w;
                }
            }
        }

        // ---- split-K reduction ---------------------------------------------------------------------
        // Partial tiles travel as 16-byte buffer stores / loads marked agent-scope coherent (sc1): the
        // stores write through the XCD's L2 and the loads are served coherently across the XCDs, so no
        // cache-wide write-back or invalidate (what a device-scope fence costs here) is needed.  Order:
        // this block's slab stores are waited for, then the block is counted in with an agent-scope
        // atomic; the block that finds S-1 earlier arrivals knows every slab is in memory.
        if (WK == 1 && args.splits > 1) {   // (split-K keys are built on WK = 1 kernels only)
            constexpr int NREG = T::FM * T::FN * T::ACC;
            constexpr int NQ = NREG / 4;                      // 16-byte pieces per lane
            constexpr int QPT = T::ACC / 4;                   // pieces per MFMA tile
            constexpr uint32_t SLAB_BYTES = static_cast<uint32_t>(NREG) * T::NT * 4;   // = BM*BN*4
            constexpr int SC1 = 16;                           // cache-policy bit: agent-scope coherence
            static_assert(T::ACC % 4 == 0, "accumulators move in groups of four");
            const int S = args.splits;
            const __amdgpu_buffer_rsrc_t ws_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                args.ws + static_cast<size_t>(tile) * S * (SLAB_BYTES / 4), 0, static_cast<int>(S * SLAB_BYTES), 0x00020000);
            const uint32_t lane_off = threadIdx.x * 16u;
            const uint32_t mine = static_cast<uint32_t>(split) * SLAB_BYTES + lane_off;
    #pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int ij = q / QPT, e0 = 4 * (q % QPT);
                const acc_t& a = acc[ij / T::FN][ij % T::FN];
                const u32x4 v = {__float_as_uint(a[e0]), __float_as_uint(a[e0 + 1]), __float_as_uint(a[e0 + 2]),
                                 __float_as_uint(a[e0 + 3])};
                __builtin_amdgcn_raw_buffer_store_b128(v, ws_rsrc, mine + q * (T::NT * 16), 0, SC1);
            }
            wait_vmcnt<0>();   // this lane's slab stores have been acknowledged
            __syncthreads();   // ... and everybody's; every wavefront is also past its last LDS access
            int* flag = reinterpret_cast<int*>(smem);
            if (threadIdx.x == 0)
                *flag = __hip_atomic_fetch_add(args.counters + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*flag != S - 1) return;
            // Sum in split order, whatever the arrival order.  S is dispatched to a compile-time constant
            // so that the loads of all slabs are independent and in flight together.
            auto reduce = [&](auto s_tag) {
                constexpr int SS = decltype(s_tag)::value;
    #pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int ij = q / QPT, e0 = 4 * (q % QPT);
                    float v0 = 0.0f, v1 = 0.0f, v2 = 0.0f, v3 = 0.0f;
    #pragma unroll
                    for (int sp = 0; sp < SS; ++sp) {
                        const u32x4 p = __builtin_amdgcn_raw_buffer_load_b128(
                            ws_rsrc, sp * SLAB_BYTES + lane_off + q * (T::NT * 16), 0, SC1);
                        v0 += __uint_as_float(p.x); v1 += __uint_as_float(p.y);
                        v2 += __uint_as_float(p.z); v3 += __uint_as_float(p.w);
                    }
                    acc_t& a = acc[ij / T::FN][ij % T::FN];
                    a[e0] = v0; a[e0 + 1] = v1; a[e0 + 2] = v2; a[e0 + 3] = v3;
                }
            };
            if (S == 2) reduce(std::integral_constant<int, 2>{});
            else if (S == 4) reduce(std::integral_constant<int, 4>{});
            else reduce(std::integral_constant<int, 8>{});
            if (threadIdx.x == 0)   // ready for the next launch on this stream
                __hip_atomic_store(args.counters + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // ---- epilogue ---------------------------------------------------------------------------------
        float scale = 1.0f;
        if constexpr (IN == 1) scale = args.scaleA[0] * args.scaleB[0];
        const int M = m_end, N = args.N;
        if constexpr (T::LDS_EPI) {
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            constexpr int EPV = 16 / T::OSIZE;           // elements per 16-byte piece
            constexpr int NGRP = T::ACC / 4;             // column groups a lane holds per MFMA tile
            // rows of C keep 16-byte alignment when N is a multiple of EPV and C itself is aligned (wave-uniform)
            const bool vec_ok = (N % EPV == 0) && ((reinterpret_cast<uintptr_t>(args.C) & 15) == 0);
            if (!vec_ok) {
                // rows of C are not 16-byte aligned: element by element straight from the registers
                const int lrow = lane % T::MI, lcol = 4 * (lane / T::MI);
    #pragma unroll
                for (int i = 0; i < T::FM; ++i) {
                    const int row = row0 + wm * T::TM + i * T::MI + lrow;
    #pragma unroll
                    for (int j = 0; j < T::FN; ++j) {
    #pragma unroll
                        for (int e = 0; e < T::ACC; ++e) {
                            const int col = col0 + wn * T::TN + j * T::MI + 8 * (e / 4) + lcol + (e % 4);
                            if (row < M && col < N) {
                                float v = acc[i][j][e];
                                if constexpr (IN == 1) v *= scale;
                                const int64_t idx = static_cast<int64_t>(row) * N + col;
                                if constexpr (OUT == 0)
                                    static_cast<float*>(args.C)[idx] = v;
                                else
                                    static_cast<__bf16*>(args.C)[idx] = static_cast<__bf16>(v);
                            }
                        }
                    }
                }
                return;
            }
            // the persistent kernel stages C behind the stages, which may already be receiving the next task
            constexpr int EPI_BASE = (PIPE && T::PIPE_OK) ? T::LDS_BYTES : 0;
            if (!(PIPE && T::PIPE_OK) || args.splits > 1)
                __syncthreads();   // every wavefront is past its last read of the stages (and of the split-K flag)
            char* const mine = smem + EPI_BASE + wv * T::EPI_WAVE_BYTES;
            char* const wr = mine + (lane % T::MI) * T::EPI_STRIDE + (4 * (lane / T::MI)) * T::OSIZE;
    #pragma unroll
            for (int i = 0; i < T::FM; ++i) {
    #pragma unroll
                for (int j = 0; j < T::FN; ++j) {
    #pragma unroll
                    for (int g = 0; g < NGRP; ++g) {
                        float v[4];
    #pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            v[e] = acc[i][j][4 * g + e];
                            if constexpr (IN == 1) v[e] *= scale;
                        }
                        char* dst = wr + (j * T::MI + 8 * g) * T::OSIZE;
                        if constexpr (OUT == 0)
                            *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                        else
                            *reinterpret_cast<bf16x4*>(dst) = bf16x4{static_cast<__bf16>(v[0]), static_cast<__bf16>(v[1]),
                                                                      static_cast<__bf16>(v[2]), static_cast<__bf16>(v[3])};
                    }
                }
                // (LDS serves one wavefront's accesses in order: the reads below see the writes above)
    #pragma unroll
                for (int t = 0; t < T::EPI_READS; ++t) {
                    const int p = t * kWave + lane;
                    const int r = p / T::EPI_LPR, k = p % T::EPI_LPR;
                    const f32x4 piece = *reinterpret_cast<const f32x4*>(mine + r * T::EPI_STRIDE + k * 16);
                    const int row = row0 + wm * T::TM + i * T::MI + r;
                    const int col = col0 + wn * T::TN + k * EPV;
                    // col and N are multiples of EPV here, so a piece that starts inside the matrix lies wholly inside
                    if (row < M && col < N) {
                        f32x4* const dst =
                            reinterpret_cast<f32x4*>(static_cast<char*>(args.C) + (static_cast<int64_t>(row) * N + col) * T::OSIZE);
                        // A C too large to stay cached only evicts operand panels on its way out: mark it streaming
                        // (1.5 % on 16384 x 8192 x 8192; no effect on 4096 x 11008 x 4096).  Wave-uniform choice.
                        if (args.stream_c)
                            __builtin_nontemporal_store(piece, dst);
                        else
                            *dst = piece;
                    }
                }
                wait_lgkmcnt0();   // the pieces are in registers before the next tile row overwrites the region
            }
        } else {
    #pragma unroll
            for (int i = 0; i < T::FM; ++i) {
    #pragma unroll
                for (int j = 0; j < T::FN; ++j) {
                    const int col = col0 + wn * T::TN + j * T::MI + (lane % T::MI);
    #pragma unroll
                    for (int e = 0; e < T::ACC; ++e) {
                        // 32x32: row = 8*(e/4) + 4*(lane/32) + e%4 ; 16x16: row = 4*(lane/16) + e
                        const int rin = (T::MI == 32) ? (8 * (e / 4) + 4 * (lane / 32) + (e % 4)) : (4 * (lane / 16) + e);
                        const int row = row0 + wm * T::TM + i * T::MI + rin;
                        if (row < M && col < N) {
                            float v = acc[i][j][e];
                            if constexpr (IN == 1) v *= scale;
                            const int64_t idx = static_cast<int64_t>(row) * N + col;
                            if constexpr (OUT == 0)
                                static_cast<float*>(args.C)[idx] = v;
                            else
                                static_cast<__bf16*>(args.C)[idx] = static_cast<__bf16>(v);
                        }
                    }
                }
            }
        }
    }
}

// One block per task.
template <int BM, int BN, int BK, int WM, int WN, int ST, int IN, int OUT, int WK = 1, int MIF = 0>
__global__ __launch_bounds__(WM* WN* WK* kWave) void gemm_kernel(const GemmArgs args) {
    using T = GemmTraits<BM, BN, BK, WM, WN, ST, IN, OUT, WK, MIF>;
    const TaskDesc d = task_setup<T, BM, BN>(args, blockIdx.x, threadIdx.x & (kWave - 1));
    if (!d.valid) return;
    gemm_task<BM, BN, BK, WM, WN, ST, IN, OUT, WK, MIF>(args, d);
}

// Persistent launch (Sec. 3.2, note on persistent kernels): the host starts only as many blocks as can be resident at
// once and every block works through tasks of the same task list, so G stays the logical task count while the
// physical grid is clamped.  A block's first task is its own index; further tasks are either index + grid, ... or, when
// args.queue is set, fetched from a global counter as the block gets to them (workers drawing from a queue).  Where
// the layout allows (T::PIPE_OK, unsplit tasks) a task's first k-tiles are requested before the previous task's
// epilogue, so the C stores of one tile and the first loads of the next overlap.
template <int BM, int BN, int BK, int WM, int WN, int ST, int IN, int OUT, int WK = 1, int MIF = 0>
__global__ __launch_bounds__(WM* WN* WK* kWave) void gemm_kernel_persistent(const GemmArgs args) {
    using T = GemmTraits<BM, BN, BK, WM, WN, ST, IN, OUT, WK, MIF>;
    static_assert(T::LDS_BYTES_PERSISTENT <= 160 * 1024, "LDS per workgroup");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int lane = threadIdx.x & (kWave - 1);
    int* const slot = reinterpret_cast<int*>(smem + T::SLOT_OFF);
    PipeState ps;
    ps.prefetched = false;
    int id = blockIdx.x;
    TaskDesc cur = task_setup<T, BM, BN>(args, id, lane);
    while (id < args.vgrid) {
        // the index of the task after this one: asked for now, needed when this task's main loop is over
        ps.my_next = id + static_cast<int>(gridDim.x);
        if (args.queue && threadIdx.x == 0)
            ps.my_next = static_cast<int>(gridDim.x) +
                         __hip_atomic_fetch_add(args.queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ps.have_next = false;
        if (cur.valid) gemm_task<BM, BN, BK, WM, WN, ST, IN, OUT, WK, MIF, true>(args, cur, &ps);
        if (!ps.have_next) {
            // no hand-over inside the task: agree on the next index here; LDS is free again after the barrier
            __syncthreads();
            if (threadIdx.x == 0) *slot = ps.my_next;
            __syncthreads();
            ps.next_id = __builtin_amdgcn_readfirstlane(*slot);
            if constexpr (!T::PIPE_OK) __syncthreads();   // the slot lies inside the stages: read it before they refill
            ps.prefetched = false;
            if (ps.next_id < args.vgrid) ps.next = task_setup<T, BM, BN>(args, ps.next_id, lane);
        }
        id = ps.next_id;
        cur = ps.next;
    }
    if (args.queue) {
        // the last block to run out of tasks puts both counters back to zero for the next launch
        if (threadIdx.x == 0) {
            const int done = __hip_atomic_fetch_add(args.queue + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == static_cast<int>(gridDim.x) - 1) {
                __hip_atomic_store(args.queue, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(args.queue + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

}  // namespace wt
