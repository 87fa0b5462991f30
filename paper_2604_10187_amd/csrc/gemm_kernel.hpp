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
//     side); fp8 uses v_mfma_f32_16x16x128_f8f6f4.  fp32 accumulation in registers.
//   * pipeline: ST LDS stages in a ring; loads of tile kt+ST-1 are issued right after the barrier
//     that frees their stage and complete behind the MFMAs of tiles kt..kt+ST-2.  vmcnt is
//     managed by hand (the direct-to-LDS loads are issued from inline asm so that the compiler
//     does not serialise them against every LDS read).
//   * block rasterisation (the micro parameter): 0 = row-major, 1 = groups of 8 tile rows,
//     2 = per-XCD contiguous ranges (workgroups are dealt round-robin to the 8 XCDs, each with its
//     own L2) followed by the grouping of mode 1.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
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
};

constexpr int kWave = 64;
constexpr uint32_t kOobOffset = 0x7FFFFFF0u;  // >= any num_records we set: reads as zeros
constexpr int kXcd = 8;
constexpr int kGroupM = 8;

__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int mode, int& tm, int& tn) {
    if (mode == 0) {
        tm = bid / tiles_n;
        tn = bid - tm * tiles_n;
        return;
    }
    int id = bid;
    if (mode == 2) {
        const int total = tiles_m * tiles_n;
        const int per = total / kXcd, rem = total - per * kXcd;
        const int xcd = bid % kXcd, local = bid / kXcd;
        id = xcd * per + (xcd < rem ? xcd : rem) + local;
    }
    const int group = kGroupM * tiles_n;
    const int gid = id / group;
    const int first_m = gid * kGroupM;
    const int gm = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
    const int in_group = id - gid * group;
    tm = first_m + in_group % gm;
    tn = in_group / gm;
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
// 1 KiB destination; lane l lands at lds_base + 16*l.
__device__ __forceinline__ void load_lds_16B(i32x4 rsrc, uint32_t voffset, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "buffer_load_dwordx4 %1, %2, 0 offen lds"
        :
        : "s"(lds_base), "v"(voffset), "s"(rsrc)
        : "memory");
}

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

template <int BM, int BN, int BK, int WM, int WN, int ST, int IN, int OUT>
struct GemmTraits {
    static constexpr int NW = WM * WN;
    static constexpr int NT = NW * kWave;
    static constexpr int esize = InTraits<IN>::esize;
    static constexpr int epc = InTraits<IN>::epc;
    static constexpr int RB = BK * esize;        // bytes per staged row
    static constexpr int CPR = RB / 16;          // 16-byte chunks per row
    static constexpr int TM = BM / WM;           // wavefront sub-tile
    static constexpr int TN = BN / WN;
    static constexpr int MI = (IN == 0 && TM % 32 == 0 && TN % 32 == 0) ? 32 : 16;
    // k extent of one MFMA: bf16 32x32x16 / 16x16x32; fp8 16x16x128
    static constexpr int KS = (IN == 0) ? (MI == 32 ? 16 : 32) : 128;
    static constexpr int CPK = KS * esize / 16;  // chunks one MFMA consumes along k per row
    static constexpr int CPL = CPK / (kWave / MI);  // chunks per lane per MFMA operand
    static constexpr int STAGE_BYTES = (BM + BN) * RB;
    static constexpr int LDS_BYTES = STAGE_BYTES * ST;
    static constexpr int A_INSTR = BM * CPR / kWave;  // 1 KiB wavefront loads per stage
    static constexpr int B_INSTR = BN * CPR / kWave;
    static constexpr int LPW = (A_INSTR + B_INSTR) / NW;  // loads per wavefront per stage
    // when both counts divide evenly, load t of every wavefront is known at compile time to be A or B
    static constexpr bool SPLIT = (A_INSTR % NW == 0) && (B_INSTR % NW == 0);
    static constexpr int SWZ_SH = (RB >= 256) ? 0 : (RB == 128 ? 1 : 2);
    static constexpr int FM = TM / MI, FN = TN / MI;
    static constexpr int ACC = MI * MI / kWave;  // accumulator floats per lane per MFMA tile
    static_assert(BK % KS == 0, "BK must hold whole MFMA k-steps");
    static_assert((BM * CPR) % kWave == 0 && (BN * CPR) % kWave == 0, "whole 1 KiB loads");
    static_assert((A_INSTR + B_INSTR) % NW == 0, "equal loads per wavefront");
    static_assert(TM % MI == 0 && TN % MI == 0, "sub-tile is a whole number of MFMA tiles");
    static_assert(CPR >= 4 && (CPR & (CPR - 1)) == 0, "row of 64..512 bytes");
    static_assert(LPW * (ST > 2 ? ST - 2 : 0) <= 63, "vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
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

template <int BM, int BN, int BK, int WM, int WN, int ST, int IN, int OUT>
__global__ __launch_bounds__(WM* WN* kWave) void gemm_kernel(const GemmArgs args) {
    using T = GemmTraits<BM, BN, BK, WM, WN, ST, IN, OUT>;
    using acc_t = typename AccType<T::MI>::type;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wv / WN, wn = wv - wm * WN;

    int tm, tn;
    tile_coords(blockIdx.x, args.tiles_m, args.tiles_n, args.swizzle, tm, tn);
    const int row0 = tm * BM, col0 = tn * BN;
    const int K = args.K;

    // ---- global -> LDS plan: this wavefront's LPW loads per stage --------------------------
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) char*)smem));
    const int64_t row_bytes = static_cast<int64_t>(K) * T::esize;
    auto records = [&](int rows_left) -> uint32_t {
        const int64_t b = static_cast<int64_t>(rows_left) * row_bytes;
        return b > static_cast<int64_t>(kOobOffset) ? kOobOffset : static_cast<uint32_t>(b);
    };
    const i32x4 rsrcA = make_rsrc(static_cast<const char*>(args.A) + static_cast<int64_t>(row0) * row_bytes,
                                  records(args.M - row0));
    const i32x4 rsrcB = make_rsrc(static_cast<const char*>(args.B) + static_cast<int64_t>(col0) * row_bytes,
                                  records(args.N - col0));
    uint32_t ld_voff[T::LPW];  // byte offset of this lane's piece at k-tile 0 (relative to the tile's first row)
    uint32_t ld_k[T::LPW];     // element offset of the piece inside a k-tile
#pragma unroll
    for (int t = 0; t < T::LPW; ++t) {
        const int j = wv + t * T::NW;                 // 1 KiB slot index inside the stage
        const int p = j * kWave + lane;               // 16-byte slot index inside the stage
        const int r = p / T::CPR;                     // staged row: [0,BM) = A, [BM,BM+BN) = B
        const int slot = p % T::CPR;
        const int chunk = slot ^ ((r >> T::SWZ_SH) & (T::CPR - 1));
        const int rl = (j < T::A_INSTR) ? r : r - BM; // row inside its own matrix tile
        ld_voff[t] = static_cast<uint32_t>(rl) * static_cast<uint32_t>(row_bytes) + chunk * 16;
        ld_k[t] = chunk * T::epc;
    }
    auto issue_tile = [&](int kt, int stage) {
        const int k0 = kt * BK;
#pragma unroll
        for (int t = 0; t < T::LPW; ++t) {
            const int j = wv + t * T::NW;
            const bool in_k = (k0 + static_cast<int>(ld_k[t])) < K;
            const uint32_t off = in_k ? ld_voff[t] + static_cast<uint32_t>(k0) * T::esize : kOobOffset;
            const uint32_t dst = lds0 + stage * T::STAGE_BYTES + j * 1024;
            if constexpr (T::SPLIT) {
                if (t < T::A_INSTR / T::NW)
                    load_lds_16B(rsrcA, off, dst);
                else
                    load_lds_16B(rsrcB, off, dst);
            } else {
                const bool is_a = j < T::A_INSTR;  // wave-uniform
                i32x4 rs;
                rs.x = is_a ? rsrcA.x : rsrcB.x;
                rs.y = is_a ? rsrcA.y : rsrcB.y;
                rs.z = is_a ? rsrcA.z : rsrcB.z;
                rs.w = rsrcA.w;
                load_lds_16B(rs, off, dst);
            }
        }
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

    auto frag_ptr = [&](int stage, int r, int chunk) -> const char* {
        const int slot = chunk ^ ((r >> T::SWZ_SH) & (T::CPR - 1));
        return smem + stage * T::STAGE_BYTES + r * T::RB + slot * 16;
    };

    auto compute_tile = [&](int stage) {
#pragma unroll
        for (int ks = 0; ks < BK / T::KS; ++ks) {
            if constexpr (IN == 0) {
                bf16x8 af[T::FM], bfr[T::FN];
#pragma unroll
                for (int i = 0; i < T::FM; ++i)
                    af[i] = *reinterpret_cast<const bf16x8*>(
                        frag_ptr(stage, wm * T::TM + i * T::MI + frow, ks * T::CPK + fchunk));
#pragma unroll
                for (int j = 0; j < T::FN; ++j)
                    bfr[j] = *reinterpret_cast<const bf16x8*>(
                        frag_ptr(stage, BM + wn * T::TN + j * T::MI + frow, ks * T::CPK + fchunk));
#pragma unroll
                for (int i = 0; i < T::FM; ++i)
#pragma unroll
                    for (int j = 0; j < T::FN; ++j) {
                        if constexpr (T::MI == 32)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
                    }
            } else {
                // fp8: each lane feeds 32 consecutive k (two 16-byte chunks) of its row
                i32x8 af[T::FM], bfr[T::FN];
#pragma unroll
                for (int i = 0; i < T::FM; ++i) {
                    const int r = wm * T::TM + i * T::MI + frow;
                    const i32x4 lo = *reinterpret_cast<const i32x4*>(frag_ptr(stage, r, ks * T::CPK + fchunk));
                    const i32x4 hi = *reinterpret_cast<const i32x4*>(frag_ptr(stage, r, ks * T::CPK + fchunk + 1));
                    af[i] = i32x8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                }
#pragma unroll
                for (int j = 0; j < T::FN; ++j) {
                    const int r = BM + wn * T::TN + j * T::MI + frow;
                    const i32x4 lo = *reinterpret_cast<const i32x4*>(frag_ptr(stage, r, ks * T::CPK + fchunk));
                    const i32x4 hi = *reinterpret_cast<const i32x4*>(frag_ptr(stage, r, ks * T::CPK + fchunk + 1));
                    bfr[j] = i32x8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                }
#pragma unroll
                for (int i = 0; i < T::FM; ++i)
#pragma unroll
                    for (int j = 0; j < T::FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                            af[i], bfr[j], acc[i][j], 0 /*A: e4m3*/, 0 /*B: e4m3*/, 0, 0, 0, 0);
            }
        }
    };

    // ---- main loop --------------------------------------------------------------------------------
    const int L = (K + BK - 1) / BK;
    if constexpr (ST == 1) {
        for (int kt = 0; kt < L; ++kt) {
            issue_tile(kt, 0);
            wait_vmcnt<0>();
            block_barrier();
            compute_tile(0);
            block_barrier();
        }
    } else {
        // prologue: tiles 0..ST-2 (tiles past L are all out of range and load zeros)
#pragma unroll
        for (int s = 0; s < ST - 1; ++s) issue_tile(s, s);
        int stage = 0;
        for (int kt = 0; kt < L; ++kt) {
            wait_vmcnt<T::LPW*(ST - 2)>();  // tile kt has landed (this wavefront's share)
            block_barrier();                // ... everyone's share; and stage (kt-1)%ST is free
            int nxt = stage + (ST - 1);
            if (nxt >= ST) nxt -= ST;
            issue_tile(kt + ST - 1, nxt);
            compute_tile(stage);
            stage = (stage + 1 == ST) ? 0 : stage + 1;
        }
        wait_vmcnt<0>();
    }

    // ---- epilogue ---------------------------------------------------------------------------------
    float scale = 1.0f;
    if constexpr (IN == 1) scale = args.scaleA[0] * args.scaleB[0];
    const int M = args.M, N = args.N;
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

}  // namespace wt
