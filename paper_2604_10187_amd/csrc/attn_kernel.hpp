// FlashAttention-style forward kernel for gfx950 (bf16 in / bf16 out, head dimension 128), the second tile-based
// kernel behind the <G, L> abstraction (Table 2, FlashAttention row: a block owns T_Q query rows of one head and
// loops over ceil(S_kv / T_KV) key/value tiles).
//
// Layout.  Q and O are [batch, S_q, H_q, 128], K and V are [batch, S_kv, H_kv, 128] (token-major, head dimension
// contiguous); query head h reads KV head h / (H_q / H_kv).
//
// Per block: NW wavefronts, each owning R = T_Q / NW query rows (32 or 64) and keeping their Q fragments in
// registers.  Per KV tile:
//   * S^T = K Q^T on v_mfma_f32_32x32x16_bf16 with K as the row operand, so a lane ends up with ONE query column
//     and 16 key rows per 32-key block: the row maximum and row sum of the online softmax are in-lane reductions
//     plus a single exchange with lane ^ 32, and the rescale factor is a per-lane scalar;
//   * P^T (bf16) is fed back as the column operand of O^T += V^T P^T straight from those accumulator registers
//     (eight consecutive accumulators are one k-step); the contraction order over keys that this implies
//     (key = 32b + 8(e/4) + 4(lane/32) + e%4) is baked into how V is laid out in LDS;
//   * K and V both go to LDS row-major as loaded (16 bytes per lane, rows padded).  The V^T operand of O^T += V^T P^T
//     needs, per lane, four consecutive keys of ONE head dimension -- a column of the staged tile -- and is read
//     with the transposing LDS read (ds_read_b64_tr_b16): within 16 lanes, lane s supplies the 8-byte piece
//     (key k0 + s/4, dims d0 + 4*(s%4) .. +3) and lane j receives (keys k0 .. k0+3, dim d0 + j); two such reads make
//     one operand, and no vector ALU work goes into the transposition;
//   * the global loads of tile t+1 are issued right after the barrier that publishes tile t and land in registers
//     while tile t is computed; two barriers per tile (publish / release);
//   * softmax in base 2 with the scale folded into one fma per element (the running maximum is kept in raw score
//     units, which needs scale > 0), and the rescale of O skipped when no lane's maximum moved.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wt {

constexpr int kHeadDim = 128;
constexpr int kAttnOrders = 3;  // micro parameter: block -> (head, query tile) order
constexpr int kAttnXcd = 8;

typedef __attribute__((ext_vector_type(8))) __bf16 abf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 abf16x4;
typedef __attribute__((ext_vector_type(16))) float af32x16;
typedef __attribute__((ext_vector_type(4))) unsigned au32x4;
typedef __attribute__((ext_vector_type(2))) unsigned au32x2;
typedef __attribute__((ext_vector_type(4))) short as16x4;

struct AttnArgs {
    const __bf16* Q;
    const __bf16* K;
    const __bf16* V;
    __bf16* O;
    int S_q, S_kv, H_q, H_kv;
    int batch;         // sequences per launch (>= 1): Q/O are [batch, S_q, H_q, 128], K/V [batch, S_kv, H_kv, 128]; blocks are
                       // mapped as if the launch had batch * H_q heads (Table 2: a batch multiplies N_h in G)
    // Variable-length batch (cu_q != NULL): the sequences' tokens are packed back to back, Q/O [S_q, H_q, 128] and K/V
    // [S_kv, H_kv, 128] with S_q / S_kv the TOTAL token counts; cu_q / cu_kv are device pointers to batch + 1 ascending
    // token offsets (sequence b owns [cu[b], cu[b+1])).  q_tiles is then an upper bound, ceil(S_q / T_Q) + batch, on
    // the query tiles of all sequences together; surplus blocks exit at once.  The offsets are read on the device
    // only and clipped to [0, S_q] / [0, S_kv], so whatever they hold, every access stays inside the tensors.
    const int* cu_q;
    const int* cu_kv;
    int q_tiles;       // ceil(S_q / T_Q)
    int order;         // 0: query tiles of a head are consecutive blocks; 1: heads are consecutive blocks;
                       // 2: like 0, but every XCD (blocks are dealt round-robin to 8 of them) gets a contiguous range
    int causal;        // 1: query i sees keys j <= i + (S_kv - S_q)
    float scale_log2;  // softmax scale times log2(e)
};

// Block index -> (head, query tile).  Also run on the host by the tests.
__host__ __device__ inline void attn_block_coords(int block, int n_heads, int q_tiles, int order, int& head, int& qt) {
    if (order == 1) {
        qt = block / n_heads;
        head = block % n_heads;
        return;
    }
    int v = block;
    if (order == 2) {
        const int G = n_heads * q_tiles, x = block % kAttnXcd, r = block / kAttnXcd;
        const int per = G / kAttnXcd, rem = G % kAttnXcd;
        v = x * per + (x < rem ? x : rem) + r;  // XCD x owns per + (x < rem) consecutive entries
    }
    head = v / q_tiles;
    qt = v % q_tiles;
}

template <int TQ, int TKV, int NW>
struct AttnTraits {
    static constexpr int R = TQ / NW;   // query rows per wavefront
    static constexpr int RB = R / 32;   // 32-row blocks per wavefront
    static constexpr int NT = NW * 64;
    static constexpr int KB = TKV / 32;                 // 32-key blocks per tile
    static constexpr int K_ROW = kHeadDim * 2 + 16;     // bytes per key row in LDS (padded: conflict-free 16-byte reads)
    // bytes per key row of V in LDS: 16 dwords (mod 64) apart, so that the four key rows one transposing read touches
    // (64 contiguous bytes of each, per half wavefront) fall on disjoint banks
    static constexpr int V_ROW = kHeadDim * 2 + 64;
    static constexpr int K_BYTES = TKV * K_ROW;
    static constexpr int V_BYTES = TKV * V_ROW;
    static constexpr int LDS_BYTES = K_BYTES + V_BYTES;
    static constexpr int K_TOTAL = TKV * 16;            // 16-byte chunks of a K tile
    static constexpr int KC = (K_TOTAL + NT - 1) / NT;  // per thread
    static_assert(TQ % NW == 0 && (R == 32 || R == 64), "a wavefront owns 32 or 64 query rows");
    static_assert(TKV % 32 == 0 && TKV >= 32, "KV tile is a multiple of 32 keys");
};

template <int TQ, int TKV, int NW>
__global__ __launch_bounds__(NW * 64) void attn_kernel(const AttnArgs a) {
    using T = AttnTraits<TQ, TKV, NW>;
    extern __shared__ __attribute__((aligned(16))) char attn_smem[];
    char* const k_lds = attn_smem;
    char* const v_lds = attn_smem + T::K_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    int head, qt;
    int S_q = a.S_q, S_kv = a.S_kv;          // this block's sequence
    int64_t q_tok0 = 0, kv_tok0 = 0;         // its first query / key token in the tensors
    if (a.cu_q == nullptr) {
        attn_block_coords(static_cast<int>(blockIdx.x), a.batch * a.H_q, a.q_tiles, a.order, head, qt);
        const int seq = head / a.H_q;        // which sequence of the batch (block-uniform)
        head -= seq * a.H_q;
        q_tok0 = static_cast<int64_t>(seq) * a.S_q;
        kv_tok0 = static_cast<int64_t>(seq) * a.S_kv;
    } else {
        // qt counts query tiles over the sequences' concatenated tile lists: find the sequence it falls in.  Every
        // wavefront does the lookup for itself: lane l sums the tiles of sequences [l*c, (l+1)*c), a scan over the
        // lanes locates the lane whose range holds qt, and only that lane's <= c sequences are walked one by one.
        attn_block_coords(static_cast<int>(blockIdx.x), a.H_q, a.q_tiles, a.order, head, qt);
        const int B = a.batch;
        auto bounds = [&](const int* cu, int total, int b, int& lo, int& hi) {
            lo = min(max(cu[b], 0), total);
            hi = min(max(cu[b + 1], lo), total);
        };
        const int c = (B + 63) / 64;
        int mine = 0;
        for (int i = 0; i < c; ++i) {
            const int b = lane * c + i;
            int lo, hi;
            if (b < B) { bounds(a.cu_q, a.S_q, b, lo, hi); mine += (hi - lo + TQ - 1) / TQ; }
        }
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int v = __shfl_up(incl, d);
            if (lane >= d) incl += v;
        }
        const int excl = incl - mine;
        // Causal batch: a sequence's later query tiles loop over more keys, so the concatenated tile list is walked
        // backwards -- every sequence's longest tiles before its shortest, and the launch ends on short blocks.
        const int total_tiles = __builtin_amdgcn_readfirstlane(__shfl(incl, 63));
        if (qt >= total_tiles) return;       // past the last query tile of the batch
        if (a.causal) qt = total_tiles - 1 - qt;
        const unsigned long long hit = __ballot(qt >= excl && qt < incl);
        if (hit == 0) return;
        const int src = __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(hit)) - 1);
        int first = __builtin_amdgcn_readfirstlane(__shfl(excl, src));
        int b = src * c, lo = 0, hi = 0;
        bool found = false;
        for (int i = 0; i < c && b < B; ++i, ++b) {
            bounds(a.cu_q, a.S_q, b, lo, hi);
            const int t = (hi - lo + TQ - 1) / TQ;
            if (qt < first + t) { found = true; break; }
            first += t;
        }
        if (!found) return;
        qt -= first;
        S_q = hi - lo;
        q_tok0 = lo;
        int klo, khi;
        bounds(a.cu_kv, a.S_kv, b, klo, khi);
        S_kv = khi - klo;
        kv_tok0 = klo;
    }
    // the query tiles with the most keys start first (a variable-length batch has reversed its tile list above)
    if (a.causal && a.cu_q == nullptr) qt = a.q_tiles - 1 - qt;
    const __bf16* const Qs = a.Q + q_tok0 * a.H_q * kHeadDim;
    const __bf16* const Ks = a.K + kv_tok0 * a.H_kv * kHeadDim;
    const __bf16* const Vs = a.V + kv_tok0 * a.H_kv * kHeadDim;
    __bf16* const Os = a.O + q_tok0 * a.H_q * kHeadDim;
    const int kh = head / (a.H_q / a.H_kv);
    const int q0 = qt * TQ + wave * T::R;
    const int shift = S_kv - S_q;

    // keys this block can see at all: the causal bound of its last query row
    int kv_end = S_kv;
    if (a.causal) {
        const int last = qt * TQ + TQ + shift;  // exclusive
        kv_end = last < kv_end ? last : kv_end;
    }
    const int n_tiles = (kv_end + TKV - 1) / TKV;

    // ---- Q fragments: column operand of S^T = K Q^T; lane = (query l32, k-chunk h) ---------------------------
    abf16x8 qf[T::RB][8];
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb) {
        const int q = q0 + rb * 32 + l32;
        const __bf16* src = Qs + (static_cast<int64_t>(q) * a.H_q + head) * kHeadDim + 8 * h;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            au32x4 v = {0u, 0u, 0u, 0u};
            if (q < S_q) v = *reinterpret_cast<const au32x4*>(src + 16 * s);
            qf[rb][s] = __builtin_bit_cast(abf16x8, v);
        }
    }

    // ---- staging registers for one K tile and one V tile ----------------------------------------------------
    au32x4 kreg[T::KC];
    au32x4 vreg[T::KC];
    // Per-thread element offsets of its K chunks and V units inside a tile are loop-invariant; a tile adds a uniform
    // stride.  Tiles that lie wholly inside S_kv (all but possibly the last) are loaded without per-row predicates.
    const int64_t tile_stride = static_cast<int64_t>(TKV) * a.H_kv * kHeadDim;
    int64_t k_off[T::KC];   // (V has K's layout: the same offsets serve both)
#pragma unroll
    for (int i = 0; i < T::KC; ++i) {
        const int c = tid + i * T::NT;
        k_off[i] = (static_cast<int64_t>(c >> 4) * a.H_kv + kh) * kHeadDim + (c & 15) * 8;
    }
    auto load_k = [&](int t) {
        const int kv0 = t * TKV;
        const __bf16* base = Ks + t * tile_stride;
        if (kv0 + TKV <= S_kv) {
#pragma unroll
            for (int i = 0; i < T::KC; ++i)
                if (tid + i * T::NT < T::K_TOTAL) kreg[i] = *reinterpret_cast<const au32x4*>(base + k_off[i]);
            return;
        }
#pragma unroll
        for (int i = 0; i < T::KC; ++i) {
            const int c = tid + i * T::NT;
            au32x4 v = {0u, 0u, 0u, 0u};
            if (c < T::K_TOTAL && kv0 + (c >> 4) < S_kv) v = *reinterpret_cast<const au32x4*>(base + k_off[i]);
            kreg[i] = v;
        }
    };
    auto load_v = [&](int t) {
        const int kv0 = t * TKV;
        const __bf16* base = Vs + t * tile_stride;
        if (kv0 + TKV <= S_kv) {
#pragma unroll
            for (int i = 0; i < T::KC; ++i)
                if (tid + i * T::NT < T::K_TOTAL) vreg[i] = *reinterpret_cast<const au32x4*>(base + k_off[i]);
            return;
        }
#pragma unroll
        for (int i = 0; i < T::KC; ++i) {
            const int c = tid + i * T::NT;
            au32x4 v = {0u, 0u, 0u, 0u};
            if (c < T::K_TOTAL && kv0 + (c >> 4) < S_kv) v = *reinterpret_cast<const au32x4*>(base + k_off[i]);
            vreg[i] = v;
        }
    };
    auto store_k = [&]() {
        char* const base = k_lds;
#pragma unroll
        for (int i = 0; i < T::KC; ++i) {
            const int c = tid + i * T::NT;
            if (c < T::K_TOTAL) *reinterpret_cast<au32x4*>(base + (c >> 4) * T::K_ROW + (c & 15) * 16) = kreg[i];
        }
    };
    auto store_v = [&]() {
        char* const base = v_lds;
#pragma unroll
        for (int i = 0; i < T::KC; ++i) {
            const int c = tid + i * T::NT;
            if (c < T::K_TOTAL) *reinterpret_cast<au32x4*>(base + (c >> 4) * T::V_ROW + (c & 15) * 16) = vreg[i];
        }
    };

    // ---- online softmax state: one query column per lane (lanes l and l^32 hold the same query) -------------
    // m_run is kept in raw score units (scale > 0, so the maximum commutes with the scaling)
    af32x16 o[T::RB][4];
    float m_run[T::RB], l_run[T::RB];
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.0f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[rb][db][e] = 0.0f;
    }

    struct Scores {
        af32x16 v[T::KB][T::RB];
    };
    // S^T[key][query] of the tile in LDS
    auto qk = [&](Scores& s) {
        const char* const base = k_lds;
#pragma unroll
        for (int b = 0; b < T::KB; ++b) {
#pragma unroll
            for (int rb = 0; rb < T::RB; ++rb)
#pragma unroll
                for (int e = 0; e < 16; ++e) s.v[b][rb][e] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const abf16x8 kf = *reinterpret_cast<const abf16x8*>(base + (32 * b + l32) * T::K_ROW + (2 * ks + h) * 16);
#pragma unroll
                for (int rb = 0; rb < T::RB; ++rb)
                    s.v[b][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][ks], s.v[b][rb], 0, 0, 0);
            }
        }
    };
    // online softmax in base 2 over the tile starting at key kv0: s becomes the unnormalised probabilities
    auto softmax = [&](Scores& s, int kv0) {
#pragma unroll
        for (int rb = 0; rb < T::RB; ++rb) {
            const int q = q0 + rb * 32 + l32;
            // wave-uniform: can any element of this tile be masked for these 32 queries?
            const bool ragged = kv0 + TKV > S_kv;
            const bool diag = a.causal && (kv0 + TKV - 1 > q0 + rb * 32 + shift);
            if (ragged || diag) {
                int limit = S_kv - 1;  // last visible key of this lane's query
                if (a.causal && q + shift < limit) limit = q + shift;
#pragma unroll
                for (int b = 0; b < T::KB; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int kv = kv0 + 32 * b + 8 * (e >> 2) + 4 * h + (e & 3);
                        if (kv > limit) s.v[b][rb][e] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int b = 0; b < T::KB; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s.v[b][rb][e]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[rb], mx);
            const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;  // a row that has seen no key yet
            const float alpha = __builtin_amdgcn_exp2f((m_run[rb] - m_use) * a.scale_log2);
            const float neg = -m_use * a.scale_log2;
            float rowsum = 0.0f;
#pragma unroll
            for (int b = 0; b < T::KB; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s.v[b][rb][e], a.scale_log2, neg));
                    s.v[b][rb][e] = p;
                    rowsum += p;
                }
            l_run[rb] = l_run[rb] * alpha + rowsum;
            m_run[rb] = m_new;
            // the running maximum moves in the first few tiles only: skip the rescale when no lane needs it
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[rb][db][e] *= alpha;
            }
        }
    };
    // O^T[d][query] += V^T[d][key] P^T[key][query].  The k slots of a k-step hold, for the lanes of k-half h, the keys
    // 32b + 16ks + 4h + {0..3} and the same + 8 (the order in which the score accumulators come out), so the V^T
    // operand is two transposing reads: lane (s = lane % 16, group = lane / 16) supplies the piece at key
    // 32b + 16ks + 4h + s/4 (+ 8), dims 32db + 16*(group % 2) + 4*(s % 4), and receives dim 32db + lane % 32.
    auto pv = [&](const Scores& s) {
        const int sl = lane & 15;
        const char* const base = v_lds + (4 * h + (sl >> 2)) * T::V_ROW + (16 * ((lane >> 4) & 1) + 4 * (sl & 3)) * 2;
        typedef __attribute__((address_space(3))) as16x4 lds_s16x4;
#pragma unroll
        for (int b = 0; b < T::KB; ++b)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                abf16x8 pf[T::RB];
#pragma unroll
                for (int rb = 0; rb < T::RB; ++rb)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pf[rb][e] = static_cast<__bf16>(s.v[b][rb][8 * ks + e]);
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const char* p = base + (32 * b + 16 * ks) * T::V_ROW + 64 * db;
                    const as16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
                    const as16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * T::V_ROW));
                    typedef __attribute__((ext_vector_type(8))) short as16x8;
                    const as16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    const abf16x8 vf = __builtin_bit_cast(abf16x8, both);
#pragma unroll
                    for (int rb = 0; rb < T::RB; ++rb)
                        o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[rb], o[rb][db], 0, 0, 0);
                }
            }
    };

    if (n_tiles > 0) { load_k(0); load_v(0); }
    for (int t = 0; t < n_tiles; ++t) {
        store_k();
        store_v();
        __syncthreads();
        if (t + 1 < n_tiles) { load_k(t + 1); load_v(t + 1); }
        Scores s;
        qk(s);
        softmax(s, t * TKV);
        pv(s);
        __syncthreads();  // every wavefront is done with this tile's LDS
    }

    // ---- normalise and store: lane holds query q, dims 32db + 8jj + 4h + r --------------------------------
#pragma unroll
    for (int rb = 0; rb < T::RB; ++rb) {
        const int q = q0 + rb * 32 + l32;
        const float lsum = l_run[rb] + __shfl_xor(l_run[rb], 32);
        const float inv = lsum > 0.0f ? 1.0f / lsum : 0.0f;
        if (q >= S_q) continue;
        __bf16* dst = Os + (static_cast<int64_t>(q) * a.H_q + head) * kHeadDim + 4 * h;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                abf16x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = static_cast<__bf16>(o[rb][db][4 * jj + r] * inv);
                *reinterpret_cast<abf16x4*>(dst + 32 * db + 8 * jj) = v;
            }
    }
}

}  // namespace wt
