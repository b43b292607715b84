// Block selection for block-sparse attention on gfx950:
//   pool_kernel    mean-pooled block representations of Q and K (pooling
//                  equation, phi = mean);
//   select_block   block-level scores (block-level attention equation, in its
//                  rank-equivalent raw dot-product form) and the top-n key
//                  blocks of every query block (Selection paragraph);
//   pool_select_kernel  both in one launch: the pooling of one part of the
//                  batch beside the ranking of the part pooled just before.
// The scores of a query block live in LDS between the two phases of
// select_block and nowhere else: nothing of the m x m score matrix reaches HBM.
//
// The arithmetic is pinned so that the emitted indices are reproducible bit
// for bit by a scalar loop: pooled sums are fp32 adds in in-tile row-major
// order followed by one multiply by 1/b; a score is the fp32 chain
// acc = fma(qbar[d], kbar[d], acc) for d ascending from +0; candidates are
// ranked by (score descending, block index ascending) and the query block
// itself is never a candidate.  MFMA is deliberately not used here: its
// internal accumulation order cannot be reproduced by such a loop.
#include "bsa_device.h"
#include "bsa_launch.h"

namespace bsa {

// ---------------------------------------------------------------------------
// pooling
// ---------------------------------------------------------------------------
// A work item is (tile, group of VEC channels); it walks the tile's tokens in
// in-tile row-major order, which is the pinned summation order.  The items of
// one (tensor, batch*head) are numbered tile-major and dealt to workgroups of
// 256 in order: consecutive lanes take consecutive channel groups, so every
// load covers whole 128-byte lines and the tiles of a tile row (bw*D elements
// each, contiguous in memory) are consumed side by side.
// `vblock` numbers the workgroups of one pooling pass: (slice, chunk of 256
// items), the n_q query slices from q_first on, then the n_k key slices from
// k_first on (fewer under grouped query attention).
template <typename T, int VEC>
__device__ __forceinline__ void pool_block(const T* __restrict__ q, const T* __restrict__ k,
                                           float* __restrict__ qbar, float* __restrict__ kbar,
                                           float* __restrict__ kbar_il,
                                           const Geom& g, int D, int64_t q_first, int64_t n_q,
                                           int64_t k_first, int wgs_per_slice, uint32_t vblock)
{
    const int chunk = (int)(vblock % (uint32_t)wgs_per_slice);
    int64_t bh_idx = vblock / (uint32_t)wgs_per_slice;
    const bool is_k = bh_idx >= n_q;
    bh_idx = is_k ? bh_idx - n_q + k_first : bh_idx + q_first;
    const T* __restrict__ x = is_k ? k : q;
    float* __restrict__ xbar = is_k ? kbar : qbar;
    const int groups = D / VEC;
    const int items = g.n_blocks * groups;
    const float inv_b = 1.0f / (float)g.block_tokens;
    x += bh_idx * g.n_tokens * D;

    const int item = chunk * 256 + (int)threadIdx.x;
    if (item >= items) return;
    const int beta = item / groups;
    const int ch = (item - beta * groups) * VEC;
    const int tile_row = beta / g.blocks_per_row, tile_col = beta - tile_row * g.blocks_per_row;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
    for (int rr = 0; rr < g.block_h; ++rr) {
        const T* row = x + ((int64_t)(tile_row * g.block_h + rr) * g.grid_w +
                            (int64_t)tile_col * g.block_w) * D + ch;
#pragma unroll 8
        for (int cc = 0; cc < g.block_w; ++cc) {
#pragma unroll
            for (int e4 = 0; e4 < VEC; e4 += 4) {
                // streamed: every byte is used once here, nothing is worth caching
                const float4 v = load4_stream(row + (int64_t)cc * D + e4);
                acc[e4 + 0] = acc[e4 + 0] + v.x;
                acc[e4 + 1] = acc[e4 + 1] + v.y;
                acc[e4 + 2] = acc[e4 + 2] + v.z;
                acc[e4 + 3] = acc[e4 + 3] + v.w;
            }
        }
    }
    float* dst = xbar + (bh_idx * g.n_blocks + beta) * D + ch;
#pragma unroll
    for (int e4 = 0; e4 < VEC; e4 += 4)
        store4(dst + e4, make_float4(acc[e4] * inv_b, acc[e4 + 1] * inv_b,
                                     acc[e4 + 2] * inv_b, acc[e4 + 3] * inv_b));
    // second copy of the pooled keys for the ranking, per slice [D/4][m][4]: a
    // wavefront whose lanes hold 64 consecutive key blocks then reads 1 KiB runs
    if (is_k && kbar_il) {
        float* il = kbar_il + bh_idx * g.n_blocks * D;
#pragma unroll
        for (int e4 = 0; e4 < VEC; e4 += 4)
            store4(il + ((int64_t)((ch + e4) >> 2) * g.n_blocks + beta) * 4,
                   make_float4(acc[e4] * inv_b, acc[e4 + 1] * inv_b, acc[e4 + 2] * inv_b,
                               acc[e4 + 3] * inv_b));
    }
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void pool_kernel(const T* __restrict__ q,
                                                   const T* __restrict__ k,
                                                   float* __restrict__ qbar,
                                                   float* __restrict__ kbar, Geom g, int D,
                                                   int64_t BH, int wgs_per_slice)
{
    pool_block<T, VEC>(q, k, qbar, kbar, nullptr, g, D, 0, BH, 0, wgs_per_slice, blockIdx.x);
}

// ---------------------------------------------------------------------------
// scores + top-n
// ---------------------------------------------------------------------------
// Order-preserving map fp32 -> u32 (larger float <=> larger integer).  Every
// non-NaN input maps to a value >= 0x007fffff; the clamp keeps even a NaN bit
// pattern away from 0, which marks "removed".
__device__ __forceinline__ uint32_t rank_key(float s)
{
    const uint32_t u = __float_as_uint(s + 0.0f);    // -0 -> +0
    return max((u & 0x80000000u) ? ~u : (u | 0x80000000u), 1u);
}

// Wave-wide reductions over all 64 lanes (all lanes must be active); the
// result is wave-uniform.  Four DPP butterfly steps inside each row of 16
// lanes, then two row broadcasts (lane 15 of a row into the next row, lane 31
// into rows 2 and 3; lanes of the other rows are not written) leave the result
// in lane 63.  Written as one instruction per step: the compiler emits three
// for a row broadcast.  A DPP operand must not be read in the two issue slots
// after it was written, hence the s_nop between the steps.
#define BSA_WAVE_REDUCE(OP, V)                                                              \
    asm volatile("s_nop 1\n\t"                                                             \
                 OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t" \
                 OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t" \
                 OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"      \
                 OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"           \
                 OP " %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t"         \
                 OP " %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\ts_nop 1"              \
                 : "+v"(V))

__device__ __forceinline__ uint32_t wave_umax(uint32_t v)
{
    BSA_WAVE_REDUCE("v_max_u32_dpp", v);
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ uint32_t wave_umin(uint32_t v)
{
    BSA_WAVE_REDUCE("v_min_u32_dpp", v);
    return __builtin_amdgcn_readlane(v, 63);
}

// Descending sort of 8 distinct 64-bit values held in registers (Batcher's
// odd-even merge network, 19 compare-exchanges).
__device__ __forceinline__ void sort8_desc(uint64_t (&a)[9])
{
#define BSA_CE(i, j) { const uint64_t x = a[i], y = a[j]; const bool sw = y > x; \
                       a[i] = sw ? y : x; a[j] = sw ? x : y; }
    BSA_CE(0, 1) BSA_CE(2, 3) BSA_CE(4, 5) BSA_CE(6, 7)
    BSA_CE(0, 2) BSA_CE(1, 3) BSA_CE(4, 6) BSA_CE(5, 7)
    BSA_CE(1, 2) BSA_CE(5, 6)
    BSA_CE(0, 4) BSA_CE(1, 5) BSA_CE(2, 6) BSA_CE(3, 7)
    BSA_CE(2, 4) BSA_CE(3, 5)
    BSA_CE(1, 2) BSA_CE(3, 4) BSA_CE(5, 6)
#undef BSA_CE
}

// Candidates a lane keeps in registers in the top-n phase: 8 for m <= 512
// (sorted once), 64 for 512 < m <= 4096 (best of every group of 8 cached).
constexpr int kSlots = 8;
constexpr int kBigSlots = 64;

typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));

// One group of 8 candidate slots of a lane (a vector value, so that it lives in
// registers): remove slot `which` (0..7; 8 = none), then re-derive the group's
// best key and its slot.  Equal keys keep the lower slot, i.e. the smaller block
// index.
__device__ __forceinline__ void regroup(u32x8& grp, uint32_t& gbest, uint32_t& gslot,
                                        uint32_t which)
{
#pragma unroll
    for (int u = 0; u < 8; ++u) grp[u] = which == (uint32_t)u ? 0u : grp[u];
    uint32_t b = grp[0], sl = 0;
#pragma unroll
    for (int u = 1; u < 8; ++u)
        if (grp[u] > b) { b = grp[u]; sl = (uint32_t)u; }
    gbest = b;
    gslot = sl;
}

// Top-n of one row of m <= 4096 ranking keys (in LDS) by one wavefront.  Lane l
// keeps the candidates j == l (mod 64) in registers, slot j / 64, with the best
// of every group of 8 slots cached; per round: wave-wide max of the lanes' best
// keys, the winner is the lane holding it (smallest block index among equal
// keys), and only the winner's group of 8 is rescanned.
__device__ __forceinline__ void topn_of_row_in_registers(const uint32_t* keys,
                                                         int32_t* __restrict__ dst, int m, int n,
                                                         int lane)
{
    u32x8 g0, g1, g2, g3, g4, g5, g6, g7;
    uint32_t gbest[8], gslot[8];
#define BSA_LOAD_GROUP(GI, GRP)                                                                 \
    _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                              \
        const int j = lane + 64 * (GI * 8 + u);                                                  \
        GRP[u] = j < m ? keys[j] : 0u;                                                           \
    }                                                                                            \
    regroup(GRP, gbest[GI], gslot[GI], 8u);
    BSA_LOAD_GROUP(0, g0) BSA_LOAD_GROUP(1, g1) BSA_LOAD_GROUP(2, g2) BSA_LOAD_GROUP(3, g3)
    BSA_LOAD_GROUP(4, g4) BSA_LOAD_GROUP(5, g5) BSA_LOAD_GROUP(6, g6) BSA_LOAD_GROUP(7, g7)
#undef BSA_LOAD_GROUP
    auto lane_best = [&](uint32_t& best, uint32_t& best_j) {
        best = gbest[0]; uint32_t slot = gslot[0];
#pragma unroll
        for (int gi = 1; gi < 8; ++gi)
            if (gbest[gi] > best) { best = gbest[gi]; slot = 8u * gi + gslot[gi]; }
        best_j = best ? (uint32_t)lane + 64u * slot : 0xffffffffu;
    };
    uint32_t best, best_j;
    lane_best(best, best_j);
    uint32_t picks = 0;
    for (int t = 0; t < n; ++t) {
        const uint32_t top = wave_umax(best);
        const uint64_t holders = __builtin_amdgcn_ballot_w64(best == top);
        uint32_t win;
        if (__builtin_expect(__builtin_popcountll(holders) == 1, 1))
            win = __builtin_amdgcn_readlane(best_j, (int)__builtin_ctzll(holders));
        else
            win = wave_umin(best == top ? best_j : 0xffffffffu);
        picks = lane == (t & 63) ? win : picks;          // lane t % 64 keeps pick t
        if ((win & 63u) == (uint32_t)lane) {
            const uint32_t slot = win >> 6, which = slot & 7u;   // wave-uniform values
            switch (slot >> 3) {
            case 0: regroup(g0, gbest[0], gslot[0], which); break;
            case 1: regroup(g1, gbest[1], gslot[1], which); break;
            case 2: regroup(g2, gbest[2], gslot[2], which); break;
            case 3: regroup(g3, gbest[3], gslot[3], which); break;
            case 4: regroup(g4, gbest[4], gslot[4], which); break;
            case 5: regroup(g5, gbest[5], gslot[5], which); break;
            case 6: regroup(g6, gbest[6], gslot[6], which); break;
            default: regroup(g7, gbest[7], gslot[7], which); break;
            }
            lane_best(best, best_j);
        }
        if ((t & 63) == 63 || t == n - 1) {
            if (lane <= (t & 63)) dst[(t & ~63) + lane] = (int32_t)picks;
        }
    }
}

// One workgroup of 256 threads ranks G consecutive query blocks of one
// (batch, head).
//   phase 1: thread t owns key block j = t, t + 256, ..., holds kbar_j in
//            registers (loaded from the channel-interleaved copy of the pooled
//            keys where there is one: consecutive lanes then read consecutive
//            16-byte groups) and runs the pinned fma chain against each of the
//            G pooled queries (wave-uniform: scalar loads, scalar operands); the
//            ranking keys of all m candidates of each query land in LDS.
//   phase 2: one wavefront per query block extracts the n best candidates by
//            repeated arg-max over the lanes' best remaining candidates
//            (j == lane mod 64): a wave-wide max of the scores, then, only if
//            several lanes hold it, a wave-wide min of their block indices.
// LDS: G*m u32 (ranking keys).  BIG: the variant for 512 < m <= 4096, whose
// second phase keeps 64 candidates per lane (a kernel of its own: its register
// count must not cost the common case its occupancy).
template <int D, bool BIG>
__device__ __forceinline__ void select_block(const float* __restrict__ qbar,
                                             const float* __restrict__ kbar,
                                             const float* __restrict__ kbar_il,
                                             int32_t* __restrict__ sel_idx, const Geom& g, int G,
                                             uint32_t vblock)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint32_t* key_s = (uint32_t*)smem;               // [G][m]

    const int m = g.n_blocks, n = g.n_select;
    // vblock = batch*head * groups + group
    const int groups = (m + G - 1) / G;
    const int64_t bh_idx = vblock / (uint32_t)groups;
    const int i0 = (int)(vblock - (uint32_t)bh_idx * (uint32_t)groups) * G;
    const int rows = min(G, m - i0);
    qbar += (bh_idx * m + i0) * D;
    kbar += kv_slice_of(g, bh_idx) * m * D;

    if (kbar_il) kbar_il += kv_slice_of(g, bh_idx) * m * D;   // per slice [D/4][m][4]

    // ---- phase 1: scores.  The pooled queries are wave-uniform and are fetched
    // with scalar loads straight into the fma's scalar operand.
    auto load_key = [&](int j, float (&kr)[D]) {
        // the interleaved copy where there is one, else the key block's row
        const float4* ksrc = kbar_il ? (const float4*)kbar_il + j
                                     : (const float4*)(kbar + (int64_t)j * D);
        const int64_t kstep = kbar_il ? (int64_t)m : 1;
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const float4 v = ksrc[d4 * kstep];
            kr[4 * d4 + 0] = v.x; kr[4 * d4 + 1] = v.y;
            kr[4 * d4 + 2] = v.z; kr[4 * d4 + 3] = v.w;
        }
    };
    auto put_key = [&](int r, int j, float acc) {
        key_s[r * m + j] = (j == i0 + r && !g.own_is_candidate) ? 0u : rank_key(acc);
    };
    int j = threadIdx.x;
    if constexpr (BIG && D <= 64) {
        // Two key blocks per thread at a time: with this many blocks the LDS rows
        // leave one workgroup per CU, i.e. one wavefront per SIMD, and the two
        // independent chains (same scalar operand) hide the latency of one.
        for (; j + (int)blockDim.x < m; j += 2 * (int)blockDim.x) {
            float ka[D], kb[D];
            load_key(j, ka);
            load_key(j + (int)blockDim.x, kb);
            for (int r = 0; r < rows; ++r) {
                const float* __restrict__ qrow = qbar + r * D;
                float a = 0.0f, b = 0.0f;
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    a = __builtin_fmaf(qrow[d], ka[d], a);
                    b = __builtin_fmaf(qrow[d], kb[d], b);
                }
                put_key(r, j, a);
                put_key(r, j + (int)blockDim.x, b);
            }
        }
    }
    for (; j < m; j += blockDim.x) {
        float kr[D];
        load_key(j, kr);
        for (int r = 0; r < rows; ++r) {
            const float* __restrict__ qrow = qbar + r * D;
            float acc = 0.0f;
#pragma unroll
            for (int d = 0; d < D; ++d) acc = __builtin_fmaf(qrow[d], kr[d], acc);
            put_key(r, j, acc);
        }
    }
    __syncthreads();

    // ---- phase 2: top-n per query block, one wavefront each
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < rows; r += (int)(blockDim.x >> 6)) {
        uint32_t* keys = key_s + r * m;
        int32_t* dst = sel_idx + ((bh_idx * m) + i0 + r) * n;
        if constexpr (BIG) {
            topn_of_row_in_registers(keys, dst, m, n, lane);
            continue;
        }
        if (m <= 64 * kSlots) {
            // Candidates j == lane (mod 64) live in registers as composites
            // (key << 32 | ~j), which are all distinct and order the
            // candidates exactly as the ranking does.  Every lane sorts its 8
            // composites (descending) once; per round: wave-wide max of the
            // lanes' head keys, the winner is the lane holding it (the
            // smallest block index among them when several do, which only
            // happens for exactly equal scores), and that lane moves on to its
            // next composite.  Lane t % 64 keeps pick t; 64 picks go out in
            // one store.
            uint64_t srt[kSlots + 1];
#pragma unroll
            for (int t = 0; t < kSlots; ++t) {
                const int j = lane + 64 * t;
                srt[t] = ((uint64_t)(j < m ? keys[j] : 0u) << 32) | (uint32_t)~j;
            }
            srt[kSlots] = 0xffffffffull;                 // key 0: nothing left
            sort8_desc(srt);
            uint32_t best = (uint32_t)(srt[0] >> 32), best_j = ~(uint32_t)srt[0], head = 0;
            uint32_t picks = 0;
            for (int t = 0; t < n; ++t) {
                const uint32_t top = wave_umax(best);
                const uint64_t holders = __builtin_amdgcn_ballot_w64(best == top);
                uint32_t win;
                if (__builtin_expect(__builtin_popcountll(holders) == 1, 1))
                    win = __builtin_amdgcn_readlane(best_j, (int)__builtin_ctzll(holders));
                else
                    win = wave_umin(best == top ? best_j : 0xffffffffu);
                const int win_lane = (int)(win & 63u);
                picks = lane == (t & 63) ? win : picks;
                const uint32_t next = (uint32_t)__builtin_amdgcn_readlane((int)head, win_lane) + 1u;
                if (lane == win_lane) {
                    const uint64_t c = srt[next];        // wave-uniform register index
                    best = (uint32_t)(c >> 32);
                    best_j = ~(uint32_t)c;
                    head = next;
                }
                if ((t & 63) == 63 || t == n - 1) {
                    if (lane <= (t & 63)) dst[(t & ~63) + lane] = (int32_t)picks;
                }
            }
            continue;
        }
        uint32_t best = 0u, best_j = 0xffffffffu;
        for (int j = lane; j < m; j += 64) {
            const uint32_t u = keys[j];
            if (u > best) { best = u; best_j = (uint32_t)j; }
        }
        for (int t = 0; t < n; ++t) {
            const uint32_t top = wave_umax(best);
            const uint32_t win = wave_umin(best == top ? best_j : 0xffffffffu);
            if (lane == 0) dst[t] = (int32_t)win;
            if ((win & 63u) == (uint32_t)lane) {
                keys[win] = 0u;
                best = 0u; best_j = 0xffffffffu;
                for (int j = lane; j < m; j += 64) {
                    const uint32_t u = keys[j];
                    if (u > best) { best = u; best_j = (uint32_t)j; }
                }
            }
        }
    }
}

// Pooling of one part of the batch beside the ranking of the part pooled by
// the launch before: pooling is bound by HBM and leaves the vector ALUs idle,
// the ranking is bound by the vector ALUs and reads only cached pooled means.
// The first n_poolers workgroups of the launch pool: they are dispatched
// first and each walks the part's n_pool_blocks pooling blocks with stride
// n_poolers, so a fixed number of them stays resident on every CU until the
// part is pooled (pooling workgroups dealt one block each are short-lived and
// would be crowded out by the long-lived ranking workgroups).  The other
// workgroups rank (virtual ids from select_first on).  No workgroup waits for
// another: what a ranking workgroup reads was written by an earlier launch.
// The pooled means are passed twice: written through qbar_w / kbar_w / kbar_il_w
// (the part being pooled), read through qbar_r / kbar_r / kbar_il_r (the part
// being ranked).
template <typename T, int VEC, int D, bool BIG>
__global__ __launch_bounds__(256) void pool_select_kernel(
    const T* __restrict__ q, const T* __restrict__ k, float* __restrict__ qbar_w,
    float* __restrict__ kbar_w, float* __restrict__ kbar_il_w, const float* __restrict__ qbar_r,
    const float* __restrict__ kbar_r, const float* __restrict__ kbar_il_r,
    int32_t* __restrict__ sel_idx, Geom g, int G,
    int64_t pool_q_first, int64_t pool_n_q, int64_t pool_k_first, int wgs_per_slice,
    uint32_t n_pool_blocks, uint32_t n_poolers, uint32_t select_first)
{
    if (blockIdx.x >= n_poolers) {
        select_block<D, BIG>(qbar_r, kbar_r, kbar_il_r, sel_idx, g, G,
                        select_first + (blockIdx.x - n_poolers));
        return;
    }
    for (uint32_t v = blockIdx.x; v < n_pool_blocks; v += n_poolers)
        pool_block<T, VEC>(q, k, qbar_w, kbar_w, kbar_il_w, g, D, pool_q_first, pool_n_q, pool_k_first,
                           wgs_per_slice, v);
}

// ---------------------------------------------------------------------------
// Checker for caller-made selections (the attention kernels trust sel_idx):
// one thread per row counts the entries that are out of range, repeat an
// earlier entry of the row or, unless own_ok, name the row's own block.
// ---------------------------------------------------------------------------
__global__ void zero_counter_kernel(int32_t* counter) { *counter = 0; }

__global__ __launch_bounds__(256) void check_selection_kernel(const int32_t* __restrict__ sel_idx,
                                                              int32_t* __restrict__ n_bad, Geom g,
                                                              int own_ok, int64_t rows)
{
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int bad = 0;
    if (row < rows) {
        const int n = g.n_select, m = g.n_blocks;
        const int own = (int)(row % m);
        const int32_t* r = sel_idx + row * n;
        for (int a = 0; a < n; ++a) {
            const int32_t x = r[a];
            bool is_bad = x < 0 || x >= m || (!own_ok && x == own);
            for (int c = 0; c < a && !is_bad; ++c) is_bad = r[c] == x;
            bad += is_bad ? 1 : 0;
        }
    }
    // one integer atomic per wavefront with something to report
    for (int off = 32; off >= 1; off >>= 1) bad += __shfl_xor(bad, off);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(n_bad, bad);
}

hipError_t launch_check_selection(const int32_t* sel_idx, int32_t* n_bad, const Geom& g,
                                  bool own_ok, int64_t BH, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, stream, n_bad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || g.n_select == 0) return e;
    const int64_t rows = BH * g.n_blocks;
    hipLaunchKernelGGL(check_selection_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0,
                       stream, sel_idx, n_bad, g, own_ok ? 1 : 0, rows);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// host-side launchers
// ---------------------------------------------------------------------------
static constexpr size_t kSelectLdsBudget = 144 * 1024;

static size_t select_lds_bytes(int G, int m, int D)
{
    (void)D;
    return (size_t)G * (size_t)m * 4;
}

int select_group_size(int m, int D)
{
    // the largest G in [1, 8] whose LDS footprint fits, and fits twice where
    // that is possible with G >= 4 (two workgroups per CU cover each other's
    // loads, and a pooling workgroup fits beside a ranking one); 0 if even
    // G = 1 does not fit
    for (int G = 8; G >= 4; G >>= 1)
        if (2 * select_lds_bytes(G, m, D) <= kSelectLdsBudget) return G;
    for (int G = 8; G >= 1; G >>= 1)
        if (select_lds_bytes(G, m, D) <= kSelectLdsBudget) return G;
    return 0;
}

template <typename T, int VEC>
static hipError_t launch_pool_t(const void* q, const void* k, float* qbar, float* kbar,
                                const Geom& g, int D, int64_t BH, hipStream_t stream)
{
    const int items = g.n_blocks * (D / VEC);
    const int wgs_per_slice = (items + 255) / 256;
    dim3 grid((unsigned)((BH + BH / g.kv_group) * wgs_per_slice));
    hipLaunchKernelGGL((pool_kernel<T, VEC>), grid, dim3(256), 0, stream, (const T*)q,
                       (const T*)k, qbar, kbar, g, D, BH, wgs_per_slice);
    return hipGetLastError();
}

hipError_t launch_pool(bool is_bf16, const void* q, const void* k, float* qbar, float* kbar,
                       const Geom& g, int D, int64_t BH, hipStream_t stream)
{
    return is_bf16 ? launch_pool_t<uint16_t, 8>(q, k, qbar, kbar, g, D, BH, stream)
                   : launch_pool_t<float, 4>(q, k, qbar, kbar, g, D, BH, stream);
}

hipError_t launch_pool_one(bool is_bf16, const void* x, float* xbar, const Geom& g, int D,
                           int64_t slices, hipStream_t stream)
{
    // the pooling kernel with no query slices: every slice is a "key" slice
    const int items = g.n_blocks * (D / (is_bf16 ? 8 : 4));
    const int wgs_per_slice = (items + 255) / 256;
    dim3 grid((unsigned)(slices * wgs_per_slice));
    if (is_bf16)
        hipLaunchKernelGGL((pool_kernel<uint16_t, 8>), grid, dim3(256), 0, stream,
                           (const uint16_t*)nullptr, (const uint16_t*)x, (float*)nullptr, xbar, g,
                           D, (int64_t)0, wgs_per_slice);
    else
        hipLaunchKernelGGL((pool_kernel<float, 4>), grid, dim3(256), 0, stream,
                           (const float*)nullptr, (const float*)x, (float*)nullptr, xbar, g, D,
                           (int64_t)0, wgs_per_slice);
    return hipGetLastError();
}

size_t select_scratch_bytes(int m, int D, int64_t BH, int64_t BKV)
{
    (void)BH;
    // the ranking reads a second, channel-interleaved copy of the pooled keys
    return (size_t)BKV * (size_t)m * (size_t)D * 4;
}

#ifndef BSA_SELECT_PARTS
#define BSA_SELECT_PARTS 4
#endif
#ifndef BSA_POOLERS
#define BSA_POOLERS 256
#endif
// pooling workgroups that stay resident beside the ranking (one per CU)
constexpr int64_t kPoolers = BSA_POOLERS;

bool select_interleaves_keys(int m) { (void)m; return true; }

template <typename T, int VEC, int D, bool BIG>
static hipError_t launch_pool_select_t(const void* q, const void* k, float* qbar, float* kbar,
                                       float* kbar_il, int32_t* sel_idx, const Geom& g,
                                       int64_t BH, hipStream_t stream)
{
    const int m = g.n_blocks;
    const int G = select_group_size(m, D);
    if (G == 0) return hipErrorInvalidValue;
    const size_t lds = select_lds_bytes(G, m, D);
    // the attribute is per device; setting it twice (two host threads racing) is harmless
    static bool attr_set[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute((const void*)pool_select_kernel<T, VEC, D, BIG>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kSelectLdsBudget);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    const int64_t BKV = BH / g.kv_group;
    const int parts = (int)(BKV < BSA_SELECT_PARTS ? BKV : BSA_SELECT_PARTS);
    const int wgs_per_slice = (m * (D / VEC) + 255) / 256;
    const int groups = (m + G - 1) / G;
    // launch t pools part t and ranks part t - 1
    for (int t = 0; t <= parts; ++t) {
        int64_t pq0 = 0, pnq = 0, pk0 = 0, n_pool = 0, sel_first = 0, n_sel = 0;
        if (t < parts) {
            pk0 = BKV * t / parts;
            const int64_t pk1 = BKV * (t + 1) / parts;
            pq0 = pk0 * g.kv_group;
            pnq = (pk1 - pk0) * g.kv_group;
            n_pool = (pnq + (pk1 - pk0)) * wgs_per_slice;
        }
        if (t >= 1) {
            const int64_t k0 = BKV * (t - 1) / parts, k1 = BKV * t / parts;
            sel_first = k0 * g.kv_group * groups;
            n_sel = (k1 - k0) * g.kv_group * groups;
        }
        if (n_pool + n_sel == 0) continue;
        // alone, the pooling blocks get a workgroup each
        const int64_t n_poolers = n_sel == 0 ? n_pool : (n_pool < kPoolers ? n_pool : kPoolers);
        if (n_pool >= ((int64_t)1 << 31) || n_poolers + n_sel >= ((int64_t)1 << 31) ||
            sel_first + n_sel >= ((int64_t)1 << 32))
            return hipErrorInvalidValue;
        hipLaunchKernelGGL((pool_select_kernel<T, VEC, D, BIG>), dim3((unsigned)(n_poolers + n_sel)),
                           dim3(256), lds, stream, (const T*)q, (const T*)k, qbar, kbar, kbar_il,
                           (const float*)qbar, (const float*)kbar, (const float*)kbar_il, sel_idx,
                           g, G, pq0, pnq, pk0,
                           wgs_per_slice, (uint32_t)n_pool, (uint32_t)n_poolers,
                           (uint32_t)sel_first);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_pool_select(bool is_bf16, const void* q, const void* k, float* qbar,
                              float* kbar, void* scratch, int32_t* sel_idx, const Geom& g, int D,
                              int64_t BH, hipStream_t stream)
{
    // the channel-interleaved copy of the pooled keys
    const int m = g.n_blocks;
    float* il = (float*)scratch;
    if (!il) return hipErrorInvalidValue;
    const bool big = m > 64 * kSlots && m <= 64 * kBigSlots;
#define BSA_PS(T, VEC, D_)                                                                        \
    (big ? launch_pool_select_t<T, VEC, D_, true>(q, k, qbar, kbar, il, sel_idx, g, BH, stream)   \
         : launch_pool_select_t<T, VEC, D_, false>(q, k, qbar, kbar, il, sel_idx, g, BH, stream))
    switch (D) {
    case 32: return is_bf16 ? BSA_PS(uint16_t, 8, 32) : BSA_PS(float, 4, 32);
    case 64: return is_bf16 ? BSA_PS(uint16_t, 8, 64) : BSA_PS(float, 4, 64);
    case 128: return is_bf16 ? BSA_PS(uint16_t, 8, 128) : BSA_PS(float, 4, 128);
    }
#undef BSA_PS
    return hipErrorInvalidValue;
}

}  // namespace bsa
