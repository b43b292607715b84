// Block-sparse attention forward on the gfx950 matrix cores (bf16 MFMA, fp32
// online softmax).  Specialised for head dim 64 and tiles of 64*T tokens whose
// width is a power of two; a tile is processed as T sub-blocks of 64 queries (one
// wavefront each) against T sub-tiles of 64 keys per attended block.
//
// Every token of query block i attends, in one softmax, to the tokens of block
// i and of its n selected blocks (fine-grained attention equation plus the
// local block).  Per (query block, key/value block) pair the work is two dense
// 64x64x64 contractions, S = Q K^T and O += P V, which is what the matrix cores
// are for.
//
// One wavefront owns one query block (64 rows) for its whole life:
//   * transposed products are computed, S^T = K Q^T and O^T = V^T P^T, with
//     v_mfma_f32_32x32x16_bf16.  In the accumulator layout of that instruction
//     a lane then holds ONE query (column) and 16 keys (rows) per 32x32 tile, so
//     the softmax row reductions are in-register plus a single exchange between
//     lane l and lane l+32;
//   * the accumulator layout of S^T is, register for register, the B-operand
//     layout that O^T = V^T P^T needs (keys are the contraction index), so P
//     never leaves registers: exp2, convert to bf16, feed the next MFMA;
//   * K and V tiles are gathered from HBM/L2 straight into LDS (global_load_lds,
//     16 bytes per lane, one 1 KiB run of contiguous tokens per instruction --
//     a tile of the lat-lon grid is bh runs of bw contiguous tokens) and each
//     byte is read from LDS exactly once: K rows as 16-byte A-operand fragments,
//     V through the transposing LDS read (ds_read_b64_tr_b16) that turns the
//     token-major tile into key-contiguous A-operand fragments of V^T;
//   * LDS rows are XOR-swizzled at 16-byte granularity; the swizzle is applied
//     on the global side of the direct-to-LDS load (which lane fetches which
//     chunk), because that load always writes lanes to consecutive LDS
//     addresses.
//
// Schedule.  On this hardware a wavefront that streams MFMAs keeps the other
// wavefronts of its SIMD from issuing vector-ALU work, but the SAME wavefront
// can issue about 24 cycles of vector-ALU instructions behind each 32-cycle
// MFMA for free.  The exponentials therefore have to sit between the MFMAs of
// the wavefront that owns them.  The pair is cut into four tiles of 32 keys x
// 32 queries, t = (key half mt, query half nt), and the three stages of a
// tile -- S tile (4 MFMAs), weights (48 vector instructions), O update
// (4 MFMAs) -- are software-pipelined across tiles, also across pair
// boundaries: step s issues, alternating, the 4 MFMAs of S(s+1) and the 4 MFMAs
// of the O update with P(s-1), and behind each of these 8 MFMAs one eighth of
// the weights of tile s (2 fma, 2 exp2, 1 rounding pack, 2 adds for the row sum).
// Only two S tiles and two P tiles are live, so the wavefront fits 256
// registers and two wavefronts share a SIMD to cover each other's waits.
//
// K and V live in LDS as two 32-key halves each (four 4 KiB buffers).  A half
// is read into registers once per pair, at a fixed step, and refilled right
// after with the same half of the next tile, which then has three steps (3/4
// of a pair) to arrive.  The 8 loads of a refill are spread over the 8 MFMA
// slots of a step: a burst would hold the wavefront at the CU's shared address
// unit.  Workgroups of 2 or 4 wavefronts (blocks of 128 or 256 tokens, whose
// sub-blocks share the tiles) have the LDS for two tiles: consecutive pairs
// alternate between two sets of buffers and a half is refilled with the tile
// after the next, which has seven steps to arrive.
//
// Softmax without a row maximum per tile.  m_ref is the reference the
// exponentials are taken against.  A tile first computes its weights against
// the current m_ref; only if some row sum of the tile exceeds 2^12 (which
// covers the first tile of each query half, where m_ref = -inf) does the
// wavefront take the slow path: find the row maxima, move m_ref, rescale O and
// the normaliser, and recompute the tile's weights.  Any reference gives the
// same softmax; bounded weights keep fp32 and bf16 far from overflow.
#include "bsa_device.h"
#include "bsa_launch.h"
#include "bsa_mfma_common.h"

namespace bsa {

// 16-byte chunk swizzle of a 128-byte LDS row (8 chunks per row).  The K
// fragment read takes the same chunk of 8 consecutive rows per 128 bytes of
// bank width, the transposing V read 32 bytes (a chunk pair) of 4 consecutive
// rows: the row's XOR mask is a bijection of row % 8 whose upper two bits
// differ over any 4 aligned rows.
__device__ __forceinline__ int swz(int row, int chunk)
{
    return chunk ^ (((row & 3) << 1) | ((row >> 2) & 1));
}

// Gather of a 64-token x 64-channel bf16 tile into LDS (two 4 KiB halves, rows
// swizzled) with buffer loads that write LDS directly.  A tile takes 8 such
// instructions; instruction r ("slab" r) brings tile rows 8r..8r+7 and lane l
// fills LDS chunk l of that 1 KiB slab, i.e. row 8r + l/8, swizzled chunk l%8.
// The wavefronts of a workgroup split the slabs: wavefront w issues slabs
// NW j + w, j = 0 .. 8/NW - 1, the first half of them into the lower half tile.
// The per-lane byte offsets of a wavefront's slabs inside a block (voff[j]) are
// fixed for the whole kernel, the block origin is wave-uniform (soffset) and so
// is the LDS address (half tile + ((NW j + w) % 4) KiB), so a gather costs no
// vector ALU work and no branch.  The buffer descriptor bounds the slice: an
// out-of-range block index reads zeros instead of faulting, and a descriptor
// of zero records makes the load a no-op.
template <int NW, int J>
__device__ __forceinline__ void gather_slab(__amdgpu_buffer_rsrc_t rsrc, uint32_t origin_bytes,
                                            const uint32_t (&voff)[8 / NW], unsigned char* lds_half,
                                            uint32_t wave_kib)
{
    // J-th slab of this wavefront: slab NW * J + wave of the tile
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        rsrc, LDS_PTR(void, lds_half + ((NW * J) & 3) * 1024 + wave_kib), 16, voff[J],
        origin_bytes, 0, 0);
}

// The two half tiles that a step refills, spread over its 8 MFMA slots: a
// lower half (tile rows 0..31, slabs 0..3) goes to lds_a from (rsrc_a,
// origin_a), an upper half (rows 32..63, slabs 4..7) to lds_b.
struct Refill {
    __amdgpu_buffer_rsrc_t rsrc_a, rsrc_b;
    uint32_t origin_a, origin_b;
    __attribute__((address_space(3))) unsigned char *lds_a, *lds_b;
};

// One step of the software pipeline, J = position of the tile inside its pair:
// tile J = (key half J/2, query half J%2).  Issues, alternating, the 4 MFMAs of
// the S tile J+1 and the 4 MFMAs that add tile J-1 to O, and behind each the
// vector work of one eighth of the weights of tile J, skewed by one slot
// (fma for slot k+1, exp2 for slot k, rounding pack + row sum for slot k-1) so
// that no instruction waits for the one before it.  With REFILL, every NW-th
// slot also issues one of this wavefront's slabs of a K/V refill.  S tiles and P tiles are indexed by query
// half: the tile being weighted and its neighbours in the pipeline always
// differ in it.  Returns this lane's sum of the tile's fp32 weights.
template <int J, bool REFILL, int NW, class Mid>
__device__ __forceinline__ float pipeline_step(f32x16 (&s)[2], bf16x8 (&p)[2][2],
                                               f32x16 (&oacc)[2][2], const bf16x8 (&qf)[2][4],
                                               const bf16x8 (&kf)[2][4],
                                               const bf16x8 (&vf)[2][4], float c2, float neg_m,
                                               const Refill& rf, const uint32_t (&voff)[8 / NW],
                                               uint32_t wave_kib, Mid mid)
{
    constexpr int nt = J & 1;
    constexpr int mt_n = ((J + 1) & 3) >> 1, nt_n = (J + 1) & 1;   // next tile: S
    constexpr int mt_p = ((J + 3) & 3) >> 1, nt_p = (J + 3) & 1;   // previous tile: O update
    static_assert(nt_n != nt && nt_p != nt, "pipeline neighbours use the other buffers");
    const f32x16 zero16 = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f,
                           0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    uint32_t w[8];
    float rs0, rs1;
    float f[8][2], e[8][2];
    f[0][0] = fmaf(s[nt][0], c2, neg_m);
    f[0][1] = fmaf(s[nt][1], c2, neg_m);
    asm volatile("" : "+v"(f[0][0]), "+v"(f[0][1]));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int i = k >> 1;
        if (k == 4) {
            mid();     // LDS reads of a step go here: their results are two steps away
            __builtin_amdgcn_sched_barrier(0);
        }
        if ((k & 1) == 0) {
            s[nt_n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt_n][i], qf[nt_n][i],
                                                              i == 0 ? zero16 : s[nt_n], 0, 0, 0);
        } else {
            const int dt = i & 1, h = i >> 1;
            oacc[dt][nt_p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                vf[dt][2 * mt_p + h], p[nt_p][h], oacc[dt][nt_p], 0, 0, 0);
        }
        if (REFILL && k % NW == 0) {
            // (the wavefronts of a workgroup share the refill: every NW-th slot
            // issues this wavefront's next slab, slab k + wave of the tile)
            if (k < 4)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rf.rsrc_a,
                    (__attribute__((address_space(3))) void*)(rf.lds_a + k * 1024 + wave_kib), 16,
                    voff[k / NW], rf.origin_a, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rf.rsrc_b,
                    (__attribute__((address_space(3))) void*)(rf.lds_b + (k - 4) * 1024 + wave_kib),
                    16, voff[k / NW], rf.origin_b, 0, 0);
        }
        // exp2 of this slot's pair, fma of the next slot's, pack and row sums
        // of the previous slot's: nothing waits for the instruction before it.
        // The empty asm statements "use" the slot's results: they keep their
        // producers in this slot (they would otherwise sink to the first real
        // use, after the last MFMA); no instruction is emitted for them.
        e[k][0] = __builtin_amdgcn_exp2f(f[k][0]);
        e[k][1] = __builtin_amdgcn_exp2f(f[k][1]);
        if (k + 1 < 8) {
            f[k + 1][0] = fmaf(s[nt][2 * k + 2], c2, neg_m);
            f[k + 1][1] = fmaf(s[nt][2 * k + 3], c2, neg_m);
        }
        if (k >= 1) w[k - 1] = pack_bf16(e[k - 1][0], e[k - 1][1]);
        if (k == 2) {
            rs0 = e[0][0] + e[1][0];
            rs1 = e[0][1] + e[1][1];
        } else if (k > 2) {
            rs0 += e[k - 1][0];
            rs1 += e[k - 1][1];
        }
        if (k == 0)
            asm volatile("" : "+v"(e[0][0]), "+v"(e[0][1]), "+v"(f[1][0]), "+v"(f[1][1]));
        else if (k == 1)
            asm volatile(""
                         : "+v"(e[1][0]), "+v"(e[1][1]), "+v"(f[2][0]), "+v"(f[2][1]),
                           "+v"(w[0]));
        else if (k < 7)
            asm volatile(""
                         : "+v"(e[k][0]), "+v"(e[k][1]), "+v"(f[k < 7 ? k + 1 : 7][0]),
                           "+v"(f[k < 7 ? k + 1 : 7][1]), "+v"(w[k >= 1 ? k - 1 : 0]), "+v"(rs0),
                           "+v"(rs1));
        else
            asm volatile(""
                         : "+v"(e[7][0]), "+v"(e[7][1]), "+v"(w[6]), "+v"(rs0), "+v"(rs1));
        __builtin_amdgcn_sched_barrier(0);
    }
    w[7] = pack_bf16(e[7][0], e[7][1]);
    rs0 += e[7][0];
    rs1 += e[7][1];
    p[nt][0] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    p[nt][1] = __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7]));
    return rs0 + rs1;
}

// compile-time index of an LDS set
template <int S> struct SetTag { static constexpr int value = S; };

// The kernel body for workgroups of NW wavefronts.  NW consecutive 64-query
// sub-blocks of one query block attend to the same K/V tiles, so with NW > 1
// the tiles in LDS are shared: the loads of a refill are split between the
// wavefronts and each group of half tiles takes two workgroup barriers per
// pair, "all reads done" before its refill is issued and "all loads landed"
// (each wavefront waits for its own loads first) before it is read again.
template <int NW, int DEPTH>
__device__ __forceinline__ void fwd_mfma_d64_body(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const int32_t* __restrict__ sel_idx,
    uint16_t* __restrict__ out, float* __restrict__ lse, const Geom& g, uint32_t n_units,
    int subs)
{
    constexpr int D = 64;
    static_assert(NW == 1 || NW == 2 || NW == 4, "8 loads per refill step, split between waves");
    auto wg_barrier = [] { if (NW > 1) __builtin_amdgcn_s_barrier(); };
    static_assert(DEPTH == 1 || (DEPTH == 2 && NW > 1), "one K/V tile in LDS, or two (even pair counts only)");
    // every load older than this wavefront's share (8 / NW each) of the most
    // recent 2 * DEPTH - 1 refill steps has landed
    auto wait_older_loads = [] {
        if (NW == 1 && DEPTH == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (NW == 2 && DEPTH == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        if (NW == 4 && DEPTH == 1) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        if (NW == 1 && DEPTH == 2) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
        if (NW == 2 && DEPTH == 2) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
        if (NW == 4 && DEPTH == 2) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    };
    // K and V tiles as two 32-key halves each, DEPTH sets of them (pair c lives
    // in set c % DEPTH).  Halves that are read at the same point of the
    // pipeline and refilled in the same step share an object; reads of one
    // object are not ordered behind gathers into another (the compiler tracks
    // a limited number of them, beyond which it waits for every load):
    //   x_*: V half 0 and K half 1 of a set (read in step 3 of the pair before,
    //        refilled in step 0);
    //   y_*: V half 1 of a set and K half 0 of the other set (DEPTH 1: of the
    //        same set), read in step 1 and refilled in step 2.
    __shared__ __attribute__((aligned(1024))) unsigned char x_a[2][32 * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char y_a[2][32 * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char x_b[DEPTH == 2 ? 2 : 1][DEPTH == 2 ? 32 * 128 : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char y_b[DEPTH == 2 ? 2 : 1][DEPTH == 2 ? 32 * 128 : 16];
    unsigned char* const v_lds0_a = x_a[0];
    unsigned char* const k_lds1_a = x_a[1];
    unsigned char* const v_lds0_b = x_b[0];
    unsigned char* const k_lds1_b = x_b[DEPTH - 1];
    // y_a: V half 1 of set a with K half 0 of set b (DEPTH 1: of set a)
    unsigned char* const v_lds1_a = y_a[0];
    unsigned char* const k_lds0_b = y_a[1];
    unsigned char* const v_lds1_b = y_b[0];
    unsigned char* const k_lds0_a = DEPTH == 2 ? y_b[DEPTH - 1] : y_a[1];
    __shared__ int order_s[NW][64];

    const int lane = threadIdx.x & 63;
    const int wave = NW == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;

    // Work item -> (query slice, query block); key/value slices are dealt to
    // the XCDs whole (map_workgroup).  A work item is NW consecutive
    // sub-blocks of 64 queries of one query block (NW divides subs):
    // item = block * (subs / NW) + group.
    int i, qsub;
    int64_t bh_idx;
    {
        const int groups = subs / NW;
        int item;
        map_workgroup(g, blockIdx.x, (uint32_t)(g.n_blocks * groups), n_units, bh_idx, item);
        i = item / groups;
        qsub = (item - i * groups) * NW + wave;
    }
    const int64_t base = bh_idx * g.n_tokens * D;
    const int64_t kv_base = kv_slice_of(g, bh_idx) * g.n_tokens * D;
    // The attended blocks: block i itself followed by its selected blocks, or,
    // when the selection branch runs on its own, exactly the listed blocks.
    const int list_only = g.list_only;
    const int32_t* sel_row = sel_idx + (bh_idx * g.n_blocks + i) * g.n_select + list_only;
    const int first = list_only ? sel_row[-1] : i;
    const int n = g.n_select - list_only;        // blocks after the first
    q += base; out += base;
    const uint32_t slice_bytes = (uint32_t)(g.n_tokens * D * 2);
    const __amdgpu_buffer_rsrc_t k_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(k + kv_base), 0, slice_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(v + kv_base), 0, slice_bytes, 0x00020000);
    // zero records: every access is out of range, the load moves nothing
    const __amdgpu_buffer_rsrc_t null_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(k + kv_base), 0, 0, 0x00020000);

    // Visiting order: the own block first (it needs nothing from sel_idx, so
    // its gathers start at once), then the selected blocks in ascending block
    // order when they fit one wavefront: query blocks that run at the same time
    // on an XCD then sweep the slice's K/V in the same direction and find each
    // other's tiles in L2.  The result does not depend on the order (up to
    // rounding).  The order is computed after the first gathers are in flight;
    // order_v: lane c holds the c-th block to visit.
    const bool sorted = n + 1 <= 64;
    int order_v = first;
    auto block_at = [&](int c) -> int {
        if (c == 0) return first;
        if (__builtin_expect(sorted, 1)) return __builtin_amdgcn_readlane(order_v, c);
        return sel_row[c - 1];
    };

    // the tile width is a power of two
    const int bw_shift = __builtin_ctz((unsigned)g.block_w);
    // byte offset (inside a 64-token sub-tile) of the 16-byte chunk this lane
    // gathers in its wavefront's j-th slab (slab r = NW j + wave): sub-tile row
    // 8r + lane/8, global chunk = swizzle of its LDS slot
    uint32_t voff[8 / NW];
#pragma unroll
    for (int j = 0; j < 8 / NW; ++j) {
        const int t = 8 * (NW * j + wave) + (lane >> 3);
        voff[j] = (uint32_t)((sub_tile_pos(g, t) * D + swz(t, lane & 7) * 8) * 2);
    }
    const uint32_t wave_kib = (uint32_t)wave * 1024u;   // this wavefront's slab inside a group of NW
    auto origin_of = [&](int beta) -> uint32_t {     // byte offset of a block's first token
        const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
        return (uint32_t)((br * g.block_h * g.grid_w + bc * g.block_w) * (D * 2));
    };

    // this wavefront's slabs of a lower / upper half tile
#define BSA_GATHER_HALF_LO(RSRC, ORIGIN, LDS)                                          \
    gather_slab<NW, 0>(RSRC, ORIGIN, voff, LDS, wave_kib);                             \
    if (NW <= 2) gather_slab<NW, NW <= 2 ? 1 : 0>(RSRC, ORIGIN, voff, LDS, wave_kib);   \
    if (NW == 1) {                                                                     \
        gather_slab<NW, NW == 1 ? 2 : 0>(RSRC, ORIGIN, voff, LDS, wave_kib);           \
        gather_slab<NW, NW == 1 ? 3 : 0>(RSRC, ORIGIN, voff, LDS, wave_kib);           \
    }
#define BSA_GATHER_HALF_HI(RSRC, ORIGIN, LDS)                                          \
    gather_slab<NW, 4 / NW>(RSRC, ORIGIN, voff, LDS, wave_kib);                        \
    if (NW <= 2) gather_slab<NW, NW <= 2 ? 4 / NW + 1 : 0>(RSRC, ORIGIN, voff, LDS, wave_kib); \
    if (NW == 1) {                                                                     \
        gather_slab<NW, NW == 1 ? 6 : 0>(RSRC, ORIGIN, voff, LDS, wave_kib);           \
        gather_slab<NW, NW == 1 ? 7 : 0>(RSRC, ORIGIN, voff, LDS, wave_kib);           \
    }
    // K(0) and V(0) go to LDS (set a), in the order K half 0, K half 1, V half 0,
    // V half 1: the waits below count on it
    {
        const uint32_t origin_0 = origin_of(first) + (uint32_t)0;
        BSA_GATHER_HALF_LO(k_rsrc, origin_0, k_lds0_a);
        BSA_GATHER_HALF_HI(k_rsrc, origin_0, k_lds1_a);
        BSA_GATHER_HALF_LO(v_rsrc, origin_0, v_lds0_a);
        BSA_GATHER_HALF_HI(v_rsrc, origin_0, v_lds1_a);
    }

    // Q as B operand of S^T = K Q^T: lane (query l32 + 32 nt, half) holds
    // channels 16 ks + 8 half .. + 7.
    bf16x8 qf[2][4];
    int64_t q_tok[2];
    {
        const int br = i / g.blocks_per_row, bc = i - br * g.blocks_per_row;
        const int64_t tok0 = (int64_t)br * g.block_h * g.grid_w + (int64_t)bc * g.block_w;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int t = 64 * qsub + l32 + 32 * nt;
            const int rr = t >> bw_shift, cc = t & (g.block_w - 1);
            q_tok[nt] = tok0 + (int64_t)rr * g.grid_w + cc;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                qf[nt][ks] = *(const bf16x8*)(q + q_tok[nt] * D + 16 * ks + 8 * half);
        }
    }

    if (sorted) {
        // lane l in 1..n holds a selected block; rank = 1 + number of smaller ones
        const int mine = (lane >= 1 && lane <= n) ? sel_row[lane - 1] : 0x7fffffff;
        int rank = 1;
        for (int t = 1; t <= n; ++t)
            rank += __builtin_amdgcn_readlane(mine, t) < mine ? 1 : 0;
        if (lane >= 1 && lane <= n) order_s[wave][rank] = mine;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        order_v = order_s[wave][lane];
    }

    const float c2 = g.scale * 1.4426950408889634f;
    const f32x16 zero16 = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f,
                           0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    f32x16 oacc[2][2];      // [dt][nt]: O^T tile, rows = channels, cols = queries
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) oacc[a][b] = zero16;
    // Softmax state per query column (base-2 domain): reference maximum and
    // this lane's share of the normaliser.
    float m_ref[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};

    // V (transposing read): source lane s of 16-lane group gq supplies 8 bytes of
    //   V[key0 + 8 rd + 4 h + s/4][dbase + 4 (s%4)], h = gq/2, dbase = 16 (gq%2) + 32 dt
    const int s16 = lane & 15, gq = lane >> 4;
    const int v_row_in_step = 4 * (gq >> 1) + (s16 >> 2);
    const int v_col = 16 * (gq & 1) + 4 * (s16 & 3);     // channel (before + 32 dt)

    // fragments of one 32-key half: K rows as A operands of S^T, V through the
    // transposing read as A operands of O^T (kf[mt][ks], vf[dt][2 mt + h])
    bf16x8 kf[2][4], vf[2][4];
    auto read_k_half = [&](int mt, const unsigned char* lds_half) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            kf[mt][ks] = *(const bf16x8*)(lds_half + l32 * 128 + swz(l32, 2 * ks + half) * 16);
    };
    auto read_v_half = [&](int mt, const unsigned char* lds_half) {
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                bf16x4 part[2];
#pragma unroll
                for (int rd = 0; rd < 2; ++rd) {
                    const int row = 16 * h + 8 * rd + v_row_in_step;   // inside the half
                    const int col = v_col + 32 * dt;                   // channel, multiple of 4
                    const unsigned char* src =
                        lds_half + row * 128 + swz(row, col >> 3) * 16 + (col & 7) * 2;
                    part[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, src));
                }
                vf[dt][2 * mt + h] =
                    __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };

    // pairs: attended block cb = 0..n (visiting order), key sub-tile ct = 0..subs-1;
    // next_origin() walks them and returns the byte origin of the following pair
    // (past the end it repeats the last block; those gathers use null_rsrc)
    const int pairs = (n + 1) * subs;
    int pcb = 0, pct = 0;
    auto next_origin = [&]() -> uint32_t {
        if (++pct == subs) { pct = 0; ++pcb; }
        return origin_of(block_at(pcb <= n ? pcb : n)) + (uint32_t)(sub_tile_first(g, pct) * (D * 2));
    };
    // K or V of pair c, or the descriptor that loads nothing past the last pair
    auto k_of = [&](int c) { return c < pairs ? k_rsrc : null_rsrc; };
    auto v_of = [&](int c) { return c < pairs ? v_rsrc : null_rsrc; };
    uint32_t o_far = next_origin();                    // origin of pair c + DEPTH (here: pair 1)

    // ---- pipeline prologue: with DEPTH 2 all of pair 1 follows pair 0 into LDS
    // (set b); fragments of pair 0; K half 0 of pair DEPTH into the buffer just
    // read; S tile 0
    f32x16 s[2];            // S^T tiles, by query half
    bf16x8 p[2][2];         // P^T tiles, by query half; [h]: keys 16 h .. 16 h + 15 of the tile
    if (DEPTH == 2) {
        BSA_GATHER_HALF_LO(k_of(1), o_far, k_lds0_b);
        BSA_GATHER_HALF_HI(k_of(1), o_far, k_lds1_b);
        BSA_GATHER_HALF_LO(v_of(1), o_far, v_lds0_b);
        BSA_GATHER_HALF_HI(v_of(1), o_far, v_lds1_b);
        o_far = next_origin();                         // pair 2
        if (NW == 1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        if (NW == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (NW == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    wg_barrier();                                      // pair 0's tiles have landed
    read_k_half(0, k_lds0_a);
    read_k_half(1, k_lds1_a);
    read_v_half(0, v_lds0_a);
    {
        // the first step adds a zero tile to O: weights and V fragments of
        // "tile -1" are zeros
        const bf16x8 zero8 = __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u));
        p[1][0] = zero8; p[1][1] = zero8;
        vf[0][2] = zero8; vf[0][3] = zero8; vf[1][2] = zero8; vf[1][3] = zero8;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    wg_barrier();                                      // everyone has read K half 0
    BSA_GATHER_HALF_LO(k_of(DEPTH), o_far, k_lds0_a);
#undef BSA_GATHER_HALF_LO
#undef BSA_GATHER_HALF_HI
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][ks], qf[0][ks],
                                                       ks == 0 ? zero16 : s[0], 0, 0, 0);

    // slow path of a tile whose row sums are out of range: new reference from
    // the row maxima, rescale O and the normaliser, recompute the weights
    auto repair = [&](int nt) -> float {
        float mx = s[nt][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[nt][r]);
        mx = fmaxf(mx, swap32(mx));
        const float m_new = fmaxf(m_ref[nt], mx * c2);
        const float alpha = __builtin_amdgcn_exp2f(m_ref[nt] - m_new);
        m_ref[nt] = m_new;
        l_run[nt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
        return tile_weights(s[nt], c2, -m_new, p[nt]);
    };

    // One pair, c, whose tiles are in LDS set SET (pair c + 1: set SET ^ (DEPTH - 1)).
    // On entry o_far is the origin of pair c + DEPTH.  Loads in flight on entry
    // (DEPTH 1 / 2): K half 0 of pair c + 1 / c + 2; with DEPTH 2 also all of
    // pair c + 1.  A buffer is refilled, right after its fragments were read,
    // with the same half of the pair DEPTH (K half 0: DEPTH + 1) further on,
    // which then has three (DEPTH 2: seven) steps to arrive.
    auto one_pair = [&](int c, auto set_tag) {
        constexpr int SET = decltype(set_tag)::value;
        constexpr int NXT = DEPTH == 2 ? SET ^ 1 : 0;          // set of pair c + 1
        unsigned char* const k1_cur = SET == 0 ? k_lds1_a : k_lds1_b;
        unsigned char* const v0_cur = SET == 0 ? v_lds0_a : v_lds0_b;
        unsigned char* const v1_cur = SET == 0 ? v_lds1_a : v_lds1_b;
        unsigned char* const k0_nxt = NXT == 0 ? k_lds0_a : k_lds0_b;
        unsigned char* const k1_nxt = NXT == 0 ? k_lds1_a : k_lds1_b;
        unsigned char* const v0_nxt = NXT == 0 ? v_lds0_a : v_lds0_b;
        const uint32_t o_a = o_far;                    // origin of pair c + DEPTH
        const uint32_t o_b = next_origin();            // origin of pair c + DEPTH + 1
        const __amdgpu_buffer_rsrc_t k_a = k_of(c + DEPTH), v_a = v_of(c + DEPTH);
        const __amdgpu_buffer_rsrc_t k_b = k_of(c + DEPTH + 1);
        Refill rf;
        float rs;

        // ---- step 0: weights of tile (0,0); S of (0,1); O += tile (1,1) of the
        // previous pair.  K half 1 and V half 0 of this pair were read in the
        // previous step 3: refill them with pair c + DEPTH.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wg_barrier();
        rf = Refill{v_a, k_a, o_a, o_a, LDS_PTR(unsigned char, v0_cur), LDS_PTR(unsigned char, k1_cur)};
        rs = pipeline_step<0, true, NW>(s, p, oacc, qf, kf, vf, c2, -m_ref[0], rf, voff, wave_kib,
                                        [] {});
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0, 0)) rs = repair(0);
        l_run[0] += rs;

        // ---- step 1: weights of (0,1); S of (1,0); O += tile (0,0).  K half 0
        // of pair c+1 and V half 1 of pair c have landed: read their fragments.
        rs = pipeline_step<1, false, NW>(s, p, oacc, qf, kf, vf, c2, -m_ref[1], rf, voff, wave_kib, [&] {
            wait_older_loads();
            wg_barrier();
            read_k_half(0, k0_nxt);
            read_v_half(1, v1_cur);
        });
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0, 0)) rs = repair(1);
        l_run[1] += rs;

        // ---- step 2: weights of (1,0); S of (1,1); O += tile (0,1).  Refill the
        // two buffers just read: K half 0 with pair c + DEPTH + 1, V half 1 with
        // pair c + DEPTH.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wg_barrier();
        rf = Refill{k_b, v_a, o_b, o_a, LDS_PTR(unsigned char, k0_nxt), LDS_PTR(unsigned char, v1_cur)};
        rs = pipeline_step<2, true, NW>(s, p, oacc, qf, kf, vf, c2, -m_ref[0], rf, voff, wave_kib,
                                        [] {});
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0, 0)) rs = repair(0);
        l_run[0] += rs;

        // ---- step 3: weights of (1,1); S of tile (0,0) of pair c+1; O += tile
        // (1,0).  K half 1 and V half 0 of pair c+1 have landed: read them.
        rs = pipeline_step<3, false, NW>(s, p, oacc, qf, kf, vf, c2, -m_ref[1], rf, voff, wave_kib, [&] {
            wait_older_loads();
            wg_barrier();
            read_k_half(1, k1_nxt);
            read_v_half(0, v0_nxt);
        });
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0, 0)) rs = repair(1);
        l_run[1] += rs;

        o_far = o_b;
    };
    if (DEPTH == 1) {
        for (int c = 0; c < pairs; ++c) one_pair(c, SetTag<0>{});
    } else {
        // (two tiles are kept only by workgroups of 2 or 4 wavefronts, whose
        // blocks have an even number of 64-key sub-tiles: pairs is even)
        for (int c = 0; c < pairs; c += 2) {
            one_pair(c, SetTag<0>{});
            one_pair(c + 1, SetTag<1>{});
        }
    }

    // ---- pipeline epilogue: O += tile (1,1) of the last pair
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
            oacc[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][2 + h], p[1][h],
                                                                  oacc[dt][1], 0, 0, 0);

    // ---- normalise, store O rows (4 consecutive channels per store)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const float l_tot = l_run[nt] + swap32(l_run[nt]);
        const float inv_l = 1.0f / l_tot;
        uint16_t* orow = out + q_tok[nt] * D;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = 32 * dt + 8 * r4 + 4 * half;
                uint2 w;
                w.x = pack_bf16(oacc[dt][nt][4 * r4] * inv_l, oacc[dt][nt][4 * r4 + 1] * inv_l);
                w.y = pack_bf16(oacc[dt][nt][4 * r4 + 2] * inv_l,
                                oacc[dt][nt][4 * r4 + 3] * inv_l);
                *(uint2*)(orow + d) = w;
            }
        if (lse && half == 0)
            lse[bh_idx * g.n_tokens + q_tok[nt]] =
                (m_ref[nt] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}

// One kernel per workgroup size (plain functions: the body is the template).
// Workgroups of 2 or 4 wavefronts keep two K/V tiles in LDS (32 KiB: the CU's
// LDS still holds its 8 wavefronts); a lone wavefront keeps one.
#define BSA_FWD_D64_KERNEL(NAME, NW, DEPTH)                                                       \
    __global__ __launch_bounds__(64 * NW, 2) void NAME(                                           \
        const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,                           \
        const uint16_t* __restrict__ v, const int32_t* __restrict__ sel_idx,                      \
        uint16_t* __restrict__ out, float* __restrict__ lse, Geom g, uint32_t n_units,            \
        int subs)                                                                                 \
    {                                                                                             \
        fwd_mfma_d64_body<NW, DEPTH>(q, k, v, sel_idx, out, lse, g, n_units, subs);               \
    }
BSA_FWD_D64_KERNEL(fwd_mfma_b64_d64_kernel, 1, 1)
BSA_FWD_D64_KERNEL(fwd_mfma_d64_wg2_kernel, 2, 2)
BSA_FWD_D64_KERNEL(fwd_mfma_d64_wg4_kernel, 4, 2)
#undef BSA_FWD_D64_KERNEL

bool fwd_mfma_supported(bool is_bf16, const Geom& g, int D)
{
    // tiles of 64*T tokens whose width is a power of two: every 64-token
    // sub-tile is then whole tile rows or a 64-token run of one tile row
    // (a token row is 128 bytes, so 16-byte chunks never straddle tokens);
    // buffer offsets inside a slice are 32-bit
    return is_bf16 && D == 64 && g.block_tokens % 64 == 0 &&
           (g.block_w & (g.block_w - 1)) == 0 &&
           g.n_tokens * D * 2 < ((int64_t)1 << 31);
}

hipError_t launch_fwd_mfma(const void* q, const void* k, const void* v, const int32_t* sel_idx,
                           void* out, float* lse, const Geom& g, int D, int64_t BH,
                           hipStream_t stream)
{
    (void)D;
    const int subs = g.block_tokens / 64;
    // the sub-blocks of a query block share their K/V tiles in LDS, four or two
    // to a workgroup when the count allows
    const int nw = subs % 4 == 0 ? 4 : subs % 2 == 0 ? 2 : 1;
    dim3 grid((unsigned)(BH * g.n_blocks * (subs / nw)));
    auto kernel = nw == 4 ? fwd_mfma_d64_wg4_kernel
                  : nw == 2 ? fwd_mfma_d64_wg2_kernel : fwd_mfma_b64_d64_kernel;
    kernel<<<grid, dim3(64 * nw), 0, stream>>>((const uint16_t*)q, (const uint16_t*)k,
                                               (const uint16_t*)v, sel_idx, (uint16_t*)out, lse, g,
                                               (uint32_t)(BH / g.kv_group), subs);
    return hipGetLastError();
}

}  // namespace bsa
