// Block-sparse attention forward on the gfx950 matrix cores for head dim 128
// (bf16 MFMA, fp32 online softmax): the gradient configuration's shape.
//
// Every token of query block i attends, in one softmax, to the tokens of block
// i and of its n selected blocks (fine-grained attention equation plus the
// local block).  With 128 channels an output row costs twice the accumulator
// registers of the 64-channel kernel, so a wavefront owns 32 query rows and a
// workgroup of NW = b/32 wavefronts owns the query block.  Its wavefronts
// attend to the same blocks, so every K/V tile is gathered into LDS once per
// workgroup and read by all of them: the CU's load path, which limits the
// one-wavefront-per-block kernel, carries NW times fewer bytes per flop.
//
// Per wavefront, per 64-key sub-tile ("pair"), as in the 64-channel kernel:
// transposed products S^T = K Q^T and O^T = V^T P^T with
// v_mfma_f32_32x32x16_bf16 (a lane holds one query column; the S^T accumulator
// registers are the B operand of the second product), K fragments from 16-byte
// LDS reads, V^T fragments from the transposing LDS read, K/V gathered with
// direct-to-LDS buffer loads whose lane-to-chunk mapping applies the LDS
// swizzle on the global side, weights rounded to bf16 (nearest even) with the
// normaliser summed in fp32, and no row maximum per tile (slow path only when
// a row sum leaves the safe range).
//
// Schedule.  A pair is two tiles of 32 keys x 32 queries.  Step J (tile J of
// the pair) issues the 8 MFMAs of the S tile J+1, then the 8 MFMAs that add
// tile J-1 to O, and spreads the vector work of the weights of tile J behind
// them (the exponentials must sit between the MFMAs of the wavefront that owns
// them: a wavefront streaming MFMAs keeps the other wavefronts of its SIMD from
// issuing vector work).  Only one 32-key half of K fragments and one of V
// fragments is live: the K half is re-read from LDS after the S MFMAs of a
// step, the V half after its O MFMAs.
//
// LDS: K and V as two 32-key halves each (4 x 8 KiB).  A half is read once per
// pair by every wavefront and then refilled with the same half of the next
// sub-tile; the 8 loads of a half are split between the wavefronts.  A step
// has two workgroup barriers: at its start "all reads of the K half read in the
// previous step are done", after which that K half is refilled; after its S
// MFMAs "the halves refilled a step ago have landed" (each wavefront waits for
// its own loads first) and "all reads of the V half read at the end of the
// previous step are done", after which the K half is read and that V half is
// refilled.
#include <type_traits>

#include "bsa_device.h"
#include "bsa_launch.h"
#include "bsa_mfma_common.h"

namespace bsa {

namespace q32 {

// 16-byte chunk swizzle of an LDS row (16 chunks per 256-byte row, 8 per
// 128-byte row).  The K fragment read takes the same chunk of 8 consecutive
// rows per 128 bytes of bank width, the transposing V read 32 bytes (a chunk
// pair) of 4 consecutive rows: the row's XOR mask is a bijection of row % 8
// whose upper two bits differ over any 4 aligned rows.
__device__ __forceinline__ int swz(int row, int chunk)
{
    return chunk ^ (((row & 3) << 1) | ((row >> 2) & 1));
}

}  // namespace q32

// D: head dim; NW: wavefronts per workgroup = query block / 32.  Only D = 128
// is instantiated: at D = 64 the same body fits three wavefronts per SIMD (155
// registers) and measured no faster than the kernel with 64 query rows per
// wavefront (blocks of 128 tokens: the same time; blocks of 64: 8 % slower).
template <int D, int NW>
__device__ __forceinline__ void fwd_mfma_q32_body(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const int32_t* __restrict__ sel_idx,
    uint16_t* __restrict__ out, float* __restrict__ lse, const Geom& g, uint32_t n_units)
{
    using namespace q32;
    constexpr int ROW_BYTES = D * 2;               // one token row of K or V in LDS
    constexpr int HALF_BYTES = 32 * ROW_BYTES;
    constexpr int KS = D / 16;                     // k-steps of S^T = K Q^T
    constexpr int DT = D / 32;                     // 32-channel tiles of O^T
    constexpr int NSLOT = KS + 2 * DT;             // MFMAs per step
    constexpr int SPC = NSLOT / 8;                 // MFMA slots per chunk of weights
    constexpr int SLAB_ROWS = 1024 / ROW_BYTES;    // token rows per 1 KiB load
    constexpr int CHUNKS = ROW_BYTES / 16;         // 16-byte chunks per row
    constexpr int HALF_LOADS = 32 / SLAB_ROWS;     // loads per half tile
    static_assert(HALF_LOADS % NW == 0, "the loads of a half tile are split between the waves");
    constexpr int LOADS = HALF_LOADS / NW;         // loads per wavefront and half refill
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds0[HALF_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds1[HALF_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds0[HALF_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds1[HALF_BYTES];
    __shared__ int order_s[NW][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int subs = g.block_tokens / 64;          // 64-key sub-tiles per attended block

    // Workgroup -> (query slice, query block); key/value slices are dealt to
    // the XCDs whole (map_workgroup).
    int i;
    int64_t bh_idx;
    map_workgroup(g, blockIdx.x, (uint32_t)g.n_blocks, n_units, bh_idx, i);
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

    // Visiting order: own block first, then the selected blocks in ascending
    // block order when they fit one wavefront (workgroups that run together on
    // an XCD then sweep the slice's K/V in the same direction).  Every
    // wavefront computes the order for itself; lane c holds the c-th block.
    const bool sorted = n + 1 <= 64;
    int order_v = first;
    auto block_at = [&](int c) -> int {
        if (c == 0) return first;
        if (__builtin_expect(sorted, 1)) return __builtin_amdgcn_readlane(order_v, c);
        return sel_row[c - 1];
    };

    // Gather geometry.  One load moves 1 KiB = SLAB_ROWS token rows; lane l
    // fills LDS chunk l of that slab, i.e. row l / CHUNKS, swizzled chunk
    // l % CHUNKS, so it fetches the global chunk that swizzles to l % CHUNKS
    // (the swizzle is an involution).  The tile width is a power of two >=
    // SLAB_ROWS, so the tokens of a slab are contiguous in memory: a per-lane
    // offset (two variants, by the parity of the slab inside the half: the
    // swizzle looks at the row modulo 8) plus a wave-uniform offset of the
    // slab's first token.
    const int bw_shift = __builtin_ctz((unsigned)g.block_w);
    uint32_t voff_par[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int row = SLAB_ROWS * par + lane / CHUNKS;
        voff_par[par] =
            (uint32_t)((lane / CHUNKS) * ROW_BYTES + swz(row, lane % CHUNKS) * 16);
    }
    auto slab_offset = [&](int hh, int slab) -> uint32_t {   // first token of a slab, bytes
        return (uint32_t)(sub_tile_pos(g, 32 * hh + SLAB_ROWS * slab) * ROW_BYTES);
    };
    auto origin_of = [&](int beta) -> uint32_t {     // byte offset of a block's first token
        const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
        return (uint32_t)((br * g.block_h * g.grid_w + bc * g.block_w) * ROW_BYTES);
    };
    // this wavefront's share of a half refill: slabs LOADS*wave .. +LOADS-1
    auto refill_half = [&](__amdgpu_buffer_rsrc_t rsrc, uint32_t origin, int hh,
                           unsigned char* lds_half) {
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int slab = LOADS * wave + j;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc, LDS_PTR(void, lds_half + slab * 1024), 16, voff_par[slab & 1],
                origin + slab_offset(hh, slab), 0, 0);
        }
    };

    // pair 0: K (both halves) and the lower half of V go to LDS
    {
        const uint32_t origin_0 = origin_of(first);
        refill_half(k_rsrc, origin_0, 0, k_lds0);
        refill_half(k_rsrc, origin_0, 1, k_lds1);
        refill_half(v_rsrc, origin_0, 0, v_lds0);
    }

    // Q as B operand of S^T = K Q^T: lane (query l32, half) holds channels
    // 16 ks + 8 half .. + 7 of this wavefront's query row.
    bf16x8 qf[KS];
    int64_t q_tok;
    {
        const int br = i / g.blocks_per_row, bc = i - br * g.blocks_per_row;
        const int64_t tok0 = (int64_t)br * g.block_h * g.grid_w + (int64_t)bc * g.block_w;
        const int t = 32 * wave + l32;
        const int rr = t >> bw_shift, cc = t & (g.block_w - 1);
        q_tok = tok0 + (int64_t)rr * g.grid_w + cc;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = *(const bf16x8*)(q + q_tok * D + 16 * ks + 8 * half);
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
    f32x16 oacc[DT];        // [dt]: O^T tile, rows = channels 32 dt .., cols = queries
#pragma unroll
    for (int a = 0; a < DT; ++a) oacc[a] = zero16;
    float m_ref = -INFINITY, l_run = 0.0f;

    // V (transposing read): source lane s of 16-lane group gq supplies 8 bytes of
    //   V[key0 + 8 rd + 4 h + s/4][dbase + 4 (s%4)], h = gq/2, dbase = 16 (gq%2) + 32 dt
    const int s16 = lane & 15, gq = lane >> 4;
    const int v_row_in_step = 4 * (gq >> 1) + (s16 >> 2);
    const int v_col = 16 * (gq & 1) + 4 * (s16 & 3);     // channel (before + 32 dt)

    // fragments of one 32-key half: K rows as A operands of S^T (kf[ks]), V
    // through the transposing read as A operands of O^T (vf[dt][h], keys 16 h ..)
    bf16x8 kf[KS], vf[DT][2];
    auto read_k_half = [&](const unsigned char* lds_half) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            kf[ks] = *(const bf16x8*)(lds_half + l32 * ROW_BYTES + swz(l32, 2 * ks + half) * 16);
    };
    auto read_v_half = [&](const unsigned char* lds_half) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                bf16x4 part[2];
#pragma unroll
                for (int rd = 0; rd < 2; ++rd) {
                    const int row = 16 * h + 8 * rd + v_row_in_step;   // inside the half
                    const int col = v_col + 32 * dt;                   // channel, multiple of 4
                    const unsigned char* src =
                        lds_half + row * ROW_BYTES + swz(row, col >> 3) * 16 + (col & 7) * 2;
                    part[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, src));
                }
                vf[dt][h] = __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };

    // pairs: attended block cb = 0..n (visiting order), key sub-tile ct = 0..subs-1;
    // next_origin() walks them and returns the byte origin of the following pair
    // (past the end it repeats the last block; those gathers use null_rsrc)
    const int pairs = (n + 1) * subs;
    int pcb = 0, pct = 0;
    auto next_origin = [&]() -> uint32_t {
        if (++pct == subs) { pct = 0; ++pcb; }
        return origin_of(block_at(pcb <= n ? pcb : n)) + (uint32_t)(sub_tile_first(g, pct) * ROW_BYTES);
    };
    uint32_t o0 = origin_of(first);                        // origin of pair c
    uint32_t o1 = next_origin();                       // origin of pair c + 1

    // ---- pipeline prologue
    f32x16 s[2];            // S^T tiles, by tile parity (= key half)
    bf16x8 p[2][2];         // P^T tiles, by tile parity; [h]: keys 16 h .. 16 h + 15 of the tile
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                      // pair 0's K and lower V have landed
    read_k_half(k_lds0);
    {
        // the first step adds a zero tile to O
        const bf16x8 zero8 = __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u));
        p[1][0] = zero8; p[1][1] = zero8;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) { vf[dt][0] = zero8; vf[dt][1] = zero8; }
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], ks == 0 ? zero16 : s[0], 0,
                                                       0, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_k_half(k_lds1);                               // K(0) upper half, for step 0
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                      // everyone has read K half 0
    refill_half(1 < pairs ? k_rsrc : null_rsrc, o1, 0, k_lds0);

    // slow path of a tile whose row sums are out of range: new reference from
    // the row maxima, rescale O and the normaliser, recompute the weights
    auto repair = [&](int par) -> float {
        float mx = s[par][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[par][r]);
        mx = fmaxf(mx, swap32(mx));
        const float m_new = fmaxf(m_ref, mx * c2);
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
        return tile_weights(s[par], c2, -m_new, p[par]);
    };

    // The K fragment reads of the previous step are older than the 4 DT V reads
    // issued after them, so "at most 4 DT - 1 outstanding" covers them (LDS
    // operations complete in order; not so with a scalar load of the selection
    // row in flight).
    auto wait_k_reads = [&] {
        if (!sorted) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        else if (DT == 4) asm volatile("s_waitcnt lgkmcnt(15)" ::: "memory");
        else asm volatile("s_waitcnt lgkmcnt(7)" ::: "memory");
    };

    // everything but this wavefront's most recent refill share has landed, and
    // its LDS reads are done
    auto wait_older_loads = [] {
        if (LOADS == 1) asm volatile("s_waitcnt vmcnt(1) lgkmcnt(0)" ::: "memory");
        if (LOADS == 2) asm volatile("s_waitcnt vmcnt(2) lgkmcnt(0)" ::: "memory");
        if (LOADS == 4) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
    };

    // One step: tile J of the pair (key half J).  S of the next tile from the
    // K fragments in registers (KS MFMAs), then the K fragments of the tile
    // after that are requested from k_next_lds; O += previous tile with the V
    // fragments in registers (2 DT MFMAs), then the next V fragments are requested
    // from v_next_lds.  `before_k` runs before the K request (wait for the
    // refill of that half), `early` right after the first MFMA (barrier and
    // refill issue).  The weights of tile J are spread behind the MFMAs.
    auto step = [&](auto J_tag, auto early, auto before_k, const unsigned char* k_next_lds,
                    const unsigned char* v_next_lds) -> float {
        constexpr int J = decltype(J_tag)::value;
        const float neg_m = -m_ref;
        uint32_t w[8];
        float rs0 = 0.0f, rs1 = 0.0f;
        float f[9][2], e[8][2];
        f[0][0] = fmaf(s[J][0], c2, neg_m);
        f[0][1] = fmaf(s[J][1], c2, neg_m);
        asm volatile("" : "+v"(f[0][0]), "+v"(f[0][1]));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kslot = 0; kslot < NSLOT; ++kslot) {
            if (kslot < KS) {
                s[1 - J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    kf[kslot], qf[kslot], kslot == 0 ? zero16 : s[1 - J], 0, 0, 0);
            } else {
                const int dt = (kslot - KS) % DT, h = (kslot - KS) / DT;
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][h], p[1 - J][h],
                                                                   oacc[dt], 0, 0, 0);
            }
            if (kslot == 0) {
                early();
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kslot == KS) {
                // the S MFMAs have been issued: the K fragment registers are free
                before_k();
                read_k_half(k_next_lds);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kslot % SPC == SPC - 1) {
                // exp2 of this chunk, fma of the next, pack and row sums of the
                // previous one: nothing waits for the instruction before it
                const int ch = kslot / SPC;
                e[ch][0] = __builtin_amdgcn_exp2f(f[ch][0]);
                e[ch][1] = __builtin_amdgcn_exp2f(f[ch][1]);
                if (ch + 1 < 8) {
                    f[ch + 1][0] = fmaf(s[J][2 * ch + 2], c2, neg_m);
                    f[ch + 1][1] = fmaf(s[J][2 * ch + 3], c2, neg_m);
                } else {
                    f[ch + 1][0] = 0.0f; f[ch + 1][1] = 0.0f;
                }
                if (ch >= 1) {
                    w[ch - 1] = pack_bf16(e[ch - 1][0], e[ch - 1][1]);
                    rs0 += e[ch - 1][0];
                    rs1 += e[ch - 1][1];
                } else {
                    w[7] = 0;
                }
                // an empty statement that "uses" the chunk's results keeps
                // their producers here instead of after the last MFMA
                asm volatile(""
                             : "+v"(e[ch][0]), "+v"(e[ch][1]), "+v"(f[ch + 1][0]),
                               "+v"(f[ch + 1][1]), "+v"(w[ch >= 1 ? ch - 1 : 7]), "+v"(rs0),
                               "+v"(rs1));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // the O MFMAs have been issued: the V fragment registers are free
        read_v_half(v_next_lds);
        w[7] = pack_bf16(e[7][0], e[7][1]);
        rs0 += e[7][0];
        rs1 += e[7][1];
        p[J][0] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
        p[J][1] = __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7]));
        return rs0 + rs1;
    };

    for (int c = 0; c < pairs; ++c) {
        const uint32_t o2 = next_origin();             // origin of pair c + 2
        const __amdgpu_buffer_rsrc_t k1 = c + 1 < pairs ? k_rsrc : null_rsrc;
        const __amdgpu_buffer_rsrc_t v1 = c + 1 < pairs ? v_rsrc : null_rsrc;
        const __amdgpu_buffer_rsrc_t k2 = c + 2 < pairs ? k_rsrc : null_rsrc;
        float rs;

        // ---- step 0: weights of tile 0; S of tile 1 (K upper half, in
        // registers); O += tile 1 of the previous pair.  The upper halves were
        // read in the previous step 1: once everyone is past those reads,
        // refill them (K upper of pair c+1, V upper of pair c).  After the S
        // MFMAs: K lower half of pair c+1 (refilled a step ago) -> registers;
        // after the O MFMAs: V lower half of pair c -> registers.
        rs = step(
            std::integral_constant<int, 0>{},
            [&] {
                wait_k_reads();
                __builtin_amdgcn_s_barrier();
                refill_half(k1, o1, 1, k_lds1);
            },
            [&] {
                // own share of the lower-half refills has landed (everything
                // older than the K loads just issued), own V reads are done;
                // then everyone's.  The V upper half can be refilled now.
                wait_older_loads();
                __builtin_amdgcn_s_barrier();
                refill_half(v_rsrc, o0, 1, v_lds1);     // pair c itself always exists
            },
            k_lds0, v_lds0);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0, 0))
            rs = repair(0);
        l_run += rs;

        // ---- step 1: weights of tile 1; S of tile 0 of pair c+1 (K lower half,
        // in registers); O += tile 0 (V lower half, in registers).  The lower
        // halves were read in step 0: refill them (K lower of pair c+2, V lower
        // of pair c+1).  After the S MFMAs: K upper half of pair c+1 ->
        // registers; after the O MFMAs: V upper half of pair c -> registers.
        rs = step(
            std::integral_constant<int, 1>{},
            [&] {
                wait_k_reads();
                __builtin_amdgcn_s_barrier();
                refill_half(k2, o2, 0, k_lds0);
            },
            [&] {
                wait_older_loads();
                __builtin_amdgcn_s_barrier();
                refill_half(v1, o1, 0, v_lds0);
            },
            k_lds1, v_lds1);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0, 0))
            rs = repair(1);
        l_run += rs;

        o0 = o1;
        o1 = o2;
    }

    // ---- pipeline epilogue: O += tile 1 of the last pair
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][h], p[1][h], oacc[dt], 0, 0,
                                                               0);

    // ---- normalise, store O rows (4 consecutive channels per store)
    {
        const float l_tot = l_run + swap32(l_run);
        const float inv_l = 1.0f / l_tot;
        uint16_t* orow = out + q_tok * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d = 32 * dt + 8 * r4 + 4 * half;
                uint2 w;
                w.x = pack_bf16(oacc[dt][4 * r4] * inv_l, oacc[dt][4 * r4 + 1] * inv_l);
                w.y = pack_bf16(oacc[dt][4 * r4 + 2] * inv_l, oacc[dt][4 * r4 + 3] * inv_l);
                *(uint2*)(orow + d) = w;
            }
        if (lse && half == 0)
            lse[bh_idx * g.n_tokens + q_tok] =
                (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}

// head dim 128: query blocks of 128 tokens (the gradient configuration), 64 and
// 256 tokens as workgroups of 4, 2 and 8 wavefronts; two wavefronts per SIMD
#define BSA_FWD_D128_KERNEL(NAME, NW_)                                                            \
    __global__ __launch_bounds__(64 * NW_, 2) void NAME(                                          \
        const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,                           \
        const uint16_t* __restrict__ v, const int32_t* __restrict__ sel_idx,                      \
        uint16_t* __restrict__ out, float* __restrict__ lse, Geom g, uint32_t n_units)            \
    {                                                                                             \
        fwd_mfma_q32_body<128, NW_>(q, k, v, sel_idx, out, lse, g, n_units);                      \
    }
BSA_FWD_D128_KERNEL(fwd_mfma_d128_kernel, 4)
BSA_FWD_D128_KERNEL(fwd_mfma_d128_w2_kernel, 2)
BSA_FWD_D128_KERNEL(fwd_mfma_d128_w8_kernel, 8)
#undef BSA_FWD_D128_KERNEL

bool fwd_mfma_d128_supported(bool is_bf16, const Geom& g, int D)
{
    // query block = 2, 4 or 8 wavefronts x 32 rows; 64-key sub-tiles of whole
    // tile rows or 64-token runs of a row (the tile width is a power of two)
    // whose 4-token load slabs are contiguous (the width is at least 4); buffer
    // offsets inside a slice are 32-bit
    const int b = g.block_tokens;
    return is_bf16 && D == 128 && (b == 64 || b == 128 || b == 256) &&
           (g.block_w & (g.block_w - 1)) == 0 && g.block_w >= 4 && g.n_tokens * D * 2 < ((int64_t)1 << 31);
}

hipError_t launch_fwd_mfma_d128(const void* q, const void* k, const void* v,
                                const int32_t* sel_idx, void* out, float* lse, const Geom& g,
                                int64_t BH, hipStream_t stream)
{
    dim3 grid((unsigned)(BH * g.n_blocks));
    const int nw = g.block_tokens / 32;
    auto kernel = nw == 4 ? fwd_mfma_d128_kernel
                  : nw == 2 ? fwd_mfma_d128_w2_kernel : fwd_mfma_d128_w8_kernel;
    kernel<<<grid, dim3(64 * nw), 0, stream>>>(
        (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, sel_idx, (uint16_t*)out, lse, g,
        (uint32_t)(BH / g.kv_group));
    return hipGetLastError();
}

}  // namespace bsa
