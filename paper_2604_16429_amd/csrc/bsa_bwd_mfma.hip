// Backward of the block-sparse attention on the gfx950 matrix cores (bf16 MFMA,
// fp32 accumulation), selection held fixed: no gradient flows through the
// top-n choice (Appendix "Block-sparse attention implementation").
//
// With P the attention weights of the forward pass, recomputed from the stored
// log-sum-exp as P = exp(scale * q.k - lse), and delta_l = dO_l . O_l:
//   dV_t = sum_l P_lt dO_l          dP_lt = dO_l . v_t
//   dS_lt = P_lt (dP_lt - delta_l)
//   dQ_l = scale * sum_t dS_lt k_t  dK_t = scale * sum_l dS_lt q_l
// where t runs over the keys of the blocks query block i attends to (itself and
// its selection) and l over the queries of the blocks that attend to t's block.
//
// Two main kernels, both built from 32 x 32 x 16 bf16 MFMAs on 64-token tiles that
// the wavefronts of a workgroup share through LDS (direct-to-LDS gathers,
// double buffered, one workgroup barrier per tile):
//   dq kernel    one workgroup per query block, a wavefront per 32 query rows,
//                walks the attended K/V sub-tiles like the forward pass.  Per
//                32-key tile: S^T = K Q^T and dP^T = V dO^T (a lane holds one
//                query column, so lse and delta are per-lane scalars),
//                dS^T in registers is the B operand of dQ^T += K^T dS^T, whose A
//                operand comes from the transposing LDS read of the K tile.
//   dk/dv kernel one workgroup per key/value block, a wavefront per 32 key rows
//                (their K and V rows stay in registers as B operands).  It
//                lists, in ascending order, the query blocks that attend to
//                its block (the paper's "query blocks connected to a key/value
//                block"), from a reverse map of the selection that a small
//                kernel builds first: a bit matrix, one bit per (key block,
//                query block).  No floating-point atomics: the ascending list
//                fixes the summation order.  It then walks their Q/dO
//                sub-tiles.  Per 32-query tile: S = Q K^T and dP = dO V^T (rows
//                are queries now: lse and delta come from LDS per row), and
//                dV^T += dO^T P, dK^T += Q^T dS with the transposing LDS read
//                of the dO / Q tile.  For head dim 128 the two accumulators do
//                not fit next to the operands, so dV and dK are two passes.
#include "bsa_device.h"
#include "bsa_launch.h"
#include "bsa_mfma_common.h"

namespace bsa {

namespace bwdm {

constexpr float kLog2e = 1.4426950408889634f;

// 16-byte chunk swizzle of an LDS row (8 or 16 chunks): a bijection of row % 8
// whose upper two bits differ over 4 aligned rows (row-fragment reads take the
// same chunk of 8 consecutive rows, transposing reads a chunk pair of 4 rows).
__device__ __forceinline__ int swz(int row, int chunk)
{
    return chunk ^ (((row & 3) << 1) | ((row >> 2) & 1));
}

// Geometry of 64-token x D tiles gathered into LDS by a workgroup of NW
// wavefronts.  A tile is SLABS loads of 1 KiB (RPS token rows each); wavefront
// w issues slabs w, w + NW, ...; lane l fills LDS chunk l of the slab, i.e. row
// l / LPR, swizzled chunk l % LPR, and therefore fetches the global chunk that
// swizzles to that slot.
template <int D, int NW>
struct TileIO {
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int TILE_BYTES = 64 * ROW_BYTES;
    static constexpr int SLABS = TILE_BYTES / 1024;
    static constexpr int RPS = 1024 / ROW_BYTES;       // token rows per slab
    static constexpr int LPR = ROW_BYTES / 16;         // lanes per token row
    static constexpr int MINE = SLABS / NW;            // slabs per wavefront
    static_assert(SLABS % NW == 0, "slabs split evenly between wavefronts");

    uint32_t voff[MINE];        // byte offset of this lane's chunk inside a sub-tile
    uint32_t tok_off;           // byte offset (fp32 rows) of token `lane` of a sub-tile
    int wave;

    __device__ __forceinline__ void init(const Geom& g, int lane, int wave_)
    {
        wave = wave_;
#pragma unroll
        for (int j = 0; j < MINE; ++j) {
            const int slab = wave + j * NW;
            const int t = RPS * slab + lane / LPR;                    // token row 0..63
            voff[j] = (uint32_t)(sub_tile_pos(g, t) * ROW_BYTES + swz(t, lane % LPR) * 16);
        }
        tok_off = (uint32_t)(sub_tile_pos(g, lane) * 4);
    }
    // this wavefront's share of one tile (origin: byte offset of the sub-tile's
    // first token in a [N, D] bf16 slice)
    __device__ __forceinline__ void gather(__amdgpu_buffer_rsrc_t rsrc, uint32_t origin,
                                           unsigned char* lds_tile) const
    {
#pragma unroll
        for (int j = 0; j < MINE; ++j) {
            const int slab = wave + j * NW;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(void, lds_tile + slab * 1024), 16,
                                                     voff[j], origin, 0, 0);
        }
    }
    // 64 fp32 values (one per token of the sub-tile) from a [N] fp32 slice;
    // origin_tok: index of the sub-tile's first token
    __device__ __forceinline__ void gather_f32(__amdgpu_buffer_rsrc_t rsrc, uint32_t origin_tok,
                                               float* lds_vec) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(void, lds_vec), 4, tok_off,
                                                 origin_tok * 4u, 0, 0);
    }
};

// Row fragment: lane (l32, half) reads channels 16 ks + 8 half .. + 7 of tile
// row row0 + l32 (A operand "rows x channels", or B operand of the same shape).
template <int D>
__device__ __forceinline__ bf16x8 row_frag(const unsigned char* tile, int row0, int ks, int l32,
                                           int half)
{
    const int row = row0 + l32;
    return *(const bf16x8*)(tile + row * (D * 2) + swz(row, 2 * ks + half) * 16);
}

// Transposed fragment: A operand "channels 32 dt .. x tile rows row0 .. row0+15"
// through the transposing LDS read (source lane s of 16-lane group gq supplies
// 8 bytes of row row0 + 8 rd + 4 (gq/2) + s/4, channel 16 (gq%2) + 4 (s%4) + 32 dt).
template <int D>
__device__ __forceinline__ bf16x8 trans_frag(const unsigned char* tile, int row0, int dt,
                                             int lane)
{
    const int s16 = lane & 15, gq = lane >> 4;
    const int col = 16 * (gq & 1) + 4 * (s16 & 3) + 32 * dt;
    bf16x4 part[2];
#pragma unroll
    for (int rd = 0; rd < 2; ++rd) {
        const int row = row0 + 8 * rd + 4 * (gq >> 1) + (s16 >> 2);
        const unsigned char* src = tile + row * (D * 2) + swz(row, col >> 3) * 16 + (col & 7) * 2;
        part[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, src));
    }
    return __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
}

// 16 fp32 accumulator values -> two bf16 B operands (round to nearest even)
__device__ __forceinline__ void pack_tile(const f32x16& x, bf16x8 (&b)[2])
{
#pragma unroll
    for (int h = 0; h < 2; ++h)
        b[h] = __builtin_bit_cast(
            bf16x8, make_uint4(pack_bf16(x[8 * h + 0], x[8 * h + 1]),
                               pack_bf16(x[8 * h + 2], x[8 * h + 3]),
                               pack_bf16(x[8 * h + 4], x[8 * h + 5]),
                               pack_bf16(x[8 * h + 6], x[8 * h + 7])));
}

// Store one accumulator tile (rows = channels 32 dt .., this lane's column =
// one token row) scaled by f: 4 consecutive channels per 8-byte store.  With
// `extra` (fp32 row of D channels) the tile is added to what the row holds,
// together with extra * inv_b.
__device__ __forceinline__ void store_tile(uint16_t* row_ptr, int dt, int half, const f32x16& a,
                                           float f, const float* extra = nullptr,
                                           float inv_b = 0.0f)
{
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
        const int d = 32 * dt + 8 * r4 + 4 * half;
        float x0 = a[4 * r4] * f, x1 = a[4 * r4 + 1] * f, x2 = a[4 * r4 + 2] * f,
              x3 = a[4 * r4 + 3] * f;
        if (extra) {
            const uint2 old = *(const uint2*)(row_ptr + d);
            const float4 e = *(const float4*)(extra + d);
            x0 += __uint_as_float(old.x << 16) + e.x * inv_b;
            x1 += __uint_as_float(old.x & 0xffff0000u) + e.y * inv_b;
            x2 += __uint_as_float(old.y << 16) + e.z * inv_b;
            x3 += __uint_as_float(old.y & 0xffff0000u) + e.w * inv_b;
        }
        uint2 w;
        w.x = pack_bf16(x0, x1);
        w.y = pack_bf16(x2, x3);
        *(uint2*)(row_ptr + d) = w;
    }
}

__device__ __forceinline__ f32x16 zero_tile()
{
    const f32x16 z = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f,
                      0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    return z;
}

// ---------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------
template <int D, int NW>
__device__ __forceinline__ void dq_body(const uint16_t* __restrict__ q,
                                        const uint16_t* __restrict__ k,
                                        const uint16_t* __restrict__ v,
                                        const uint16_t* __restrict__ dout,
                                        const float* __restrict__ lse2,
                                        const float* __restrict__ delta,
                                        const int32_t* __restrict__ sel_idx,
                                        uint16_t* __restrict__ dq, const Geom& g,
                                        uint32_t n_units)
{
    constexpr int KS = D / 16, DT = D / 32;
    using IO = TileIO<D, NW>;
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[2][IO::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds[2][IO::TILE_BYTES];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int subs = g.block_tokens / 64;

    // workgroup -> (query slice, query block), key/value slices dealt to the 8
    // XCDs whole
    int i;
    int64_t bh_idx;
    map_workgroup(g, blockIdx.x, (uint32_t)g.n_blocks, n_units, bh_idx, i);
    const int64_t base = bh_idx * g.n_tokens * D;
    const int64_t kv_base = kv_slice_of(g, bh_idx) * g.n_tokens * D;
    // The attended blocks: block i itself followed by its selected blocks, or,
    // in list-only mode, exactly the listed blocks.
    const int list_only = g.list_only;
    const int32_t* sel_row = sel_idx + (bh_idx * g.n_blocks + i) * g.n_select + list_only;
    const int first = list_only ? sel_row[-1] : i;
    const int n = g.n_select - list_only;        // blocks after the first
    const uint32_t slice_bytes = (uint32_t)(g.n_tokens * D * 2);
    const __amdgpu_buffer_rsrc_t k_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(k + kv_base), 0, slice_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(v + kv_base), 0, slice_bytes, 0x00020000);

    IO io;
    io.init(g, lane, wave);
    auto origin_of = [&](int beta) -> uint32_t {     // byte offset of a block's first token
        const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
        return (uint32_t)((br * g.block_h * g.grid_w + bc * g.block_w) * (D * 2));
    };
    const int pairs = (n + 1) * subs;
    // the listed blocks sit in the lanes of one register (up to 64 of them), so
    // that finding the next tile costs no memory access inside the loop
    const int sel_mine = (n <= 64 && lane < n) ? sel_row[lane] : 0;
    auto origin_of_pair = [&](int c) -> uint32_t {   // attended block c / subs, sub-tile c % subs
        const int cb = c / subs, ct = c - cb * subs;
        const int beta = cb == 0 ? first
                                 : (n <= 64 ? __builtin_amdgcn_readlane(sel_mine, cb - 1)
                                            : sel_row[cb - 1]);
        return origin_of(beta) + (uint32_t)(sub_tile_first(g, ct) * (D * 2));
    };

    io.gather(k_rsrc, origin_of_pair(0), k_lds[0]);
    io.gather(v_rsrc, origin_of_pair(0), v_lds[0]);

    // this wavefront's 32 query rows: Q and dO as B operands, lse and delta of
    // the lane's query column
    bf16x8 qf[KS], dof[KS];
    int64_t q_tok;
    {
        const int bw_shift = __builtin_ctz((unsigned)g.block_w);
        const int br = i / g.blocks_per_row, bc = i - br * g.blocks_per_row;
        const int64_t tok0 = (int64_t)br * g.block_h * g.grid_w + (int64_t)bc * g.block_w;
        const int t = 32 * wave + l32;
        const int rr = t >> bw_shift, cc = t & (g.block_w - 1);
        q_tok = tok0 + (int64_t)rr * g.grid_w + cc;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = *(const bf16x8*)(q + base + q_tok * D + 16 * ks + 8 * half);
            dof[ks] = *(const bf16x8*)(dout + base + q_tok * D + 16 * ks + 8 * half);
        }
    }
    const float neg_l2 = -lse2[bh_idx * g.n_tokens + q_tok];
    const float dl = delta[bh_idx * g.n_tokens + q_tok];
    const float c2 = g.scale * kLog2e;

    f32x16 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[dt] = zero_tile();

    if constexpr (D == 64) {
        // Software pipeline over the 32-key halves of the tiles: the
        // exponentials and products that turn S^T, dP^T of one half into dS^T
        // are issued behind the matrix instructions of the next half, two
        // elements per instruction slot, in an order that is written out and
        // pinned (the scheduler would otherwise group them after the matrix
        // instructions, and the two wavefronts of a SIMD do not overlap such
        // phases for each other).  Per tile:
        //   G1  S^T, dP^T of half 0 (8 slots)      | dS^T of the previous half 1
        //   G2  dQ^T += K^T dS^T of the previous half 1 (4 slots),
        //       S^T, dP^T of half 1 (8 slots)      | dS^T of half 0
        //   G3  dQ^T += K^T dS^T of half 0 (4 slots)
        // Carried between tiles: S^T, dP^T of half 1 and its transposed K
        // fragments.  The sums run in the same order as in the plain loop below.
        f32x16 s1, dp1;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s1[r] = -1.0e30f; dp1[r] = 0.0f; }   // weights 0
        bf16x8 ktf[2][2];                                  // [h][dt]
        {
            const bf16x8 z = __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u));
            ktf[0][0] = z; ktf[0][1] = z; ktf[1][0] = z; ktf[1][1] = z;
        }
        // dS^T of elements 2k, 2k+1 of a half, packed
        auto ds_pair = [&](const f32x16& sv, const f32x16& dpv, int k) -> uint32_t {
            const float f0 = fmaf(sv[2 * k], c2, neg_l2), f1 = fmaf(sv[2 * k + 1], c2, neg_l2);
            const float d0 = dpv[2 * k] - dl, d1 = dpv[2 * k + 1] - dl;
            const float e0 = __builtin_amdgcn_exp2f(f0), e1 = __builtin_amdgcn_exp2f(f1);
            return pack_bf16(e0 * d0, e1 * d1);
        };
        // an empty statement that "uses" a slot's result keeps its producers in
        // the slot; no instruction is emitted for it
        auto pin = [](uint32_t& w) {
            asm volatile("" : "+v"(w));
            __builtin_amdgcn_sched_barrier(0);
        };
        for (int c = 0; c < pairs; ++c) {
            // tile c has landed (own loads, then everyone's), every LDS read of
            // the tile before has returned and everyone is done with the other
            // buffer: refill it with tile c + 1
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __syncthreads();
            if (c + 1 < pairs) {
                const uint32_t o = origin_of_pair(c + 1);
                io.gather(k_rsrc, o, k_lds[(c + 1) & 1]);
                io.gather(v_rsrc, o, v_lds[(c + 1) & 1]);
            }
            const unsigned char* kt_lds = k_lds[c & 1];
            const unsigned char* vt_lds = v_lds[c & 1];
            bf16x8 kf[KS], vf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                kf[ks] = row_frag<D>(kt_lds, 0, ks, l32, half);
                vf[ks] = row_frag<D>(vt_lds, 0, ks, l32, half);
            }
            f32x16 s0 = zero_tile(), dp0 = zero_tile();
            uint32_t w[8];
            __builtin_amdgcn_sched_barrier(0);
            // ---- G1
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (k < 4)
                    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[k], qf[k], s0, 0, 0, 0);
                else
                    dp0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[k - 4], dof[k - 4], dp0, 0, 0,
                                                                  0);
                if (k == 3) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) kf[ks] = row_frag<D>(kt_lds, 32, ks, l32, half);
                }
                if (k == 7) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) vf[ks] = row_frag<D>(vt_lds, 32, ks, l32, half);
                }
                w[k] = ds_pair(s1, dp1, k);
                pin(w[k]);
            }
            bf16x8 dsb[2];
            dsb[0] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
            dsb[1] = __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7]));
            // ---- G2
            s1 = zero_tile();
            dp1 = zero_tile();
#pragma unroll
            for (int k = 0; k < 12; ++k) {
                if (k < 4)
                    acc[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf[k >> 1][k & 1],
                                                                         dsb[k >> 1], acc[k & 1],
                                                                         0, 0, 0);
                else if (k < 8)
                    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[k - 4], qf[k - 4], s1, 0, 0, 0);
                else
                    dp1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[k - 8], dof[k - 8], dp1, 0, 0,
                                                                  0);
                if (k == 3) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
                            ktf[h][dt] = trans_frag<D>(kt_lds, 16 * h, dt, lane);
                }
                if (k >= 2 && k < 10) {
                    w[k - 2] = ds_pair(s0, dp0, k - 2);
                    pin(w[k - 2]);
                } else {
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            dsb[0] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
            dsb[1] = __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7]));
            // ---- G3
#pragma unroll
            for (int k = 0; k < 4; ++k)
                acc[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf[k >> 1][k & 1], dsb[k >> 1],
                                                                     acc[k & 1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    ktf[h][dt] = trans_frag<D>(kt_lds, 32 + 16 * h, dt, lane);
        }
        // the last half 1
        {
            uint32_t w[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) w[k] = ds_pair(s1, dp1, k);
            bf16x8 dsb[2];
            dsb[0] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
            dsb[1] = __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7]));
#pragma unroll
            for (int k = 0; k < 4; ++k)
                acc[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf[k >> 1][k & 1], dsb[k >> 1],
                                                                     acc[k & 1], 0, 0, 0);
        }
    } else
    for (int c = 0; c < pairs; ++c) {
        // tile c has landed (own loads, then everyone's) and everyone is done
        // with the other buffer: refill it with tile c + 1
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (c + 1 < pairs) {
            const uint32_t o = origin_of_pair(c + 1);
            io.gather(k_rsrc, o, k_lds[(c + 1) & 1]);
            io.gather(v_rsrc, o, v_lds[(c + 1) & 1]);
        }
        const unsigned char* kt_lds = k_lds[c & 1];
        const unsigned char* vt_lds = v_lds[c & 1];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            f32x16 s = zero_tile(), dp = zero_tile();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    row_frag<D>(kt_lds, 32 * kt, ks, l32, half), qf[ks], s, 0, 0, 0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    row_frag<D>(vt_lds, 32 * kt, ks, l32, half), dof[ks], dp, 0, 0, 0);
            f32x16 ds;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, neg_l2));
                ds[r] = p * (dp[r] - dl);
            }
            bf16x8 dsb[2];
            pack_tile(ds, dsb);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        trans_frag<D>(kt_lds, 32 * kt + 16 * h, dt, lane), dsb[h], acc[dt], 0, 0,
                        0);
        }
    }

    uint16_t* row_ptr = dq + base + q_tok * D;
    const float inv_b = 1.0f / (float)g.block_tokens;
    const float* extra = g.add_dq ? g.add_dq + (bh_idx * g.n_blocks + i) * D : nullptr;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) store_tile(row_ptr, dt, half, acc[dt], g.scale, extra, inv_b);
}

// ---------------------------------------------------------------------------
// dK / dV
// ---------------------------------------------------------------------------
constexpr int PASS_DV = 1, PASS_DK = 2;

template <int D, int NW, int PASS>
__device__ __forceinline__ void dkdv_body(const uint16_t* __restrict__ q,
                                          const uint16_t* __restrict__ k,
                                          const uint16_t* __restrict__ v,
                                          const uint16_t* __restrict__ dout,
                                          const float* __restrict__ lse2,
                                          const float* __restrict__ delta,
                                          const uint32_t* __restrict__ conn,
                                          uint16_t* __restrict__ dk, uint16_t* __restrict__ dv,
                                          const Geom& g, uint32_t n_units)
{
    constexpr int KS = D / 16, DT = D / 32;
    constexpr bool DO_DV = (PASS & PASS_DV) != 0, DO_DK = (PASS & PASS_DK) != 0;
    constexpr int SCAN = 64 * NW;                  // query blocks examined per scan round
    using IO = TileIO<D, NW>;
    __shared__ __attribute__((aligned(1024))) unsigned char q_lds[2][IO::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char g_lds[2][IO::TILE_BYTES];
    __shared__ __attribute__((aligned(256))) float l_lds[2][64];
    __shared__ __attribute__((aligned(256))) float d_lds[2][64];
    __shared__ int list_s[SCAN];
    __shared__ int wave_cnt[NW];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int m = g.n_blocks;
    const int subs = g.block_tokens / 64;
    const int words = (m + 31) >> 5;               // of a key block's row of the connection map

    // workgroup -> (key/value slice, key block), slices dealt to the 8 XCDs
    // whole; the query slices that share the key/value slice are consecutive
    int j;
    int64_t base, bh_first, kv_unit;
    {
        uint32_t unit, r;
        map_unit(blockIdx.x, (uint32_t)m, n_units, unit, r);
        j = (int)r;
        kv_unit = unit;
        base = (int64_t)unit * g.n_tokens * D;
        const uint32_t kv_heads = (uint32_t)(g.heads / g.kv_group);
        const uint32_t e = unit / kv_heads, a = unit - e * kv_heads;
        bh_first = (int64_t)e * g.heads + (int64_t)a * g.kv_group;
    }
    const uint32_t slice_bytes = (uint32_t)(g.n_tokens * D * 2);

    IO io;
    io.init(g, lane, wave);
    auto origin_of = [&](int beta) -> uint32_t {     // byte offset of a block's first token
        const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
        return (uint32_t)((br * g.block_h * g.grid_w + bc * g.block_w) * (D * 2));
    };

    // this wavefront's 32 key rows: K (and V) as B operands
    bf16x8 kfb[KS], vfb[DO_DK ? KS : 1];
    int64_t k_tok;
    {
        const int bw_shift = __builtin_ctz((unsigned)g.block_w);
        const int br = j / g.blocks_per_row, bc = j - br * g.blocks_per_row;
        const int64_t tok0 = (int64_t)br * g.block_h * g.grid_w + (int64_t)bc * g.block_w;
        const int t = 32 * wave + l32;
        const int rr = t >> bw_shift, cc = t & (g.block_w - 1);
        k_tok = tok0 + (int64_t)rr * g.grid_w + cc;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kfb[ks] = *(const bf16x8*)(k + base + k_tok * D + 16 * ks + 8 * half);
            if constexpr (DO_DK)
                vfb[ks] = *(const bf16x8*)(v + base + k_tok * D + 16 * ks + 8 * half);
        }
    }
    const float c2 = g.scale * kLog2e;

    f32x16 acck[DO_DK ? DT : 1], accv[DO_DV ? DT : 1];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        if constexpr (DO_DK) acck[dt] = zero_tile();
        if constexpr (DO_DV) accv[dt] = zero_tile();
    }

    // query heads of the group in ascending order, query blocks in ascending
    // order within each: the summation order is fixed
    for (int gq = 0; gq < g.kv_group; ++gq) {
    const int64_t bh_idx = bh_first + gq;
    const uint32_t* conn_row = conn + (bh_idx * (int64_t)m + j) * words;
    const __amdgpu_buffer_rsrc_t q_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(q + bh_idx * g.n_tokens * D), 0, slice_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t g_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(dout + bh_idx * g.n_tokens * D), 0, slice_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t l_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(lse2 + bh_idx * g.n_tokens), 0, (uint32_t)(g.n_tokens * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t d_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(delta + bh_idx * g.n_tokens), 0, (uint32_t)(g.n_tokens * 4), 0x00020000);

    // items of a round: (connected query block e, sub-tile ct), e-major
    auto issue_item = [&](int item, int buf) {
        const int e = item / subs, ct = item - e * subs;
        const uint32_t o = origin_of(list_s[e]) + (uint32_t)(sub_tile_first(g, ct) * (D * 2));
        io.gather(q_rsrc, o, q_lds[buf]);
        io.gather(g_rsrc, o, g_lds[buf]);
        if (wave == 0) io.gather_f32(l_rsrc, o / (uint32_t)(D * 2), l_lds[buf]);
        if (wave == NW - 1) io.gather_f32(d_rsrc, o / (uint32_t)(D * 2), d_lds[buf]);
    };

    for (int i0 = 0; i0 < m; i0 += SCAN) {
        // ---- which of the query blocks i0 .. i0+SCAN-1 attend to block j?  One
        // bit each in the connection map; ascending order, so the summation
        // order below is fixed
        const int i_mine = i0 + (int)threadIdx.x;
        const bool hit = i_mine < m && ((conn_row[i_mine >> 5] >> (i_mine & 31)) & 1u) != 0;
        const uint64_t mask = __builtin_amdgcn_ballot_w64(hit);
        __syncthreads();                      // previous round's list and tiles fully consumed
        if (lane == 0) wave_cnt[wave] = __builtin_popcountll(mask);
        __syncthreads();
        int offset = 0, total = 0;
        for (int w = 0; w < NW; ++w) {
            if (w < wave) offset += wave_cnt[w];
            total += wave_cnt[w];
        }
        if (hit) list_s[offset + __builtin_popcountll(mask & ((1ull << lane) - 1))] = i_mine;
        __syncthreads();

        const int items = total * subs;
        if (items > 0) issue_item(0, 0);
        for (int it = 0; it < items; ++it) {
            // item `it` has landed and everyone is done with the other buffers
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (it + 1 < items) issue_item(it + 1, (it + 1) & 1);
            const unsigned char* qt_lds = q_lds[it & 1];
            const unsigned char* gt_lds = g_lds[it & 1];
            const float* lt = l_lds[it & 1];
            const float* dtl = d_lds[it & 1];
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                // S = Q K^T: rows = queries 32 qt .., this lane's column = its key
                f32x16 s = zero_tile();
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        row_frag<D>(qt_lds, 32 * qt, ks, l32, half), kfb[ks], s, 0, 0, 0);
                // accumulator element r is query row 8 (r/4) + 4 half + r%4 of the tile
                f32x16 p;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const float4 l4 = *(const float4*)(lt + 32 * qt + 8 * r4 + 4 * half);
                    p[4 * r4 + 0] = __builtin_amdgcn_exp2f(fmaf(s[4 * r4 + 0], c2, -l4.x));
                    p[4 * r4 + 1] = __builtin_amdgcn_exp2f(fmaf(s[4 * r4 + 1], c2, -l4.y));
                    p[4 * r4 + 2] = __builtin_amdgcn_exp2f(fmaf(s[4 * r4 + 2], c2, -l4.z));
                    p[4 * r4 + 3] = __builtin_amdgcn_exp2f(fmaf(s[4 * r4 + 3], c2, -l4.w));
                }
                if constexpr (DO_DV) {
                    bf16x8 pb[2];
                    pack_tile(p, pb);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
                            accv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                trans_frag<D>(gt_lds, 32 * qt + 16 * h, dt, lane), pb[h], accv[dt],
                                0, 0, 0);
                }
                if constexpr (DO_DK) {
                    f32x16 dp = zero_tile();
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            row_frag<D>(gt_lds, 32 * qt, ks, l32, half), vfb[ks], dp, 0, 0, 0);
                    f32x16 ds;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const float4 d4 = *(const float4*)(dtl + 32 * qt + 8 * r4 + 4 * half);
                        ds[4 * r4 + 0] = p[4 * r4 + 0] * (dp[4 * r4 + 0] - d4.x);
                        ds[4 * r4 + 1] = p[4 * r4 + 1] * (dp[4 * r4 + 1] - d4.y);
                        ds[4 * r4 + 2] = p[4 * r4 + 2] * (dp[4 * r4 + 2] - d4.z);
                        ds[4 * r4 + 3] = p[4 * r4 + 3] * (dp[4 * r4 + 3] - d4.w);
                    }
                    bf16x8 dsb[2];
                    pack_tile(ds, dsb);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
                            acck[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                trans_frag<D>(qt_lds, 32 * qt + 16 * h, dt, lane), dsb[h],
                                acck[dt], 0, 0, 0);
                }
            }
        }
    }
    }

    const float inv_b = 1.0f / (float)g.block_tokens;
    const int64_t pooled_row = (kv_unit * m + j) * D;
    const float* extra_k = g.add_dk ? g.add_dk + pooled_row : nullptr;
    const float* extra_v = g.add_dv ? g.add_dv + pooled_row : nullptr;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        if constexpr (DO_DK)
            store_tile(dk + base + k_tok * D, dt, half, acck[dt], g.scale, extra_k, inv_b);
        if constexpr (DO_DV)
            store_tile(dv + base + k_tok * D, dt, half, accv[dt], 1.0f, extra_v, inv_b);
    }
}

}  // namespace bwdm

// delta_l = dO_l . O_l and lse_l * log2(e).  A row (D bf16 = 128 or 256 bytes)
// is read by D/8 adjacent lanes, 16 bytes each, so a wavefront's loads cover
// whole lines; the partial dot products are summed inside the lane group with
// DPP steps.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(
                   __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

template <int D>
__global__ __launch_bounds__(256) void bwd_mfma_prep_kernel(const uint16_t* __restrict__ out,
                                                            const uint16_t* __restrict__ dout,
                                                            const float* __restrict__ lse,
                                                            float* __restrict__ delta,
                                                            float* __restrict__ lse2,
                                                            int64_t rows)
{
    constexpr int LPR = D / 8;                      // lanes per row: 8 or 16
    const int sub = threadIdx.x % LPR;
    int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / LPR;
    const bool valid = row < rows;
    if (!valid) row = rows - 1;                     // keep the lane group whole for the DPP sums
    const uint4 a = *(const uint4*)(out + row * D + 8 * sub);
    const uint4 b = *(const uint4*)(dout + row * D + 8 * sub);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    float acc = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        acc = fmaf(__uint_as_float(aw[e] << 16), __uint_as_float(bw[e] << 16), acc);
        acc = fmaf(__uint_as_float(aw[e] & 0xffff0000u), __uint_as_float(bw[e] & 0xffff0000u),
                   acc);
    }
    acc = dpp_add<0xB1>(acc);                       // quad_perm [1,0,3,2]
    acc = dpp_add<0x4E>(acc);                       // quad_perm [2,3,0,1]
    acc = dpp_add<0x141>(acc);                      // row_half_mirror: 8 lanes
    if (LPR == 16) acc = dpp_add<0x140>(acc);       // row_mirror: 16 lanes
    if (valid && sub == 0) {
        delta[row] = acc;
        lse2[row] = lse[row] * bwdm::kLog2e;
    }
}

// The reverse map of the selection ("the query blocks connected to a key/value
// block", Appendix, kernel design paragraph) as a bit matrix: bit i of row
// [query slice][key block j] says that query block i attends to block j.  One
// thread per (query slice, query block) sets the bits of its row of sel_idx
// (and its own block's, unless only the lists count) with integer atomic ORs:
// the final state does not depend on their order.  A dK/dV workgroup then reads
// its m bits instead of scanning all m * n entries of the slice, and walking
// the set bits upwards is the fixed summation order.
__global__ __launch_bounds__(256) void bwd_connect_clear_kernel(uint32_t* __restrict__ conn,
                                                                int64_t n_words)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n_words) conn[t] = 0u;
}

__global__ __launch_bounds__(256) void bwd_connect_kernel(const int32_t* __restrict__ sel_idx,
                                                          uint32_t* __restrict__ conn, Geom g,
                                                          int64_t rows)
{
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;    // slice * m + i
    if (row >= rows) return;
    const int m = g.n_blocks, n = g.n_select, words = (m + 31) >> 5;
    const int64_t bh_idx = row / m;
    const int i = (int)(row - bh_idx * m);
    uint32_t* base = conn + bh_idx * (int64_t)m * words + (i >> 5);
    const uint32_t bit = 1u << (i & 31);
    if (!g.list_only) atomicOr(base + (int64_t)i * words, bit);
    const int32_t* r = sel_idx + row * n;
    for (int a = 0; a < n; ++a) {
        const int j = r[a];
        if ((unsigned)j < (unsigned)m) atomicOr(base + (int64_t)j * words, bit);
    }
}

// plain kernels per (head dim, wavefronts per workgroup); the bodies are templates
#define BSA_BWD_KERNELS(D, NW)                                                                    \
    __global__ __launch_bounds__(64 * NW, 2) void bwd_mfma_dq_d##D##_w##NW(                       \
        const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* dout,            \
        const float* lse2, const float* delta, const int32_t* sel_idx, uint16_t* dq, Geom g,      \
        uint32_t n_units)                                                                       \
    {                                                                                             \
        bwdm::dq_body<D, NW>(q, k, v, dout, lse2, delta, sel_idx, dq, g, n_units);             \
    }                                                                                             \
    __global__ __launch_bounds__(64 * NW, 2) void bwd_mfma_dv_d##D##_w##NW(                       \
        const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* dout,            \
        const float* lse2, const float* delta, const uint32_t* conn, uint16_t* dk,                \
        uint16_t* dv, Geom g, uint32_t n_units)                                                 \
    {                                                                                             \
        bwdm::dkdv_body<D, NW, bwdm::PASS_DV>(q, k, v, dout, lse2, delta, conn, dk, dv, g,        \
                                              n_units);                                        \
    }                                                                                             \
    __global__ __launch_bounds__(64 * NW, 2) void bwd_mfma_dk_d##D##_w##NW(                       \
        const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* dout,            \
        const float* lse2, const float* delta, const uint32_t* conn, uint16_t* dk,                \
        uint16_t* dv, Geom g, uint32_t n_units)                                                 \
    {                                                                                             \
        bwdm::dkdv_body<D, NW, bwdm::PASS_DK>(q, k, v, dout, lse2, delta, conn, dk, dv, g,        \
                                              n_units);                                        \
    }
BSA_BWD_KERNELS(64, 2)
BSA_BWD_KERNELS(64, 4)
BSA_BWD_KERNELS(64, 8)
// head dim 64: both accumulators fit, dK and dV in one pass
#define BSA_BWD_FUSED(NW)                                                                         \
    __global__ __launch_bounds__(64 * NW, 2) void bwd_mfma_dkdv_d64_w##NW(                        \
        const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* dout,            \
        const float* lse2, const float* delta, const uint32_t* conn, uint16_t* dk,                \
        uint16_t* dv, Geom g, uint32_t n_units)                                                 \
    {                                                                                             \
        bwdm::dkdv_body<64, NW, bwdm::PASS_DV | bwdm::PASS_DK>(q, k, v, dout, lse2, delta,        \
                                                               conn, dk, dv, g, n_units);      \
    }
BSA_BWD_FUSED(2)
BSA_BWD_FUSED(4)
BSA_BWD_FUSED(8)
#undef BSA_BWD_FUSED
BSA_BWD_KERNELS(128, 4)
BSA_BWD_KERNELS(128, 8)
#undef BSA_BWD_KERNELS

bool bwd_mfma_supported(bool is_bf16, const Geom& g, int D)
{
    // a wavefront per 32 rows of a block of 64, 128 or 256 tokens; 64-token
    // sub-tiles (tile width a power of two: whole tile rows, or 64-token runs of
    // one row); 32-bit buffer offsets inside a slice
    // (head dim 128 with 64-token blocks would leave one wavefront per SIMD)
    const int b = g.block_tokens;
    return is_bf16 && (D == 64 || D == 128) && (b == 64 || b == 128 || b == 256) &&
           !(D == 128 && b == 64) &&
           (g.block_w & (g.block_w - 1)) == 0 && g.n_tokens * D * 2 < ((int64_t)1 << 31);
}

hipError_t launch_bwd_mfma(const void* q, const void* k, const void* v, const void* out,
                           const float* lse, const void* dout, const int32_t* sel_idx, void* dq,
                           void* dk, void* dv, float* delta, float* lse2, uint32_t* conn,
                           const Geom& g, int D, int64_t BH, hipStream_t stream)
{
    {
        const int64_t crows = BH * g.n_blocks, n_words = crows * ((g.n_blocks + 31) >> 5);
        bwd_connect_clear_kernel<<<dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, stream>>>(
            conn, n_words);
        bwd_connect_kernel<<<dim3((unsigned)((crows + 255) / 256)), dim3(256), 0, stream>>>(
            sel_idx, conn, g, crows);
        const hipError_t ce = hipGetLastError();
        if (ce != hipSuccess) return ce;
    }
    const int64_t rows = BH * g.n_tokens;
    {
        const int64_t threads = rows * (D / 8);
        const dim3 pgrid((unsigned)((threads + 255) / 256));
        if (D == 64)
            bwd_mfma_prep_kernel<64><<<pgrid, dim3(256), 0, stream>>>(
                (const uint16_t*)out, (const uint16_t*)dout, lse, delta, lse2, rows);
        else
            bwd_mfma_prep_kernel<128><<<pgrid, dim3(256), 0, stream>>>(
                (const uint16_t*)out, (const uint16_t*)dout, lse, delta, lse2, rows);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int nw = g.block_tokens / 32;
    const uint32_t sx = (uint32_t)(BH / g.kv_group);           // key/value slices
    const dim3 grid((unsigned)(BH * g.n_blocks)), grid_kv(sx * (unsigned)g.n_blocks), block(64 * nw);
#define BSA_LAUNCH(D_, NW_)                                                                       \
    if (D == D_ && nw == NW_) {                                                                   \
        bwd_mfma_dq_d##D_##_w##NW_<<<grid, block, 0, stream>>>(                                   \
            (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout,    \
            lse2, delta, sel_idx, (uint16_t*)dq, g, sx);                                          \
        if ((e = hipGetLastError()) != hipSuccess) return e;                                      \
        bwd_mfma_dv_d##D_##_w##NW_<<<grid_kv, block, 0, stream>>>(                                   \
            (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout,    \
            lse2, delta, conn, (uint16_t*)dk, (uint16_t*)dv, g, sx);                              \
        if ((e = hipGetLastError()) != hipSuccess) return e;                                      \
        bwd_mfma_dk_d##D_##_w##NW_<<<grid_kv, block, 0, stream>>>(                                   \
            (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout,    \
            lse2, delta, conn, (uint16_t*)dk, (uint16_t*)dv, g, sx);                              \
        return hipGetLastError();                                                                 \
    }
#define BSA_LAUNCH_FUSED(NW_)                                                                     \
    if (D == 64 && nw == NW_) {                                                                   \
        bwd_mfma_dq_d64_w##NW_<<<grid, block, 0, stream>>>(                                       \
            (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout,    \
            lse2, delta, sel_idx, (uint16_t*)dq, g, sx);                                          \
        if ((e = hipGetLastError()) != hipSuccess) return e;                                      \
        bwd_mfma_dkdv_d64_w##NW_<<<grid_kv, block, 0, stream>>>(                                     \
            (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout,    \
            lse2, delta, conn, (uint16_t*)dk, (uint16_t*)dv, g, sx);                              \
        return hipGetLastError();                                                                 \
    }
    BSA_LAUNCH_FUSED(2)
    BSA_LAUNCH_FUSED(4)
    BSA_LAUNCH_FUSED(8)
#undef BSA_LAUNCH_FUSED
    BSA_LAUNCH(128, 4)
    BSA_LAUNCH(128, 8)
#undef BSA_LAUNCH
    return hipErrorInvalidValue;
}

}  // namespace bsa
