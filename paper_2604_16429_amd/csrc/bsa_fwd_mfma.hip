// Block-sparse attention forward on the gfx950 matrix cores (bf16 MFMA, fp32
// online softmax).  Specialised for head dim 64 and tiles of 64*T tokens whose
// width divides 64; a tile is processed as T sub-blocks of 64 queries (one
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
// Order of work for pair c (K(c) fragments are already in registers):
//   1. S^T = K(c) Q^T, 16 MFMAs, with the 8 loads of the K(c+1) gather issued
//      between them (the K tile in LDS is free: its fragments are in registers);
//   2. the weights P(c) on the vector ALU; half-way, the V(c) fragments are
//      requested from LDS;
//   3. the K(c+1) fragments are requested from LDS;
//   4. O^T += V(c)^T P(c)^T, 16 MFMAs, with the 8 loads of the V(c+1) gather
//      issued between them.
// A gather issued in one burst would hold the wavefront at the CU's shared
// address unit for hundreds of cycles; spread over a run of MFMAs, whose issue
// is paced by the matrix pipe anyway, it costs nothing.  Two wavefronts per
// SIMD overlap one wave's MFMA runs with the other's exponentials.
//
// Softmax without a row maximum per pair.  m_ref is the reference the
// exponentials are taken against.  A pair first computes its weights against
// the current m_ref; only if some row sum of the pair exceeds 2^12 (which
// covers the first pair, where m_ref = -inf) does the wavefront take the slow
// path: find the row maxima, move m_ref, rescale O and the normaliser, and
// recompute the pair's weights.  Any reference gives the same softmax; bounded
// weights keep fp32 and bf16 far from overflow.
#include "bsa_device.h"
#include "bsa_launch.h"

namespace bsa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// 16-byte chunk swizzle of a 128-byte LDS row (8 chunks per row).
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// Exchange with the lane 32 away (lanes l < 32 get the value of l + 32 and
// vice versa).
__device__ __forceinline__ float swap32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false,
                                                    false);
    // r[0] holds, for lanes < 32, their own value and for lanes >= 32 the value
    // of lane - 32; r[1] the opposite halves.
    return __uint_as_float(threadIdx.x & 32 ? r[0] : r[1]);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    const f32x2 v = {a, b};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// Gather one 64-token x 64-channel bf16 tile into LDS (8 KiB, rows swizzled)
// with buffer loads that write LDS directly.  Instruction r brings tile rows
// 8r..8r+7; lane l fills LDS chunk l of that 1 KiB slab, i.e. row 8r + l/8,
// swizzled chunk l%8.  The per-lane byte offsets inside a block (voff) are
// fixed for the whole kernel and the block origin is wave-uniform (soffset),
// so a gather costs no vector ALU work.  The buffer descriptor bounds the
// slice: an out-of-range block index reads zeros instead of faulting.
__device__ __forceinline__ void gather_tile(__amdgpu_buffer_rsrc_t rsrc, uint32_t origin_bytes,
                                            const uint32_t (&voff)[8], unsigned char* lds_tile)
{
#pragma unroll
    for (int r = 0; r < 8; ++r)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(void, lds_tile + r * 1024), 16,
                                                 voff[r], origin_bytes, 0, 0);
}

// P^T = exp2(S^T c2 - m_ref) for one query half nt, packed to bf16 B operands;
// returns this lane's sum of the rounded weights (two per instruction).  Only
// builtins touch the MFMA results (never inline asm): the compiler must see
// these reads to place the wait states the hardware requires.
__device__ __forceinline__ float softmax_weights(const f32x16 (&s)[2][2], int nt, float c2,
                                                 float neg_m, bf16x8 (&pf)[2][4])
{
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
    float rs = 0.0f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int h8 = 0; h8 < 2; ++h8) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s[mt][nt][8 * h8 + e], c2, neg_m));
                const float p1 =
                    __builtin_amdgcn_exp2f(fmaf(s[mt][nt][8 * h8 + e + 1], c2, neg_m));
                w[e >> 1] = pack_bf16(p0, p1);
                rs = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e >> 1]), ones,
                                                     rs, false);
            }
            const uint4 packed = make_uint4(w[0], w[1], w[2], w[3]);
            pf[nt][2 * mt + h8] = __builtin_bit_cast(bf16x8, packed);
        }
    return rs;
}

constexpr float kSumLimit = 4096.0f;

__global__ __launch_bounds__(64, 2) void fwd_mfma_b64_d64_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const int32_t* __restrict__ sel_idx,
    uint16_t* __restrict__ out, float* __restrict__ lse, Geom g, int64_t slices_xcd, int subs)
{
    constexpr int D = 64;
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[64 * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds[64 * 128];
    __shared__ int order_s[64];

    const int lane = threadIdx.x;
    const int l32 = lane & 31, half = lane >> 5;
    const int n = g.n_select;

    // Work item -> (batch*head slice, query block).  Workgroups are handed to
    // the 8 XCDs round-robin by id; each XCD has its own L2.  Slices are dealt
    // to XCDs whole (slice s runs on XCD s % 8, its query blocks back to back),
    // so the K/V tiles a slice's query blocks share are fetched into one L2
    // instead of eight.  The last BH % 8 slices use the plain linear order.
    // A work item is one sub-block of 64 queries: item = block * subs + sub.
    int i, qsub;
    int64_t bh_idx;
    {
        const int64_t w = blockIdx.x;
        const int64_t per_slice = (int64_t)g.n_blocks * subs;
        int64_t item;
        if (w < slices_xcd * per_slice) {
            const int64_t seq = w >> 3;
            bh_idx = (seq / per_slice) * 8 + (w & 7);
            item = seq % per_slice;
        } else {
            bh_idx = w / per_slice;
            item = w % per_slice;
        }
        i = (int)(item / subs);
        qsub = (int)(item - (int64_t)i * subs);
    }
    // byte distance between consecutive 64-token sub-tiles of a block: 64/bw
    // grid rows (the tile width divides 64)
    const uint32_t sub_stride = (uint32_t)((64 / g.block_w) * g.grid_w * (D * 2));
    const int64_t base = bh_idx * g.n_tokens * D;
    const int32_t* sel_row = sel_idx + (bh_idx * g.n_blocks + i) * n;
    q += base; out += base;
    const uint32_t slice_bytes = (uint32_t)(g.n_tokens * D * 2);
    const __amdgpu_buffer_rsrc_t k_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(k + base), 0, slice_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(v + base), 0, slice_bytes, 0x00020000);
    // zero records: every access is out of range, the load moves nothing
    const __amdgpu_buffer_rsrc_t null_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(k + base), 0, 0, 0x00020000);

    // Visiting order: the own block first (it needs nothing from sel_idx, so
    // its gathers start at once), then the selected blocks in ascending block
    // order when they fit one wavefront: query blocks that run at the same time
    // on an XCD then sweep the slice's K/V in the same direction and find each
    // other's tiles in L2.  The result does not depend on the order (up to
    // rounding).  The order is computed after the first gathers are in flight;
    // order_v: lane c holds the c-th block to visit.
    const bool sorted = n + 1 <= 64;
    int order_v = i;
    auto block_at = [&](int c) -> int {
        if (c == 0) return i;
        if (sorted) return __builtin_amdgcn_readlane(order_v, c);
        return sel_row[c - 1];
    };

    // byte offset (inside a block) of the 16-byte chunk this lane gathers in
    // instruction r: tile row 8r + lane/8, global chunk = swizzle of its LDS slot
    uint32_t voff[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int t = 8 * r + (lane >> 3);
        const int rr = t / g.block_w, cc = t - rr * g.block_w;
        voff[r] = (uint32_t)(((rr * g.grid_w + cc) * D + swz(t, lane & 7) * 8) * 2);
    }
    auto origin_of = [&](int beta) -> uint32_t {     // byte offset of a block's first token
        const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
        return (uint32_t)((br * g.block_h * g.grid_w + bc * g.block_w) * (D * 2));
    };

    // K(0) and V(0) go to LDS
    {
        const uint32_t origin_0 = origin_of(block_at(0));
        gather_tile(k_rsrc, origin_0, voff, k_lds);
        gather_tile(v_rsrc, origin_0, voff, v_lds);
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
            const int rr = t / g.block_w, cc = t - rr * g.block_w;
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
        if (lane >= 1 && lane <= n) order_s[rank] = mine;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        order_v = order_s[lane];
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

    auto read_k_frags = [&](bf16x8 (&kf)[2][4]) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int row = l32 + 32 * mt;
                kf[mt][ks] = *(const bf16x8*)(k_lds + row * 128 + swz(row, 2 * ks + half) * 16);
            }
    };

    // K(0) has landed: loads complete in order, and K(0) is older than the loads
    // of V(0) and Q and of the selection row (8 + 8 + 1)
    bf16x8 kf[2][4];
    asm volatile("s_waitcnt vmcnt(17)" ::: "memory");
    read_k_frags(kf);

    // pairs: attended block cb = 0..n (visiting order), key sub-tile ct = 0..subs-1
    int cb = 0, ct = 0;
    const int pairs = (n + 1) * subs;
    for (int c = 0; c < pairs; ++c) {
        const bool has_next = c + 1 < pairs;
        if (++ct == subs) { ct = 0; ++cb; }           // (cb, ct) now names pair c+1
        const uint32_t origin_next =
            origin_of(block_at(has_next ? cb : n)) + (has_next ? ct : 0) * sub_stride;
        const __amdgpu_buffer_rsrc_t k_next = has_next ? k_rsrc : null_rsrc;
        const __amdgpu_buffer_rsrc_t v_next = has_next ? v_rsrc : null_rsrc;

        // ---- 1. S^T = K(c) Q^T, with the K(c+1) gather between the MFMAs (the
        // K fragments are in registers, so the K tile may be overwritten)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        f32x16 sacc[2][2];   // [mt][nt]
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    sacc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        kf[mt][ks], qf[nt][ks], ks == 0 ? zero16 : sacc[mt][nt], 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    k_next, LDS_PTR(void, k_lds + (2 * ks + nt) * 1024), 16, voff[2 * ks + nt],
                    origin_next, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }

        // ---- 2. P^T = exp2(S^T c2 - m_ref) against the current reference, one
        // query half at a time; the slow path finds a new reference from the
        // row maxima, rescales O and the normaliser and recomputes the weights
        bf16x8 pf[2][4];     // [nt][kk]: keys 16 kk .. 16 kk + 15
        bf16x8 vf[2][4];     // [dt][kk]
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            float rs = softmax_weights(sacc, nt, c2, -m_ref[nt], pf);
            if (__builtin_amdgcn_ballot_w64(!(rs <= kSumLimit)) != 0) {
                float mx = sacc[0][nt][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[0][nt][r]);
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[1][nt][r]);
                mx = fmaxf(mx, swap32(mx));
                const float m_new = fmaxf(m_ref[nt], mx * c2);
                const float alpha = __builtin_amdgcn_exp2f(m_ref[nt] - m_new);
                m_ref[nt] = m_new;
                l_run[nt] *= alpha;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
                rs = softmax_weights(sacc, nt, c2, -m_new, pf);
            }
            l_run[nt] += rs;

            if (nt == 0) {
                // V(c) has landed (it is older than the 8 loads of the K(c+1)
                // gather): request its fragments now that half of S is dead;
                // they arrive while the other half's weights are computed
                asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        bf16x4 part[2];
#pragma unroll
                        for (int rd = 0; rd < 2; ++rd) {
                            const int row = 16 * kk + 8 * rd + v_row_in_step;
                            const int col = v_col + 32 * dt;   // channel, multiple of 4
                            const unsigned char* p =
                                v_lds + row * 128 + swz(row, col >> 3) * 16 + (col & 7) * 2;
                            part[rd] =
                                __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                        }
                        vf[dt][kk] =
                            __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
                    }
            }
        }

        // ---- 3. K(c+1) has landed (nothing younger is in flight): request its
        // fragments; they arrive during the PV product
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        if (has_next) read_k_frags(kf);

        // ---- 4. O^T += V^T P^T, with the V(c+1) gather between the MFMAs (the
        // V fragments are in registers, so the V tile may be overwritten)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    oacc[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        vf[dt][kk], pf[nt][kk], oacc[dt][nt], 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    v_next, LDS_PTR(void, v_lds + (2 * kk + nt) * 1024), 16, voff[2 * kk + nt],
                    origin_next, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
    }

    // ---- epilogue: normalise, store O rows (4 consecutive channels per store)
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

bool fwd_mfma_supported(bool is_bf16, const Geom& g, int D)
{
    // tiles of 64*T tokens whose width divides 64: every 64-token sub-tile is
    // then a whole number of tile rows, a fixed byte distance apart
    // (a token row is 128 bytes, so 16-byte chunks never straddle tokens);
    // buffer offsets inside a slice are 32-bit
    return is_bf16 && D == 64 && g.block_tokens % 64 == 0 && 64 % g.block_w == 0 &&
           g.n_tokens * D * 2 < ((int64_t)1 << 31);
}

hipError_t launch_fwd_mfma(const void* q, const void* k, const void* v, const int32_t* sel_idx,
                           void* out, float* lse, const Geom& g, int D, int64_t BH,
                           hipStream_t stream)
{
    (void)D;
    const int subs = g.block_tokens / 64;
    dim3 grid((unsigned)(BH * g.n_blocks * subs));
    hipLaunchKernelGGL(fwd_mfma_b64_d64_kernel, grid, dim3(64), 0, stream, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, sel_idx, (uint16_t*)out, lse, g,
                       BH - BH % 8, subs);
    return hipGetLastError();
}

}  // namespace bsa
