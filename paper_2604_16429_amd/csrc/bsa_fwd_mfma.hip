// Block-sparse attention forward on the gfx950 matrix cores (bf16 MFMA, fp32
// online softmax).  Specialised for head dim 64 and tiles of 64 tokens.
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
// The loads of the next K tile are issued as soon as the current K fragments
// are in registers, and likewise for V, so the gather of pair c+1 overlaps the
// matrix work of pair c; with two such wavefronts per SIMD one wave's softmax
// (vector ALU) overlaps the other's MFMAs.
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

// Gather one 64-token x 64-channel bf16 tile into LDS (8 KiB, rows swizzled).
// Instruction r brings tile rows 8r..8r+7; lane l writes LDS chunk l of that
// 1 KiB slab, i.e. row 8r + l/8, swizzled chunk l%8.
__device__ __forceinline__ void gather_tile(const uint16_t* __restrict__ src_bh, int64_t origin,
                                            const int (&row_off)[8], int chunk_of_lane[8],
                                            unsigned char* lds_tile)
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const uint16_t* src = src_bh + origin + row_off[r] + chunk_of_lane[r];
        __builtin_amdgcn_global_load_lds(src, LDS_PTR(void, lds_tile + r * 1024), 16, 0, 0);
    }
}

__global__ __launch_bounds__(64, 2) void fwd_mfma_b64_d64_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, const int32_t* __restrict__ sel_idx,
    uint16_t* __restrict__ out, float* __restrict__ lse, Geom g)
{
    constexpr int D = 64;
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[64 * 128];
    __shared__ __attribute__((aligned(1024))) unsigned char v_lds[64 * 128];

    const int lane = threadIdx.x;
    const int l32 = lane & 31, half = lane >> 5;
    const int i = (int)(blockIdx.x % g.n_blocks);
    const int64_t bh_idx = blockIdx.x / g.n_blocks;
    const int n = g.n_select;
    const int64_t base = bh_idx * g.n_tokens * D;
    const int32_t* sel_row = sel_idx + (bh_idx * g.n_blocks + i) * n;
    q += base; k += base; v += base; out += base;

    // element offset (inside a block) of the tile row this lane gathers in
    // instruction r, and the global chunk it fetches for its LDS slot
    int row_off[8], chunk_off[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int t = 8 * r + (lane >> 3);
        const int rr = t / g.block_w, cc = t - rr * g.block_w;
        row_off[r] = (rr * g.grid_w + cc) * D;
        chunk_off[r] = swz(t, lane & 7) * 8;          // swizzle is an involution
    }
    auto origin_of = [&](int beta) -> int64_t {
        const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
        return ((int64_t)br * g.block_h * g.grid_w + (int64_t)bc * g.block_w) * D;
    };

    const int64_t origin_q = origin_of(i);
    gather_tile(k, origin_q, row_off, chunk_off, k_lds);
    gather_tile(v, origin_q, row_off, chunk_off, v_lds);

    // Q as B operand of S^T = K Q^T: lane (query l32 + 32 nt, half) holds
    // channels 16 ks + 8 half .. + 7.
    bf16x8 qf[2][4];
    int64_t q_tok[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int t = l32 + 32 * nt;
        const int rr = t / g.block_w, cc = t - rr * g.block_w;
        q_tok[nt] = origin_q / D + (int64_t)rr * g.grid_w + cc;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            qf[nt][ks] = *(const bf16x8*)(q + q_tok[nt] * D + 16 * ks + 8 * half);
    }

    const float c2 = g.scale * 1.4426950408889634f;
    f32x16 oacc[2][2];      // [dt][nt]: O^T tile, rows = channels, cols = queries
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[a][b][r] = 0.0f;
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};

    // LDS byte offsets of this lane's fragment reads
    // K: row = l32 + 32 mt, chunk 2 ks + half
    // V (transposing read): source lane s of 16-lane group gq supplies 8 bytes of
    //   V[key0 + 8 rd + 4 h + s/4][dbase + 4 (s%4)], h = gq/2, dbase = 16 (gq%2) + 32 dt
    const int s16 = lane & 15, gq = lane >> 4;
    const int v_row_in_step = 4 * (gq >> 1) + (s16 >> 2);
    const int v_col = 16 * (gq & 1) + 4 * (s16 & 3);     // channel (before + 32 dt)

    for (int c = 0; c <= n; ++c) {
        const int beta_next = (c < n) ? sel_row[c] : 0;
        const int64_t origin_next = origin_of(beta_next);

        // ---- K(c) has landed: K fragments -> registers
        // (loads complete in order: all but the 8 most recent -- the V(c) gather
        // -- are done)
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        bf16x8 kf[2][4];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int row = l32 + 32 * mt;
                kf[mt][ks] = *(const bf16x8*)(k_lds + row * 128 + swz(row, 2 * ks + half) * 16);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (c < n) gather_tile(k, origin_next, row_off, chunk_off, k_lds);

        // ---- S^T = K Q^T
        f32x16 sacc[2][2];   // [mt][nt]
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[mt][nt][r] = 0.0f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    sacc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        kf[mt][ks], qf[nt][ks], sacc[mt][nt], 0, 0, 0);
            }

        // ---- online softmax, base-2 domain; P^T packed as B operands
        bf16x8 pf[2][4];     // [nt][kk]: keys 16 kk .. 16 kk + 15
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            float mx = sacc[0][nt][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[0][nt][r]);
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[1][nt][r]);
            mx = fmaxf(mx, swap32(mx));
            const float m_new = fmaxf(m_run[nt], mx * c2);
            const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_new);
            m_run[nt] = m_new;
            float rs = 0.0f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8) {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float p0 = __builtin_amdgcn_exp2f(
                            fmaf(sacc[mt][nt][8 * h8 + e], c2, -m_new));
                        const float p1 = __builtin_amdgcn_exp2f(
                            fmaf(sacc[mt][nt][8 * h8 + e + 1], c2, -m_new));
                        rs += p0 + p1;
                        w[e >> 1] = pack_bf16(p0, p1);
                    }
                    const uint4 packed = make_uint4(w[0], w[1], w[2], w[3]);
                    pf[nt][2 * mt + h8] = __builtin_bit_cast(bf16x8, packed);
                }
            l_run[nt] = l_run[nt] * alpha + rs;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
        }

        // ---- V(c) has landed: V^T fragments through the transposing read
        if (c < n) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        bf16x8 vf[2][4];     // [dt][kk]
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                bf16x4 part[2];
#pragma unroll
                for (int rd = 0; rd < 2; ++rd) {
                    const int row = 16 * kk + 8 * rd + v_row_in_step;
                    const int col = v_col + 32 * dt;           // channel, multiple of 4
                    const unsigned char* p =
                        v_lds + row * 128 + swz(row, col >> 3) * 16 + (col & 7) * 2;
                    part[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p));
                }
                vf[dt][kk] = __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (c < n) gather_tile(v, origin_next, row_off, chunk_off, v_lds);

        // ---- O^T += V^T P^T
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    oacc[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        vf[dt][kk], pf[nt][kk], oacc[dt][nt], 0, 0, 0);
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
                (m_run[nt] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}

bool fwd_mfma_supported(bool is_bf16, const Geom& g, int D)
{
    // 16-byte chunks of a token row must not straddle tokens: always true for
    // D = 64 bf16 (128 bytes per token).
    return is_bf16 && D == 64 && g.block_tokens == 64;
}

hipError_t launch_fwd_mfma(const void* q, const void* k, const void* v, const int32_t* sel_idx,
                           void* out, float* lse, const Geom& g, int D, int64_t BH,
                           hipStream_t stream)
{
    (void)D;
    dim3 grid((unsigned)(BH * g.n_blocks));
    hipLaunchKernelGGL(fwd_mfma_b64_d64_kernel, grid, dim3(64), 0, stream, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, sel_idx, (uint16_t*)out, lse, g);
    return hipGetLastError();
}

}  // namespace bsa
