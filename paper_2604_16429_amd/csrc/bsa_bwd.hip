// Block-sparse attention backward with the selection held fixed (gfx950).
//
// With P the attention weights of the forward pass (recomputed from lse),
//   delta_l = sum_d dO_l[d] O_l[d]
//   dV_t    = sum_l P_lt dO_l
//   dP_lt   = dO_l . v_t,   dS_lt = P_lt (dP_lt - delta_l)
//   dQ_l    = scale sum_t dS_lt k_t,   dK_t = scale sum_l dS_lt q_l
// where (l, t) runs over the pairs the forward pass connects: t in the query's
// own block or in one of its selected blocks.  No gradient flows through the
// top-n choice (Appendix, kernel design paragraph: the backward pass walks, for
// every key/value block, the query blocks connected to it).
//
// Three kernels, general in tile shape, head dim (32/64/128) and element type,
// fp32 vector arithmetic throughout:
//   bwd_delta_kernel  delta per query row (workspace, fp32 [B, heads, N]);
//   bwd_dq_kernel     one workgroup per 64 query rows; walks the n+1 attended
//                     blocks like the forward pass;
//   bwd_dkdv_kernel   one workgroup per 64 key rows of a key/value block j; it
//                     first lists, in ascending order, the query blocks i that
//                     attend to j (i == j, or j in sel_idx[i]) by scanning the
//                     selection of its (batch, head), then walks that list.
//                     The order of the list fixes the summation order: results
//                     are reproducible run to run, and there are no
//                     floating-point atomics.
// In the two main kernels four adjacent lanes share a row, each holding a
// quarter of the channels; the two dot products per (query, key) pair are
// completed with two DPP steps inside the quad.
#include "bsa_device.h"
#include "bsa_launch.h"

namespace bsa {

constexpr float kLog2e = 1.4426950408889634f;

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Sum over the four lanes of a quad (all lanes receive the sum).
__device__ __forceinline__ float quad_sum(float x)
{
    x += dpp_f<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_f<0x4E>(x);    // quad_perm [2,3,0,1]
    return x;
}

template <typename T>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const T* __restrict__ out,
                                                        const T* __restrict__ dout,
                                                        float* __restrict__ delta,
                                                        int64_t rows, int D)
{
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const T* o = out + row * D;
    const T* g = dout + row * D;
    float acc = 0.0f;
    for (int d = 0; d < D; d += 4) {
        const float4 a = load4(o + d), b = load4(g + d);
        acc = fmaf(a.x, b.x, acc);
        acc = fmaf(a.y, b.y, acc);
        acc = fmaf(a.z, b.z, acc);
        acc = fmaf(a.w, b.w, acc);
    }
    delta[row] = acc;
}

// Stage `cnt` token rows (tile positions tau0 .. tau0+cnt-1 of block beta) of
// two tensors into LDS as fp32 [cnt][D].
template <typename T, int D>
__device__ __forceinline__ void stage_rows(const Geom& g, const T* __restrict__ a,
                                           const T* __restrict__ b, int64_t base, int beta,
                                           int tau0, int cnt, float* a_s, float* b_s)
{
    for (int item = threadIdx.x; item < cnt * (D / 4); item += blockDim.x) {
        const int t = item / (D / 4), d = (item - t * (D / 4)) * 4;
        const int64_t tok = token_of(g, beta, tau0 + t);
        *(float4*)(a_s + t * D + d) = load4(a + base + tok * D + d);
        *(float4*)(b_s + t * D + d) = load4(b + base + tok * D + d);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dq_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    const T* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ sel_idx, T* __restrict__ dq, Geom g, int row_chunks)
{
    constexpr int CPT = D / 4;                     // channels per lane
    constexpr int KC = 32;                         // keys staged per chunk
    __shared__ __attribute__((aligned(16))) float k_s[KC * D];
    __shared__ __attribute__((aligned(16))) float v_s[KC * D];

    // blockIdx.x = (batch*head * m + block) * row_chunks + chunk
    const int rc = blockIdx.x % row_chunks;
    const int64_t blk = blockIdx.x / row_chunks;
    const int i = (int)(blk % g.n_blocks);
    const int64_t bh_idx = blk / g.n_blocks;
    const int b = g.block_tokens;
    const int quarter = threadIdx.x & 3;
    const int tau_q = rc * 64 + (threadIdx.x >> 2);
    const bool valid = tau_q < b;
    const int64_t base = bh_idx * g.n_tokens * D;
    const int64_t kv_base = kv_slice_of(g, bh_idx) * g.n_tokens * D;
    const int64_t tok_q = token_of(g, i, valid ? tau_q : 0);
    // The attended blocks: block i itself followed by its selected blocks, or,
    // in list-only mode, exactly the listed blocks.
    const int list_only = g.list_only;
    const int32_t* sel_row = sel_idx + (bh_idx * g.n_blocks + i) * g.n_select + list_only;
    const int first = list_only ? sel_row[-1] : i;
    const int n = g.n_select - list_only;        // blocks after the first
    const float c2 = g.scale * kLog2e;

    float qr[CPT], gr[CPT], acc[CPT];
#pragma unroll
    for (int d = 0; d < CPT; d += 4) {
        const float4 a = load4(q + base + tok_q * D + quarter * CPT + d);
        const float4 c = load4(dout + base + tok_q * D + quarter * CPT + d);
        qr[d] = a.x; qr[d + 1] = a.y; qr[d + 2] = a.z; qr[d + 3] = a.w;
        gr[d] = c.x; gr[d + 1] = c.y; gr[d + 2] = c.z; gr[d + 3] = c.w;
        acc[d] = acc[d + 1] = acc[d + 2] = acc[d + 3] = 0.0f;
    }
    const float lse2 = lse[bh_idx * g.n_tokens + tok_q] * kLog2e;
    const float dl = delta[bh_idx * g.n_tokens + tok_q];

    for (int c = 0; c <= n; ++c) {
        const int beta = (c == 0) ? first : sel_row[c - 1];
        for (int k0 = 0; k0 < b; k0 += KC) {
            const int kcnt = min(KC, b - k0);
            __syncthreads();
            stage_rows<T, D>(g, k, v, kv_base, beta, k0, kcnt, k_s, v_s);
            __syncthreads();
            for (int t = 0; t < kcnt; ++t) {
                const float* kr = k_s + t * D + quarter * CPT;
                const float* vr = v_s + t * D + quarter * CPT;
                float s = 0.0f, dp = 0.0f;
#pragma unroll
                for (int d = 0; d < CPT; ++d) {
                    s = fmaf(qr[d], kr[d], s);
                    dp = fmaf(gr[d], vr[d], dp);
                }
                s = quad_sum(s);
                dp = quad_sum(dp);
                const float p = __builtin_amdgcn_exp2f(fmaf(s, c2, -lse2));
                const float ds = p * (dp - dl);
#pragma unroll
                for (int d = 0; d < CPT; ++d) acc[d] = fmaf(ds, kr[d], acc[d]);
            }
        }
    }

    if (valid) {
        const float inv_b = 1.0f / (float)b;
        const float* extra =
            g.add_dq ? g.add_dq + (bh_idx * g.n_blocks + i) * D + quarter * CPT : nullptr;
#pragma unroll
        for (int d = 0; d < CPT; d += 4)
            store4_or_add(dq + base + tok_q * D + quarter * CPT + d,
                          make_float4(acc[d] * g.scale, acc[d + 1] * g.scale, acc[d + 2] * g.scale,
                                      acc[d + 3] * g.scale),
                          extra ? extra + d : nullptr, inv_b);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dkdv_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    const T* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ delta,
    const int32_t* __restrict__ sel_idx, T* __restrict__ dk, T* __restrict__ dv, Geom g,
    int row_chunks)
{
    constexpr int CPT = D / 4;
    constexpr int QC = 32;                         // query rows staged per chunk
    constexpr int SCAN = 256;                      // query blocks examined per scan round
    __shared__ __attribute__((aligned(16))) float q_s[QC * D];
    __shared__ __attribute__((aligned(16))) float g_s[QC * D];
    __shared__ float lse_s[QC], delta_s[QC];
    __shared__ int list_s[SCAN];
    __shared__ int wave_cnt[4];

    const int rc = blockIdx.x % row_chunks;
    const int64_t blk = blockIdx.x / row_chunks;
    const int j = (int)(blk % g.n_blocks);
    const int64_t kv_idx = blk / g.n_blocks;          // key/value slice
    const int b = g.block_tokens, n = g.n_select, m = g.n_blocks;
    const int quarter = threadIdx.x & 3;
    const int tau_k = rc * 64 + (threadIdx.x >> 2);
    const bool valid = tau_k < b;
    const int64_t base = kv_idx * g.n_tokens * D;
    const int64_t tok_k = token_of(g, j, valid ? tau_k : 0);
    // the query slices that share this key/value slice are consecutive
    const int64_t kv_heads = g.heads / g.kv_group;
    const int64_t bh_first = (kv_idx / kv_heads) * g.heads + (kv_idx % kv_heads) * g.kv_group;
    const float c2 = g.scale * kLog2e;

    float kr[CPT], vr[CPT], acck[CPT], accv[CPT];
#pragma unroll
    for (int d = 0; d < CPT; d += 4) {
        const float4 a = load4(k + base + tok_k * D + quarter * CPT + d);
        const float4 c = load4(v + base + tok_k * D + quarter * CPT + d);
        kr[d] = a.x; kr[d + 1] = a.y; kr[d + 2] = a.z; kr[d + 3] = a.w;
        vr[d] = c.x; vr[d + 1] = c.y; vr[d + 2] = c.z; vr[d + 3] = c.w;
        acck[d] = acck[d + 1] = acck[d + 2] = acck[d + 3] = 0.0f;
        accv[d] = accv[d + 1] = accv[d + 2] = accv[d + 3] = 0.0f;
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // query heads in ascending order, then query blocks in ascending order:
    // the summation order is fixed
    for (int gq = 0; gq < g.kv_group; ++gq) {
    const int64_t bh_idx = bh_first + gq;
    const int64_t q_base = bh_idx * g.n_tokens * D;
    const int32_t* sel_bh = sel_idx + bh_idx * (int64_t)m * n;
    for (int i0 = 0; i0 < m; i0 += SCAN) {
        // ---- which of the query blocks i0 .. i0+SCAN-1 attend to block j?
        // ascending order, so the summation order below is fixed
        const int i_mine = i0 + threadIdx.x;
        bool hit = false;
        if (i_mine < m) {
            hit = i_mine == j && !g.list_only;    // list-only mode: the lists say it all
            const int32_t* row = sel_bh + (int64_t)i_mine * n;
            for (int r = 0; r < n; ++r) hit |= row[r] == j;
        }
        const uint64_t mask = __builtin_amdgcn_ballot_w64(hit);
        __syncthreads();                      // previous round's list fully consumed
        if (lane == 0) wave_cnt[wave] = __builtin_popcountll(mask);
        __syncthreads();
        int offset = 0;
        for (int w = 0; w < wave; ++w) offset += wave_cnt[w];
        const int total = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
        if (hit) list_s[offset + __builtin_popcountll(mask & ((1ull << lane) - 1))] = i_mine;
        __syncthreads();

        // ---- walk the connected query blocks
        for (int e = 0; e < total; ++e) {
            const int i = list_s[e];
            for (int r0 = 0; r0 < b; r0 += QC) {
                const int qcnt = min(QC, b - r0);
                __syncthreads();
                stage_rows<T, D>(g, q, dout, q_base, i, r0, qcnt, q_s, g_s);
                if ((int)threadIdx.x < qcnt) {
                    const int64_t tok = token_of(g, i, r0 + threadIdx.x);
                    lse_s[threadIdx.x] = lse[bh_idx * g.n_tokens + tok] * kLog2e;
                    delta_s[threadIdx.x] = delta[bh_idx * g.n_tokens + tok];
                }
                __syncthreads();
                for (int l = 0; l < qcnt; ++l) {
                    const float* qr = q_s + l * D + quarter * CPT;
                    const float* gr = g_s + l * D + quarter * CPT;
                    float s = 0.0f, dp = 0.0f;
#pragma unroll
                    for (int d = 0; d < CPT; ++d) {
                        s = fmaf(kr[d], qr[d], s);
                        dp = fmaf(vr[d], gr[d], dp);
                    }
                    s = quad_sum(s);
                    dp = quad_sum(dp);
                    const float p = __builtin_amdgcn_exp2f(fmaf(s, c2, -lse_s[l]));
                    const float ds = p * (dp - delta_s[l]);
#pragma unroll
                    for (int d = 0; d < CPT; ++d) {
                        accv[d] = fmaf(p, gr[d], accv[d]);
                        acck[d] = fmaf(ds, qr[d], acck[d]);
                    }
                }
            }
        }
    }
    }

    if (valid) {
        const float inv_b = 1.0f / (float)b;
        const int64_t pooled_row = (kv_idx * g.n_blocks + j) * D + quarter * CPT;
        const float* extra_k = g.add_dk ? g.add_dk + pooled_row : nullptr;
        const float* extra_v = g.add_dv ? g.add_dv + pooled_row : nullptr;
#pragma unroll
        for (int d = 0; d < CPT; d += 4) {
            store4_or_add(dk + base + tok_k * D + quarter * CPT + d,
                          make_float4(acck[d] * g.scale, acck[d + 1] * g.scale,
                                      acck[d + 2] * g.scale, acck[d + 3] * g.scale),
                          extra_k ? extra_k + d : nullptr, inv_b);
            store4_or_add(dv + base + tok_k * D + quarter * CPT + d,
                          make_float4(accv[d], accv[d + 1], accv[d + 2], accv[d + 3]),
                          extra_v ? extra_v + d : nullptr, inv_b);
        }
    }
}

template <typename T, int D>
static hipError_t launch_bwd_t(const void* q, const void* k, const void* v, const void* out,
                               const float* lse, const void* dout, const int32_t* sel_idx,
                               void* dq, void* dk, void* dv, float* delta, const Geom& g,
                               int64_t BH, hipStream_t stream)
{
    const int64_t rows = BH * g.n_tokens;
    hipLaunchKernelGGL((bwd_delta_kernel<T>), dim3((unsigned)((rows + 255) / 256)), dim3(256), 0,
                       stream, (const T*)out, (const T*)dout, delta, rows, D);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int row_chunks = (g.block_tokens + 63) / 64;
    dim3 grid((unsigned)(BH * g.n_blocks * row_chunks));
    hipLaunchKernelGGL((bwd_dq_kernel<T, D>), grid, dim3(256), 0, stream, (const T*)q,
                       (const T*)k, (const T*)v, (const T*)dout, lse, delta, sel_idx, (T*)dq, g,
                       row_chunks);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid_kv((unsigned)(BH / g.kv_group * g.n_blocks * row_chunks));
    hipLaunchKernelGGL((bwd_dkdv_kernel<T, D>), grid_kv, dim3(256), 0, stream, (const T*)q,
                       (const T*)k, (const T*)v, (const T*)dout, lse, delta, sel_idx, (T*)dk,
                       (T*)dv, g, row_chunks);
    return hipGetLastError();
}

hipError_t launch_bwd(bool is_bf16, const void* q, const void* k, const void* v, const void* out,
                      const float* lse, const void* dout, const int32_t* sel_idx, void* dq,
                      void* dk, void* dv, float* delta, const Geom& g, int D, int64_t BH,
                      hipStream_t stream)
{
#define BSA_CASE(DD)                                                                             \
    case DD:                                                                                     \
        return is_bf16 ? launch_bwd_t<uint16_t, DD>(q, k, v, out, lse, dout, sel_idx, dq, dk,    \
                                                    dv, delta, g, BH, stream)                    \
                       : launch_bwd_t<float, DD>(q, k, v, out, lse, dout, sel_idx, dq, dk, dv,   \
                                                 delta, g, BH, stream);
    switch (D) {
        BSA_CASE(32)
        BSA_CASE(64)
        BSA_CASE(128)
    }
#undef BSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace bsa
