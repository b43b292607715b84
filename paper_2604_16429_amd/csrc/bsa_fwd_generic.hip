// Block-sparse attention forward, general-shape kernel (gfx950).
//
// Every token of query block i attends, in one softmax, to the tokens of block
// i and of its n selected blocks (fine-grained attention equation plus the
// local block).  This kernel covers every tile shape, head dim in
// {32, 64, 128} and both element types with plain fp32 vector arithmetic; the
// bf16 MFMA kernels take over the shapes they are specialised for.
//
// One wavefront per 64 query rows of a block, one lane per row.  The lane keeps
// its query row and its output accumulator in registers.  Keys and values are
// staged through LDS in chunks of KC tokens (cooperative, channel-contiguous
// loads); all lanes then read the same LDS address at the same time (a
// broadcast, free of bank conflicts).  Softmax is the online form, updated
// once per chunk, in the base-2 domain.
#include "bsa_device.h"
#include "bsa_launch.h"

namespace bsa {

template <typename T, int D>
__global__ __launch_bounds__(64) void fwd_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    const int32_t* __restrict__ sel_idx, T* __restrict__ out, float* __restrict__ lse, Geom g,
    int row_chunks)
{
    constexpr int KC = 32;                         // keys staged per chunk
    __shared__ __attribute__((aligned(16))) float k_s[KC * D];
    __shared__ __attribute__((aligned(16))) float v_s[KC * D];

    // blockIdx.x = (batch*head * m + block) * row_chunks + chunk
    const int rc = blockIdx.x % row_chunks;
    const int64_t blk = blockIdx.x / row_chunks;
    const int i = (int)(blk % g.n_blocks);
    const int64_t bh_idx = blk / g.n_blocks;
    const int b = g.block_tokens;
    const int tau_q = rc * 64 + threadIdx.x;
    const bool valid = tau_q < b;
    const int64_t base = bh_idx * g.n_tokens * D;
    const int64_t kv_base = kv_slice_of(g, bh_idx) * g.n_tokens * D;
    const int64_t tok_q = token_of(g, i, valid ? tau_q : 0);
    // The attended blocks: block i itself followed by its selected blocks, or,
    // when the selection branch runs on its own, exactly the listed blocks.
    const int list_only = g.list_only;
    const int32_t* sel_row = sel_idx + (bh_idx * g.n_blocks + i) * g.n_select + list_only;
    const int first = list_only ? sel_row[-1] : i;
    const int n = g.n_select - list_only;        // blocks after the first
    const float scale2 = g.scale * 1.4426950408889634f;   // to base-2 exponent

    float qr[D], acc[D];
#pragma unroll
    for (int d = 0; d < D; d += 4) {
        const float4 t = load4(q + base + tok_q * D + d);
        qr[d] = t.x * scale2; qr[d + 1] = t.y * scale2;
        qr[d + 2] = t.z * scale2; qr[d + 3] = t.w * scale2;
        acc[d] = acc[d + 1] = acc[d + 2] = acc[d + 3] = 0.0f;
    }
    float m_run = -INFINITY, l_run = 0.0f;

    for (int c = 0; c <= n; ++c) {
        const int beta = (c == 0) ? first : sel_row[c - 1];
        for (int k0 = 0; k0 < b; k0 += KC) {
            const int kcnt = min(KC, b - k0);
            __syncthreads();
            for (int item = threadIdx.x; item < kcnt * (D / 4); item += 64) {
                const int t = item / (D / 4), d = (item - t * (D / 4)) * 4;
                const int64_t tok = token_of(g, beta, k0 + t);
                *(float4*)(k_s + t * D + d) = load4(k + kv_base + tok * D + d);
                *(float4*)(v_s + t * D + d) = load4(v + kv_base + tok * D + d);
            }
            __syncthreads();

            float s[KC];
            float m_new = m_run;
#pragma unroll
            for (int t = 0; t < KC; ++t) {
                float dot = 0.0f;
                if (t < kcnt) {
                    const float4* kr = (const float4*)(k_s + t * D);
#pragma unroll
                    for (int d4 = 0; d4 < D / 4; ++d4) {
                        const float4 kv = kr[d4];
                        dot = fmaf(qr[4 * d4], kv.x, dot);
                        dot = fmaf(qr[4 * d4 + 1], kv.y, dot);
                        dot = fmaf(qr[4 * d4 + 2], kv.z, dot);
                        dot = fmaf(qr[4 * d4 + 3], kv.w, dot);
                    }
                    m_new = fmaxf(m_new, dot);
                }
                s[t] = dot;
            }
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);   // exp2(-inf) = 0
            m_run = m_new;
            l_run *= corr;
#pragma unroll
            for (int d = 0; d < D; ++d) acc[d] *= corr;
#pragma unroll
            for (int t = 0; t < KC; ++t) {
                if (t < kcnt) {
                    const float p = __builtin_amdgcn_exp2f(s[t] - m_new);
                    l_run += p;
                    const float4* vr = (const float4*)(v_s + t * D);
#pragma unroll
                    for (int d4 = 0; d4 < D / 4; ++d4) {
                        const float4 vv = vr[d4];
                        acc[4 * d4] = fmaf(p, vv.x, acc[4 * d4]);
                        acc[4 * d4 + 1] = fmaf(p, vv.y, acc[4 * d4 + 1]);
                        acc[4 * d4 + 2] = fmaf(p, vv.z, acc[4 * d4 + 2]);
                        acc[4 * d4 + 3] = fmaf(p, vv.w, acc[4 * d4 + 3]);
                    }
                }
            }
        }
    }

    if (valid) {
        const float inv_l = 1.0f / l_run;
#pragma unroll
        for (int d = 0; d < D; d += 4)
            store4(out + base + tok_q * D + d,
                   make_float4(acc[d] * inv_l, acc[d + 1] * inv_l, acc[d + 2] * inv_l,
                               acc[d + 3] * inv_l));
        if (lse)
            lse[bh_idx * g.n_tokens + tok_q] =
                (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
    }
}

template <typename T, int D>
static hipError_t launch_t(const void* q, const void* k, const void* v, const int32_t* sel_idx,
                           void* out, float* lse, const Geom& g, int64_t BH, hipStream_t stream)
{
    const int row_chunks = (g.block_tokens + 63) / 64;
    dim3 grid((unsigned)(BH * g.n_blocks * row_chunks));
    hipLaunchKernelGGL((fwd_generic_kernel<T, D>), grid, dim3(64), 0, stream, (const T*)q,
                       (const T*)k, (const T*)v, sel_idx, (T*)out, lse, g, row_chunks);
    return hipGetLastError();
}

hipError_t launch_fwd_generic(bool is_bf16, const void* q, const void* k, const void* v,
                              const int32_t* sel_idx, void* out, float* lse, const Geom& g, int D,
                              int64_t BH, hipStream_t stream)
{
#define BSA_CASE(DD)                                                                          \
    case DD:                                                                                  \
        return is_bf16 ? launch_t<uint16_t, DD>(q, k, v, sel_idx, out, lse, g, BH, stream)    \
                       : launch_t<float, DD>(q, k, v, sel_idx, out, lse, g, BH, stream);
    switch (D) {
        BSA_CASE(32)
        BSA_CASE(64)
        BSA_CASE(128)
    }
#undef BSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace bsa
