// The pieces of the paper's three-branch output that the single-softmax path
// does not already have (gfx950):
//
//   coarse_kernel        coarse-grained branch: for query block i the softmax
//                        over ALL m key blocks of qbar_i . kbar_j / sqrt(d_k)
//                        (block-level attention equation) applied to the
//                        mean-pooled values (coarse-grained output equation);
//                        one fp32 row [D] per query block.
//   local_lists_kernel   the other mesh tiles of the large local block that
//                        contains tile i (Local Attention paragraph); the
//                        local branch is then the forward kernel run on "tile
//                        i and these tiles".
//   combine_kernel       o = g_cg * o_cg(block of the token) + g_fg * o_fg +
//                        g_l * o_l with caller-supplied gate values
//                        (aggregation equation of the Native Sparse Attention
//                        subsection).  HBM-bound, one pass.
//
// The selection branch itself is the forward kernel in its list-only mode.
#include "bsa_device.h"
#include "bsa_launch.h"

namespace bsa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kCoarseRows = 8;                      // most query blocks per workgroup
constexpr size_t kCoarseLdsBudget = 144 * 1024;

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

}  // namespace

// One workgroup of 256 threads handles G <= 8 consecutive query blocks of one
// (batch, head).
//   phase 1: thread t owns key block j = chunk*256 + t, holds kbar_j in
//            registers and scores it against the G pooled queries (scalar
//            operands); scaled scores (base-2 domain) land in LDS.
//   phase 2: one wavefront per query block: row maximum, weights
//            exp2(s - max) written back in place, 1 / row sum.
//   phase 3: thread = (channel quad, key partition): walks the pooled values
//            of its key partition (a row of vbar is read by D/4 adjacent
//            lanes, 16 bytes each) and accumulates weight * value for all G
//            rows in registers.
//   phase 4: the partitions' partial rows are summed, first inside each
//            wavefront (lanes with the same channel quad), then through LDS,
//            in fixed order, and scaled by 1 / row sum.
// LDS: G*m (scores) + 4*G*D (partials) + G floats.
template <int D>
__global__ __launch_bounds__(256) void coarse_kernel(const float* __restrict__ qbar,
                                                     const float* __restrict__ kbar,
                                                     const float* __restrict__ kbar_il,
                                                     const float* __restrict__ vbar,
                                                     float* __restrict__ obar, Geom g, int G)
{
    constexpr int CG = D / 4;                        // channel quads
    constexpr int JP = 256 / CG;                     // key partitions
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int m = g.n_blocks;
    float* red_s = (float*)smem;                     // [4 wavefronts][G][D]
    float* inv_s = red_s + 4 * G * D;                // [8]
    float* sc_s = inv_s + kCoarseRows;               // [G][m]

    const int groups = (m + G - 1) / G;
    const int64_t bh_idx = blockIdx.x / groups;
    const int i0 = (int)(blockIdx.x - bh_idx * groups) * G;
    const int rows = min(G, m - i0);
    const int64_t kv = kv_slice_of(g, bh_idx);
    qbar += (bh_idx * m + i0) * D;
    kbar += kv * m * D;
    vbar += kv * m * D;

    if (kbar_il) kbar_il += kv * m * D;              // per slice [D/4][m][4]

    // ---- phase 1: scaled scores.  The pooled queries are wave-uniform (scalar
    // loads, scalar operands of the fma); the thread's pooled key comes from the
    // channel-interleaved copy where there is one (coalesced), else from its row.
    const float c2 = g.scale * kLog2e;
    for (int j = threadIdx.x; j < m; j += blockDim.x) {
        float kr[D];
        const float4* ksrc = kbar_il ? (const float4*)kbar_il + j
                                     : (const float4*)(kbar + (int64_t)j * D);
        const int64_t kstep = kbar_il ? (int64_t)m : 1;
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const float4 t = ksrc[d4 * kstep];
            kr[4 * d4 + 0] = t.x; kr[4 * d4 + 1] = t.y;
            kr[4 * d4 + 2] = t.z; kr[4 * d4 + 3] = t.w;
        }
        for (int r = 0; r < rows; ++r) {
            const float* __restrict__ qrow = qbar + r * D;
            float acc = 0.0f;
#pragma unroll
            for (int d = 0; d < D; ++d) acc = fmaf(qrow[d], kr[d], acc);
            sc_s[r * m + j] = acc * c2;
        }
    }
    __syncthreads();

    // ---- phase 2: softmax weights per row, one wavefront each
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < rows; r += 4) {
        float* row = sc_s + r * m;
        float mx = -INFINITY;
        for (int j = lane; j < m; j += 64) mx = fmaxf(mx, row[j]);
        mx = wave_max(mx);
        float sum = 0.0f;
        for (int j = lane; j < m; j += 64) {
            const float w = __builtin_amdgcn_exp2f(row[j] - mx);
            row[j] = w;
            sum += w;
        }
        sum = wave_sum(sum);
        if (lane == 0) inv_s[r] = 1.0f / sum;
    }
    __syncthreads();

    // ---- phase 3: weights times pooled values
    const int cg = threadIdx.x % CG, jp = threadIdx.x / CG;
    float4 acc[kCoarseRows];
#pragma unroll
    for (int r = 0; r < kCoarseRows; ++r) acc[r] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int j = jp; j < m; j += JP) {
        const float4 val = *(const float4*)(vbar + (int64_t)j * D + 4 * cg);
#pragma unroll
        for (int r = 0; r < kCoarseRows; ++r) {
            if (r < rows) {
                const float w = sc_s[r * m + j];
                acc[r].x = fmaf(w, val.x, acc[r].x);
                acc[r].y = fmaf(w, val.y, acc[r].y);
                acc[r].z = fmaf(w, val.z, acc[r].z);
                acc[r].w = fmaf(w, val.w, acc[r].w);
            }
        }
    }
    // ---- phase 4: the 64 / CG partitions of a wavefront hold the same channel
    // quad CG lanes apart: butterfly sums, then one partial row per wavefront
#pragma unroll
    for (int r = 0; r < kCoarseRows; ++r)
        for (int off = CG; off < 64; off <<= 1) {
            acc[r].x += __shfl_xor(acc[r].x, off);
            acc[r].y += __shfl_xor(acc[r].y, off);
            acc[r].z += __shfl_xor(acc[r].z, off);
            acc[r].w += __shfl_xor(acc[r].w, off);
        }
    if (lane < CG) {
#pragma unroll
        for (int r = 0; r < kCoarseRows; ++r)
            if (r < rows) *(float4*)(red_s + ((wave * G + r) * D) + 4 * cg) = acc[r];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < rows * D; e += blockDim.x) {
        const int r = e / D, d = e - r * D;
        float sum = 0.0f;
        for (int p = 0; p < 4; ++p) sum += red_s[(p * G + r) * D + d];
        obar[(bh_idx * m + i0 + r) * D + d] = sum * inv_s[r];
    }
}

static size_t coarse_lds_bytes(int G, int m, int D)
{
    return ((size_t)4 * G * D + kCoarseRows + (size_t)G * m) * 4;
}

int coarse_group_size(int m, int D)
{
    for (int G = kCoarseRows; G >= 1; G >>= 1)
        if (coarse_lds_bytes(G, m, D) <= kCoarseLdsBudget) return G;
    return 0;
}

template <int D>
static hipError_t launch_coarse_t(const float* qbar, const float* kbar, const float* kbar_il,
                                  const float* vbar, float* obar, const Geom& g, int64_t BH,
                                  hipStream_t stream)
{
    const int G = coarse_group_size(g.n_blocks, D);
    if (G == 0) return hipErrorInvalidValue;
    // the attribute is per device; setting it twice (two host threads racing) is harmless
    static bool attr_set[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute((const void*)coarse_kernel<D>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kCoarseLdsBudget);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    dim3 grid((unsigned)(BH * ((g.n_blocks + G - 1) / G)));
    hipLaunchKernelGGL((coarse_kernel<D>), grid, dim3(256), coarse_lds_bytes(G, g.n_blocks, D),
                       stream, qbar, kbar, kbar_il, vbar, obar, g, G);
    return hipGetLastError();
}

hipError_t launch_coarse(const float* qbar, const float* kbar, const float* kbar_il,
                         const float* vbar, float* obar, const Geom& g, int D, int64_t BH,
                         hipStream_t stream)
{
    switch (D) {
    case 32: return launch_coarse_t<32>(qbar, kbar, kbar_il, vbar, obar, g, BH, stream);
    case 64: return launch_coarse_t<64>(qbar, kbar, kbar_il, vbar, obar, g, BH, stream);
    case 128: return launch_coarse_t<128>(qbar, kbar, kbar_il, vbar, obar, g, BH, stream);
    }
    return hipErrorInvalidValue;
}

// lists[bh, i, c], c = 0 .. local_h*local_w - 2: the other tiles of the aligned
// group of local_h x local_w tiles that contains tile i, ascending.
__global__ __launch_bounds__(256) void local_lists_kernel(int32_t* __restrict__ lists, Geom g,
                                                          int local_h, int local_w,
                                                          int64_t total)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int nl = local_h * local_w - 1;
    const int c = (int)(e % nl);
    const int i = (int)((e / nl) % g.n_blocks);
    const int r = i / g.blocks_per_row, col = i - r * g.blocks_per_row;
    const int r0 = r - r % local_h, c0 = col - col % local_w;
    const int own = (r - r0) * local_w + (col - c0);    // position of tile i in its group
    const int pos = c < own ? c : c + 1;
    lists[e] = (r0 + pos / local_w) * g.blocks_per_row + c0 + pos % local_w;
}

hipError_t launch_local_lists(int32_t* lists, const Geom& g, int local_h, int local_w,
                              int64_t BH, hipStream_t stream)
{
    const int64_t total = BH * g.n_blocks * (local_h * local_w - 1);
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(local_lists_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       stream, lists, g, local_h, local_w, total);
    return hipGetLastError();
}

// One thread per VEC consecutive channels of one token.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ obar,
                                                      const T* __restrict__ o_fg,
                                                      const T* __restrict__ o_l,
                                                      const float* __restrict__ gates,
                                                      T* __restrict__ out, Geom g, int D,
                                                      int64_t total)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int per_row = D / VEC;
    const int64_t row = e / per_row;                 // bh * N + token
    const int ch = (int)(e - row * per_row) * VEC;
    const int64_t bh = row / g.n_tokens;
    const int64_t tok = row - bh * g.n_tokens;
    const int gr = (int)(tok / g.grid_w), gc = (int)(tok - (int64_t)gr * g.grid_w);
    const int beta = (gr / g.block_h) * g.blocks_per_row + gc / g.block_w;
    const float g_cg = gates[row * 3 + 0], g_fg = gates[row * 3 + 1], g_l = gates[row * 3 + 2];
    const float* ob = obar + (bh * g.n_blocks + beta) * D + ch;
#pragma unroll
    for (int v = 0; v < VEC; v += 4) {
        const float4 a = *(const float4*)(ob + v);
        const float4 f = load4(o_fg + row * D + ch + v);
        const float4 l = load4(o_l + row * D + ch + v);
        float4 o;
        o.x = fmaf(g_cg, a.x, fmaf(g_fg, f.x, g_l * l.x));
        o.y = fmaf(g_cg, a.y, fmaf(g_fg, f.y, g_l * l.y));
        o.z = fmaf(g_cg, a.z, fmaf(g_fg, f.z, g_l * l.z));
        o.w = fmaf(g_cg, a.w, fmaf(g_fg, f.w, g_l * l.w));
        store4(out + row * D + ch + v, o);
    }
}

hipError_t launch_combine(bool is_bf16, const float* obar, const void* o_fg, const void* o_l,
                          const float* gates, void* out, const Geom& g, int D, int64_t BH,
                          hipStream_t stream)
{
    if (is_bf16) {
        const int64_t total = BH * g.n_tokens * (D / 8);
        hipLaunchKernelGGL((combine_kernel<uint16_t, 8>), dim3((unsigned)((total + 255) / 256)),
                           dim3(256), 0, stream, obar, (const uint16_t*)o_fg,
                           (const uint16_t*)o_l, gates, (uint16_t*)out, g, D, total);
    } else {
        const int64_t total = BH * g.n_tokens * (D / 4);
        hipLaunchKernelGGL((combine_kernel<float, 4>), dim3((unsigned)((total + 255) / 256)),
                           dim3(256), 0, stream, obar, (const float*)o_fg, (const float*)o_l,
                           gates, (float*)out, g, D, total);
    }
    return hipGetLastError();
}


// ---------------------------------------------------------------------------
// Backward of the three-branch output (selection held fixed).
//   branch_grads_kernel  dO_fg = g_fg * dO and dO_l = g_l * dO (what the
//                        attention backward kernels of the two branches take
//                        as upstream gradient) and the gate gradients
//                        dg_b = dO . o_b per token.
//   gated_block_sum_kernel  d(coarse row of block i) = sum over the tokens l
//                        of the block of g_cg(l) * dO_l, fp32 [B*h, m, D].
//   coarse_bwd_rows_kernel  per query block: block attention a_i, da_ij =
//                        dobar_i . vbar_j, ds_ij = a_ij (da_ij - sum_j a_ij
//                        da_ij); writes a and ds and dqbar_i = scale * sum_j
//                        ds_ij kbar_j.
//   coarse_bwd_cols_kernel  per key block and key/value slice: dvbar_j =
//                        sum_i a_ij dobar_i and dkbar_j = scale * sum_i ds_ij
//                        qbar_i.
// The two kernels alternate over chunks of R query blocks, so that a and ds
// are fp32 [B*h, R, m] with R chosen by the caller's scratch size, not
// [B*h, m, m]: the column kernel carries its sums from chunk to chunk in
// dkbar / dvbar (unscaled until the last chunk).  Summation order: chunks
// ascending, inside a chunk the query heads of the group ascending, inside a
// head the query blocks ascending.
// The pooled gradients reach the tokens in the local branch's attention
// backward, whose stores add (pooled gradient of the token's block) / b: the
// mean pooling hands every token of a block the same share.
// ---------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void branch_grads_kernel(
    const float* __restrict__ obar, const T* __restrict__ o_fg, const T* __restrict__ o_l,
    const float* __restrict__ gates, const T* __restrict__ dout, T* __restrict__ do_fg,
    T* __restrict__ do_l, float* __restrict__ dgates, Geom g, int D, int64_t total)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = e < total;
    if (!valid) e = total - 1;                        // keep the lane groups whole
    const int per_row = D / VEC;                      // lanes per token: a power of two <= 32
    const int64_t row = e / per_row;
    const int ch = (int)(e - row * per_row) * VEC;
    const int64_t bh = row / g.n_tokens;
    const int64_t tok = row - bh * g.n_tokens;
    const int gr = (int)(tok / g.grid_w), gc = (int)(tok - (int64_t)gr * g.grid_w);
    const int beta = (gr / g.block_h) * g.blocks_per_row + gc / g.block_w;
    const float g_fg = gates[row * 3 + 1], g_l = gates[row * 3 + 2];
    const float* ob = obar + (bh * g.n_blocks + beta) * D + ch;
    float d_cg = 0.0f, d_fg = 0.0f, d_l = 0.0f;
#pragma unroll
    for (int v = 0; v < VEC; v += 4) {
        const float4 up = load4(dout + row * D + ch + v);
        const float4 a = *(const float4*)(ob + v);
        const float4 f = load4(o_fg + row * D + ch + v);
        const float4 l = load4(o_l + row * D + ch + v);
        d_cg += up.x * a.x + up.y * a.y + up.z * a.z + up.w * a.w;
        d_fg += up.x * f.x + up.y * f.y + up.z * f.z + up.w * f.w;
        d_l += up.x * l.x + up.y * l.y + up.z * l.z + up.w * l.w;
        if (valid) {
            store4(do_fg + row * D + ch + v,
                   make_float4(g_fg * up.x, g_fg * up.y, g_fg * up.z, g_fg * up.w));
            store4(do_l + row * D + ch + v,
                   make_float4(g_l * up.x, g_l * up.y, g_l * up.z, g_l * up.w));
        }
    }
    for (int off = per_row >> 1; off >= 1; off >>= 1) {
        d_cg += __shfl_xor(d_cg, off);
        d_fg += __shfl_xor(d_fg, off);
        d_l += __shfl_xor(d_l, off);
    }
    if (valid && ch == 0) {
        dgates[row * 3 + 0] = d_cg;
        dgates[row * 3 + 1] = d_fg;
        dgates[row * 3 + 2] = d_l;
    }
}

// One thread per (block, group of VEC channels); tokens in in-tile order.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gated_block_sum_kernel(const T* __restrict__ dout,
                                                              const float* __restrict__ gates,
                                                              float* __restrict__ dobar, Geom g,
                                                              int D, int64_t total)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int groups = D / VEC;
    const int64_t blk = e / groups;                   // bh * m + beta
    const int ch = (int)(e - blk * groups) * VEC;
    const int64_t bh = blk / g.n_blocks;
    const int beta = (int)(blk - bh * g.n_blocks);
    float acc[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[c] = 0.0f;
    for (int tau = 0; tau < g.block_tokens; ++tau) {
        const int64_t row = bh * g.n_tokens + token_of(g, beta, tau);
        const float w = gates[row * 3 + 0];
#pragma unroll
        for (int v = 0; v < VEC; v += 4) {
            const float4 up = load4(dout + row * D + ch + v);
            acc[v + 0] = fmaf(w, up.x, acc[v + 0]);
            acc[v + 1] = fmaf(w, up.y, acc[v + 1]);
            acc[v + 2] = fmaf(w, up.z, acc[v + 2]);
            acc[v + 3] = fmaf(w, up.w, acc[v + 3]);
        }
    }
#pragma unroll
    for (int v = 0; v < VEC; v += 4)
        *(float4*)(dobar + blk * D + ch + v) =
            make_float4(acc[v], acc[v + 1], acc[v + 2], acc[v + 3]);
}

// Same workgroup shape as coarse_kernel (G <= 8 query blocks of one slice).
// LDS: 4*G*D (partials) + 2*G*m (weights, ds) floats.
template <int D>
__global__ __launch_bounds__(256) void coarse_bwd_rows_kernel(
    const float* __restrict__ qbar, const float* __restrict__ kbar,
    const float* __restrict__ kbar_il, const float* __restrict__ vbar,
    const float* __restrict__ dobar, float* __restrict__ a_out, float* __restrict__ ds_out,
    float* __restrict__ dqbar, Geom g, int G, int R, int r0, int r1)
{
    // query blocks r0 .. r1-1 of every slice; a_out, ds_out: [B*h, R, m] with
    // R >= r1 - r0
    constexpr int CG = D / 4, JP = 256 / CG;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int m = g.n_blocks;
    float* red_s = (float*)smem;                     // [4 wavefronts][G][D]
    float* sc_s = red_s + 4 * G * D;                 // [G][m]: scores -> weights a
    float* da_s = sc_s + G * m;                      // [G][m]: da -> ds

    const int groups = (r1 - r0 + G - 1) / G;
    const int64_t bh_idx = blockIdx.x / groups;
    const int i0 = r0 + (int)(blockIdx.x - bh_idx * groups) * G;
    const int rows = min(G, r1 - i0);
    const int64_t kv = kv_slice_of(g, bh_idx);
    kbar += kv * m * D;
    vbar += kv * m * D;
    const int64_t row0 = bh_idx * m + i0;
    const int64_t out_row0 = bh_idx * R + (i0 - r0);    // row of a_out / ds_out
    if (kbar_il) kbar_il += kv * m * D;              // per slice [D/4][m][4]

    // scores (base-2 domain) and da_ij = dobar_i . vbar_j; the rows of qbar and
    // dobar are wave-uniform (scalar loads, scalar operands of the fma)
    const float c2 = g.scale * kLog2e;
    for (int j = threadIdx.x; j < m; j += blockDim.x) {
        float kr[D];
        const float4* ksrc = kbar_il ? (const float4*)kbar_il + j
                                     : (const float4*)(kbar + (int64_t)j * D);
        const int64_t kstep = kbar_il ? (int64_t)m : 1;
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const float4 t = ksrc[d4 * kstep];
            kr[4 * d4 + 0] = t.x; kr[4 * d4 + 1] = t.y; kr[4 * d4 + 2] = t.z; kr[4 * d4 + 3] = t.w;
        }
        for (int r = 0; r < rows; ++r) {
            const float* __restrict__ qrow = qbar + (row0 + r) * D;
            float acc = 0.0f;
#pragma unroll
            for (int d = 0; d < D; ++d) acc = fmaf(qrow[d], kr[d], acc);
            sc_s[r * m + j] = acc * c2;
        }
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const float4 t = *(const float4*)(vbar + (int64_t)j * D + 4 * d4);
            kr[4 * d4 + 0] = t.x; kr[4 * d4 + 1] = t.y; kr[4 * d4 + 2] = t.z; kr[4 * d4 + 3] = t.w;
        }
        for (int r = 0; r < rows; ++r) {
            const float* __restrict__ dorow = dobar + (row0 + r) * D;
            float acc = 0.0f;
#pragma unroll
            for (int d = 0; d < D; ++d) acc = fmaf(dorow[d], kr[d], acc);
            da_s[r * m + j] = acc;
        }
    }
    __syncthreads();

    // softmax weights and sum_j a_ij da_ij, one wavefront per row
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < rows; r += 4) {
        float* row = sc_s + r * m;
        float mx = -INFINITY;
        for (int j = lane; j < m; j += 64) mx = fmaxf(mx, row[j]);
        mx = wave_max(mx);
        float sum = 0.0f;
        for (int j = lane; j < m; j += 64) {
            const float w = __builtin_amdgcn_exp2f(row[j] - mx);
            row[j] = w;
            sum += w;
        }
        const float inv = 1.0f / wave_sum(sum);
        float dot = 0.0f;
        for (int j = lane; j < m; j += 64) {
            const float a = row[j] * inv;
            row[j] = a;
            dot = fmaf(a, da_s[r * m + j], dot);
        }
        dot = wave_sum(dot);
        // ds_ij, and both matrices to global memory for the column pass
        float* a_row = a_out + (out_row0 + r) * (int64_t)m;
        float* ds_row = ds_out + (out_row0 + r) * (int64_t)m;
        for (int j = lane; j < m; j += 64) {
            const float a = row[j];
            const float ds = a * (da_s[r * m + j] - dot);
            da_s[r * m + j] = ds;
            a_row[j] = a;
            ds_row[j] = ds;
        }
    }
    __syncthreads();

    // dqbar_i = scale * sum_j ds_ij kbar_j
    const int cg = threadIdx.x % CG, jp = threadIdx.x / CG;
    float4 acc[kCoarseRows];
#pragma unroll
    for (int r = 0; r < kCoarseRows; ++r) acc[r] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int j = jp; j < m; j += JP) {
        const float4 val = *(const float4*)(kbar + (int64_t)j * D + 4 * cg);
#pragma unroll
        for (int r = 0; r < kCoarseRows; ++r) {
            if (r < rows) {
                const float w = da_s[r * m + j];
                acc[r].x = fmaf(w, val.x, acc[r].x);
                acc[r].y = fmaf(w, val.y, acc[r].y);
                acc[r].z = fmaf(w, val.z, acc[r].z);
                acc[r].w = fmaf(w, val.w, acc[r].w);
            }
        }
    }
    // the partitions of a wavefront hold the same channel quad CG lanes apart
#pragma unroll
    for (int r = 0; r < kCoarseRows; ++r)
        for (int off = CG; off < 64; off <<= 1) {
            acc[r].x += __shfl_xor(acc[r].x, off);
            acc[r].y += __shfl_xor(acc[r].y, off);
            acc[r].z += __shfl_xor(acc[r].z, off);
            acc[r].w += __shfl_xor(acc[r].w, off);
        }
    if (lane < CG) {
#pragma unroll
        for (int r = 0; r < kCoarseRows; ++r)
            if (r < rows) *(float4*)(red_s + ((wave * G + r) * D) + 4 * cg) = acc[r];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < rows * D; e += blockDim.x) {
        const int r = e / D, d = e - r * D;
        float sum = 0.0f;
        for (int p = 0; p < 4; ++p) sum += red_s[(p * G + r) * D + d];
        dqbar[(row0 + r) * D + d] = sum * g.scale;
    }
}

static size_t coarse_bwd_lds_bytes(int G, int m, int D)
{
    return ((size_t)4 * G * D + (size_t)2 * G * m) * 4;
}

int coarse_bwd_group_size(int m, int D)
{
    for (int G = kCoarseRows; G >= 1; G >>= 1)
        if (coarse_bwd_lds_bytes(G, m, D) <= kCoarseLdsBudget) return G;
    return 0;
}

// One lane per key block j (a wavefront covers 64 consecutive ones of one
// key/value slice): it walks the query blocks i = r0 .. r1-1 in ascending
// order, reading column j of a and ds ([B*h, R, m]: lanes read consecutive
// addresses) and adding a_ij * dobar_i and ds_ij * qbar_i into its D-channel
// accumulators; the rows dobar_i and qbar_i are the same for the whole
// wavefront.  The sums start from what dkbar / dvbar hold unless r0 == 0 and
// are scaled only when r1 == m, so a sequence of calls over ascending chunks
// adds every term once, in a fixed order.
template <int D>
__global__ __launch_bounds__(256) void coarse_bwd_cols_kernel(
    const float* __restrict__ qbar, const float* __restrict__ dobar,
    const float* __restrict__ a_in, const float* __restrict__ ds_in, float* __restrict__ dkbar,
    float* __restrict__ dvbar, Geom g, int64_t waves, int R, int r0, int r1)
{
    const int m = g.n_blocks;
    const int chunks = (m + 63) / 64;
    // (made uniform for the compiler: the rows below then come in through scalar loads)
    const int64_t wave_id =
        (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (wave_id >= waves) return;                     // whole wavefront; no barriers below
    const int64_t kv = wave_id / chunks;              // key/value slice
    const int64_t kv_heads = g.heads / g.kv_group;
    const int j = (int)(wave_id - kv * chunks) * 64 + (int)(threadIdx.x & 63);
    const int jc = j < m ? j : m - 1;                 // clamped column of an idle lane
    const int64_t bh_first = (kv / kv_heads) * g.heads + (kv % kv_heads) * g.kv_group;

    float acc_k[D], acc_v[D];
    float* dk_row = dkbar + (kv * m + jc) * D;
    float* dv_row = dvbar + (kv * m + jc) * D;
    if (r0 == 0) {
#pragma unroll
        for (int d = 0; d < D; ++d) { acc_k[d] = 0.0f; acc_v[d] = 0.0f; }
    } else {
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 pk = *(const float4*)(dk_row + d), pv = *(const float4*)(dv_row + d);
            acc_k[d] = pk.x; acc_k[d + 1] = pk.y; acc_k[d + 2] = pk.z; acc_k[d + 3] = pk.w;
            acc_v[d] = pv.x; acc_v[d + 1] = pv.y; acc_v[d + 2] = pv.z; acc_v[d + 3] = pv.w;
        }
    }
    // query heads of the group in ascending order, query blocks ascending
    for (int gq = 0; gq < g.kv_group; ++gq) {
        const int64_t bh = bh_first + gq;
        const float* a_col = a_in + bh * R * (int64_t)m + jc;
        const float* s_col = ds_in + bh * R * (int64_t)m + jc;
        const float* q_rows = qbar + bh * m * D;
        const float* d_rows = dobar + bh * m * D;
        for (int i = r0; i < r1; ++i) {
            const float a = a_col[(int64_t)(i - r0) * m], ds = s_col[(int64_t)(i - r0) * m];
#pragma unroll
            for (int d = 0; d < D; ++d) {
                acc_v[d] = fmaf(a, d_rows[i * D + d], acc_v[d]);
                acc_k[d] = fmaf(ds, q_rows[i * D + d], acc_k[d]);
            }
        }
    }
    if (j < m) {
        const float fk = r1 == m ? g.scale : 1.0f;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            *(float4*)(dk_row + d) = make_float4(acc_k[d] * fk, acc_k[d + 1] * fk,
                                                 acc_k[d + 2] * fk, acc_k[d + 3] * fk);
            *(float4*)(dv_row + d) =
                make_float4(acc_v[d], acc_v[d + 1], acc_v[d + 2], acc_v[d + 3]);
        }
    }
}

hipError_t launch_branch_grads(bool is_bf16, const float* obar, const void* o_fg, const void* o_l,
                               const float* gates, const void* dout, void* do_fg, void* do_l,
                               float* dgates, float* dobar, const Geom& g, int D, int64_t BH,
                               hipStream_t stream)
{
    if (is_bf16) {
        typedef uint16_t T;
        const int64_t total = BH * g.n_tokens * (D / 8);
        hipLaunchKernelGGL((branch_grads_kernel<T, 8>), dim3((unsigned)((total + 255) / 256)),
                           dim3(256), 0, stream, obar, (const T*)o_fg, (const T*)o_l, gates,
                           (const T*)dout, (T*)do_fg, (T*)do_l, dgates, g, D, total);
        const int64_t blocks = BH * g.n_blocks * (D / 8);
        hipLaunchKernelGGL((gated_block_sum_kernel<T, 8>), dim3((unsigned)((blocks + 255) / 256)),
                           dim3(256), 0, stream, (const T*)dout, gates, dobar, g, D, blocks);
    } else {
        typedef float T;
        const int64_t total = BH * g.n_tokens * (D / 4);
        hipLaunchKernelGGL((branch_grads_kernel<T, 4>), dim3((unsigned)((total + 255) / 256)),
                           dim3(256), 0, stream, obar, (const T*)o_fg, (const T*)o_l, gates,
                           (const T*)dout, (T*)do_fg, (T*)do_l, dgates, g, D, total);
        const int64_t blocks = BH * g.n_blocks * (D / 4);
        hipLaunchKernelGGL((gated_block_sum_kernel<T, 4>), dim3((unsigned)((blocks + 255) / 256)),
                           dim3(256), 0, stream, (const T*)dout, gates, dobar, g, D, blocks);
    }
    return hipGetLastError();
}

template <int D>
static hipError_t launch_coarse_bwd_t(const float* qbar, const float* kbar, const float* kbar_il,
                                      const float* vbar, const float* dobar, float* a_mat, float* ds_mat,
                                      float* dqbar, float* dkbar, float* dvbar, const Geom& g,
                                      int64_t BH, int chunk_rows, hipStream_t stream)
{
    const int G = coarse_bwd_group_size(g.n_blocks, D);
    if (G == 0) return hipErrorInvalidValue;
    static bool attr_set[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev]) {
        hipError_t e = hipFuncSetAttribute((const void*)coarse_bwd_rows_kernel<D>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kCoarseLdsBudget);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    const int m = g.n_blocks;
    const int R = chunk_rows;
    if (R < 1) return hipErrorInvalidValue;
    const int64_t BKV = BH / g.kv_group;
    const int64_t waves = BKV * ((m + 63) / 64);
    for (int r0 = 0; r0 < m; r0 += R) {
        const int r1 = r0 + R < m ? r0 + R : m;
        hipLaunchKernelGGL((coarse_bwd_rows_kernel<D>),
                           dim3((unsigned)(BH * ((r1 - r0 + G - 1) / G))), dim3(256),
                           coarse_bwd_lds_bytes(G, m, D), stream, qbar, kbar, kbar_il, vbar, dobar,
                           a_mat, ds_mat, dqbar, g, G, R, r0, r1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((coarse_bwd_cols_kernel<D>), dim3((unsigned)((waves + 3) / 4)),
                           dim3(256), 0, stream, qbar, dobar, a_mat, ds_mat, dkbar, dvbar, g,
                           waves, R, r0, r1);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_coarse_bwd(const float* qbar, const float* kbar, const float* kbar_il,
                             const float* vbar, const float* dobar, float* a_mat, float* ds_mat, float* dqbar,
                             float* dkbar, float* dvbar, const Geom& g, int D, int64_t BH,
                             int chunk_rows, hipStream_t stream)
{
    switch (D) {
    case 32: return launch_coarse_bwd_t<32>(qbar, kbar, kbar_il, vbar, dobar, a_mat, ds_mat, dqbar, dkbar, dvbar, g, BH, chunk_rows, stream);
    case 64: return launch_coarse_bwd_t<64>(qbar, kbar, kbar_il, vbar, dobar, a_mat, ds_mat, dqbar, dkbar, dvbar, g, BH, chunk_rows, stream);
    case 128: return launch_coarse_bwd_t<128>(qbar, kbar, kbar_il, vbar, dobar, a_mat, ds_mat, dqbar, dkbar, dvbar, g, BH, chunk_rows, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace bsa
