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
//            registers and scores it against the G pooled queries (LDS
//            broadcasts); scaled scores (base-2 domain) land in LDS.
//   phase 2: one wavefront per query block: row maximum, weights
//            exp2(s - max) written back in place, 1 / row sum.
//   phase 3: thread = (channel quad, key partition): walks the pooled values
//            of its key partition (a row of vbar is read by D/4 adjacent
//            lanes, 16 bytes each) and accumulates weight * value for all G
//            rows in registers.
//   phase 4: the partitions' partial rows are summed through LDS in fixed
//            order and scaled by 1 / row sum.
// LDS: G*D (pooled queries) + G*m (scores) + (1024/D)*G*D (partials) + G floats.
template <int D>
__global__ __launch_bounds__(256) void coarse_kernel(const float* __restrict__ qbar,
                                                     const float* __restrict__ kbar,
                                                     const float* __restrict__ vbar,
                                                     float* __restrict__ obar, Geom g, int G)
{
    constexpr int CG = D / 4;                        // channel quads
    constexpr int JP = 256 / CG;                     // key partitions
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int m = g.n_blocks;
    float* q_s = (float*)smem;                       // [G][D]
    float* red_s = q_s + G * D;                      // [JP][G][D]
    float* inv_s = red_s + JP * G * D;               // [8]
    float* sc_s = inv_s + kCoarseRows;               // [G][m]

    const int groups = (m + G - 1) / G;
    const int64_t bh_idx = blockIdx.x / groups;
    const int i0 = (int)(blockIdx.x - bh_idx * groups) * G;
    const int rows = min(G, m - i0);
    const int64_t kv = kv_slice_of(g, bh_idx);
    qbar += (bh_idx * m + i0) * D;
    kbar += kv * m * D;
    vbar += kv * m * D;

    for (int e = threadIdx.x; e < rows * D; e += blockDim.x) q_s[e] = qbar[e];
    __syncthreads();

    // ---- phase 1: scaled scores
    const float c2 = g.scale * kLog2e;
    for (int j = threadIdx.x; j < m; j += blockDim.x) {
        float kr[D];
        const float4* krow = (const float4*)(kbar + (int64_t)j * D);
#pragma unroll
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const float4 t = krow[d4];
            kr[4 * d4 + 0] = t.x; kr[4 * d4 + 1] = t.y;
            kr[4 * d4 + 2] = t.z; kr[4 * d4 + 3] = t.w;
        }
        for (int r = 0; r < rows; ++r) {
            const float4* qrow = (const float4*)(q_s + r * D);
            float acc = 0.0f;
#pragma unroll
            for (int d4 = 0; d4 < D / 4; ++d4) {
                const float4 qv = qrow[d4];
                acc = fmaf(qv.x, kr[4 * d4 + 0], acc);
                acc = fmaf(qv.y, kr[4 * d4 + 1], acc);
                acc = fmaf(qv.z, kr[4 * d4 + 2], acc);
                acc = fmaf(qv.w, kr[4 * d4 + 3], acc);
            }
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
#pragma unroll
    for (int r = 0; r < kCoarseRows; ++r)
        if (r < rows) *(float4*)(red_s + ((jp * G + r) * D) + 4 * cg) = acc[r];
    __syncthreads();

    // ---- phase 4: sum the partitions in ascending order
    for (int e = threadIdx.x; e < rows * D; e += blockDim.x) {
        const int r = e / D, d = e - r * D;
        float sum = 0.0f;
        for (int p = 0; p < JP; ++p) sum += red_s[(p * G + r) * D + d];
        obar[(bh_idx * m + i0 + r) * D + d] = sum * inv_s[r];
    }
}

static size_t coarse_lds_bytes(int G, int m, int D)
{
    return ((size_t)G * D + (size_t)(1024 / D) * G * D + kCoarseRows + (size_t)G * m) * 4;
}

int coarse_group_size(int m, int D)
{
    for (int G = kCoarseRows; G >= 1; G >>= 1)
        if (coarse_lds_bytes(G, m, D) <= kCoarseLdsBudget) return G;
    return 0;
}

template <int D>
static hipError_t launch_coarse_t(const float* qbar, const float* kbar, const float* vbar,
                                  float* obar, const Geom& g, int64_t BH, hipStream_t stream)
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
                       stream, qbar, kbar, vbar, obar, g, G);
    return hipGetLastError();
}

hipError_t launch_coarse(const float* qbar, const float* kbar, const float* vbar, float* obar,
                         const Geom& g, int D, int64_t BH, hipStream_t stream)
{
    switch (D) {
    case 32: return launch_coarse_t<32>(qbar, kbar, vbar, obar, g, BH, stream);
    case 64: return launch_coarse_t<64>(qbar, kbar, vbar, obar, g, BH, stream);
    case 128: return launch_coarse_t<128>(qbar, kbar, vbar, obar, g, BH, stream);
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

}  // namespace bsa
