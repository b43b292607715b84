// Measurement aid: a register-resident bf16 MFMA loop, the matrix pipe's
// sustained rate on this device with nothing else in the way (no loads, no
// LDS, no vector work).  The benchmark times it beside the attention kernels:
// under matrix load the shader clock sits below its nominal value, so the
// nominal peak is not the rate the pipe can actually be driven at.
#include "bsa_launch.h"
#include "bsa_mfma_common.h"

namespace bsa {

__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ sink, int iters)
{
    // operands with full-width mantissas and mixed signs (the data decides the
    // power the pipe draws): a hash of the lane and element index
    bf16x8 a[2], b[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        uint32_t wa[4], wb[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t h = (threadIdx.x * 8u + e + 4u * u + blockIdx.x * 2048u) * 2654435761u;
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            // two bf16 in [-2, 2): sign and 7 mantissa bits from the hash, exponent 126..127
            wa[e] = (h & 0x80ff80ffu) | 0x3f003f00u;
            wb[e] = ((h >> 3) & 0x80ff80ffu) | 0x3f003f00u;
        }
        a[u] = __builtin_bit_cast(bf16x8, make_uint4(wa[0], wa[1], wa[2], wa[3]));
        b[u] = __builtin_bit_cast(bf16x8, make_uint4(wb[0], wb[1], wb[2], wb[3]));
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 4; ++rep)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rep & 1], b[j & 1], acc[j], 0, 0, 0);
    }
    float res = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) res += acc[j][r];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = res;
}

hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream, sink,
                       iters);
    return hipGetLastError();
}

}  // namespace bsa
