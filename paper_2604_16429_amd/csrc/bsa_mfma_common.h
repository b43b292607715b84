// Pieces shared by the MFMA attention kernels (gfx950): operand vector types,
// the lane-32 exchange, the bf16 packing of the attention weights and the
// weights of one 32-key x 32-query tile.
#pragma once

#include "bsa_device.h"

namespace bsa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

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

// Two fp32 values -> bf16 pair, round to nearest even (v_cvt_pk_bf16_f32; it
// issues at the rate of any other three-operand vector instruction).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    const f32x2 v = {a, b};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// P^T = exp2(S^T c2 - m_ref) for one 32-key x 32-query tile, rounded to bf16 B
// operands; returns this lane's sum of the fp32 weights.  Only builtins touch
// the MFMA results (never inline asm): the compiler must see these reads to
// place the wait states the hardware requires.
__device__ __forceinline__ float tile_weights(const f32x16& s, float c2, float neg_m,
                                              bf16x8 (&p)[2])
{
    float rs = 0.0f;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[8 * h + 2 * e], c2, neg_m));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[8 * h + 2 * e + 1], c2, neg_m));
            w[e] = pack_bf16(p0, p1);
            rs += p0 + p1;
        }
        p[h] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
    return rs;
}

constexpr float kSumLimit = 4096.0f;

}  // namespace bsa
