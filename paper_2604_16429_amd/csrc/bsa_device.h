// Device-side helpers shared by the HIP kernels of the block-sparse attention
// library (gfx950 only).  Notation follows the paper: N tokens on an H x W grid,
// blocks of b = bh*bw tokens, m = N/b blocks, n selected blocks, head dim D.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsa {

// Geometry of one call, passed by value to every kernel.
struct Geom {
    int32_t heads;        // h
    int32_t grid_w;       // W
    int32_t block_h;      // bh
    int32_t block_w;      // bw
    int32_t blocks_per_row;  // W / bw
    int32_t n_blocks;     // m
    int32_t block_tokens; // b
    int32_t n_select;     // n
    int64_t n_tokens;     // N
    float   scale;        // softmax scale
    int32_t kv_group;     // query heads per key/value head (1 = every head has its own)
    int32_t list_only;    // forward: 1 = attend exactly the n listed blocks (n >= 1), 0 = block i
                          // itself, then the n listed blocks
    int32_t own_is_candidate;  // selection: 1 = rank all m key blocks, 0 = all but block i
    // Backward: when not null, a gradient is ADDED to what dq / dk / dv hold,
    // together with row [slice, block of the token] of these fp32 [slices, m, D]
    // tensors divided by b (the three-branch form: the local branch adds to the
    // selection branch's result and brings the coarse branch's share along).
    const float* add_dq;
    const float* add_dk;
    const float* add_dv;
};

// out = v, or in accumulate mode (extra != null) out = old + v + extra[0..3] * inv_b
template <typename T>
__device__ __forceinline__ void store4_or_add(T* p, float4 v, const float* extra, float inv_b);

// [N, D] slice of K and V that the query slice bh = batch * heads + head
// attends to (grouped query attention: consecutive query heads share one).
__device__ __forceinline__ int64_t kv_slice_of(const Geom& g, int64_t bh)
{
    if (g.kv_group == 1) return bh;
    const int64_t e = bh / g.heads, a = bh - e * g.heads;
    return e * (g.heads / g.kv_group) + a / g.kv_group;
}

// Workgroup id -> (query slice, item).  Workgroup ids go round-robin over the
// 8 XCDs, each with its own L2, so key/value slices are dealt to XCDs whole:
// key/value slice u runs on XCD u % 8, the items of the query heads that share
// it back to back; the K/V tiles that those query blocks gather are then
// fetched into one L2 instead of eight.  The last (number of key/value slices
// % 8) slices use the plain linear order.  per_slice: items per query slice;
// n_units: number of key/value slices.  The grid is n_units * kv_group *
// per_slice workgroups, which the launcher keeps below 2^32.
__device__ __forceinline__ void map_unit(uint32_t w, uint32_t per_unit, uint32_t n_units,
                                         uint32_t& unit, uint32_t& r)
{
    const uint32_t units_xcd = n_units & ~7u;
    if (w < units_xcd * per_unit) {
        const uint32_t seq = w >> 3, round = seq / per_unit;
        unit = round * 8 + (w & 7);
        r = seq - round * per_unit;
    } else {
        unit = w / per_unit;
        r = w - unit * per_unit;
    }
}

__device__ __forceinline__ void map_workgroup(const Geom& g, uint32_t w, uint32_t per_slice,
                                              uint32_t n_units, int64_t& bh, int& item)
{
    uint32_t unit, r;
    map_unit(w, per_slice * (uint32_t)g.kv_group, n_units, unit, r);
    if (g.kv_group == 1) {
        bh = unit;
        item = (int)r;
        return;
    }
    const uint32_t head_in_group = r / per_slice;
    item = (int)(r - head_in_group * per_slice);
    const uint32_t kv_heads = (uint32_t)(g.heads / g.kv_group);
    const uint32_t e = unit / kv_heads, a = unit - e * kv_heads;
    bh = (int64_t)e * g.heads + a * g.kv_group + head_in_group;
}

// Token index (inside one [N, D] slice) of in-tile position tau of block beta:
// the tile partition of the grid (Compression paragraph, with tiles as blocks).
__device__ __forceinline__ int64_t token_of(const Geom& g, int beta, int tau)
{
    const int br = beta / g.blocks_per_row, bc = beta - br * g.blocks_per_row;
    const int rr = tau / g.block_w, cc = tau - rr * g.block_w;
    return (int64_t)(br * g.block_h + rr) * g.grid_w + (bc * g.block_w + cc);
}

// 64-token sub-tiles of a block whose width is a power of two: sub-tile ct holds
// the in-tile positions 64 ct .. 64 ct + 63, i.e. whole tile rows when the width
// divides 64 and a 64-token run of one tile row when 64 divides the width (a
// block-contiguous layout is the case of tiles one row high).
// Offset, in tokens, of the sub-tile's first token from the block's first token:
__device__ __forceinline__ int sub_tile_first(const Geom& g, int ct)
{
    const int t0 = 64 * ct;
    return (t0 >> __builtin_ctz((unsigned)g.block_w)) * g.grid_w + (t0 & (g.block_w - 1));
}
// Offset, in tokens, of position u (0..63) of a sub-tile from its first token:
__device__ __forceinline__ int sub_tile_pos(const Geom& g, int u)
{
    const int w = g.block_w < 64 ? g.block_w : 64;
    return (u >> __builtin_ctz((unsigned)w)) * g.grid_w + (u & (w - 1));
}

// bf16 <-> fp32 on raw bit patterns
__device__ __forceinline__ float bf16_to_f32(uint16_t b)
{
    return __uint_as_float((uint32_t)b << 16);
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f)   // round to nearest even
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Element loaders: 4 consecutive channels as fp32.
__device__ __forceinline__ float4 load4(const float* p) { return *(const float4*)p; }
__device__ __forceinline__ float4 load4(const uint16_t* p)
{
    const uint2 r = *(const uint2*)p;
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
}

// The same with the non-temporal hint (data that is read once).
__device__ __forceinline__ float4 load4_stream(const float* p)
{
    typedef float f4v __attribute__((ext_vector_type(4)));
    const f4v r = __builtin_nontemporal_load((const f4v*)p);
    return make_float4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ float4 load4_stream(const uint16_t* p)
{
    typedef uint32_t u2v __attribute__((ext_vector_type(2)));
    const u2v r = __builtin_nontemporal_load((const u2v*)p);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
}

__device__ __forceinline__ void store4(float* p, float4 v) { *(float4*)p = v; }
__device__ __forceinline__ void store4(uint16_t* p, float4 v)
{
    uint2 r;
    r.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
    r.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
    *(uint2*)p = r;
}

template <typename T>
__device__ __forceinline__ void store4_or_add(T* p, float4 v, const float* extra, float inv_b)
{
    if (extra) {
        const float4 old = load4(p);
        const float4 e = *(const float4*)extra;
        v = make_float4(old.x + v.x + e.x * inv_b, old.y + v.y + e.y * inv_b,
                        old.z + v.z + e.z * inv_b, old.w + v.w + e.w * inv_b);
    }
    store4(p, v);
}

}  // namespace bsa
