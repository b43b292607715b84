// C ABI of the block-sparse attention library: argument validation on the host,
// then kernel launches on the caller's stream.  Declarations and the contract
// of every entry point are in include/mosaic_bsa.h.
#include "mosaic_bsa.h"

#include <math.h>

#include "bsa_launch.h"

namespace {

struct Checked {
    bsa::Geom g;
    int D;
    int64_t BH;       // batch * heads: query slices
    int64_t BKV;      // batch * kv_heads: key/value slices
    bool is_bf16;
};

int check_params(const mosaic_bsa_params* p, Checked* out)
{
    if (!p) return MOSAIC_BSA_ERR_NULL;
    if (p->batch <= 0 || p->heads <= 0 || p->grid_h <= 0 || p->grid_w <= 0 || p->block_h <= 0 ||
        p->block_w <= 0)
        return MOSAIC_BSA_ERR_SHAPE;
    if (p->grid_h % p->block_h || p->grid_w % p->block_w) return MOSAIC_BSA_ERR_SHAPE;
    const int64_t b = (int64_t)p->block_h * p->block_w;
    if (b > 1024) return MOSAIC_BSA_ERR_SHAPE;
    const int64_t N = (int64_t)p->grid_h * p->grid_w;
    const int64_t m = N / b;
    const int64_t BH = (int64_t)p->batch * p->heads;
    // launch grids are linear in x: keep every product below 2^31
    if (N > (int64_t)1 << 30 || BH > (int64_t)1 << 24 || BH * m * ((b + 63) / 64) >= (int64_t)1 << 31)
        return MOSAIC_BSA_ERR_SHAPE;
    if (p->head_dim != 32 && p->head_dim != 64 && p->head_dim != 128)
        return MOSAIC_BSA_ERR_HEAD_DIM;
    if (p->dtype != MOSAIC_BSA_F32 && p->dtype != MOSAIC_BSA_BF16) return MOSAIC_BSA_ERR_DTYPE;
    if (p->n_select < 0 || p->n_select > m - 1) return MOSAIC_BSA_ERR_NSELECT;
    const int kv_heads = p->kv_heads == 0 ? p->heads : p->kv_heads;
    if (kv_heads < 0 || kv_heads > p->heads || p->heads % kv_heads) return MOSAIC_BSA_ERR_SHAPE;

    out->D = p->head_dim;
    out->BH = BH;
    out->BKV = (int64_t)p->batch * kv_heads;
    out->is_bf16 = p->dtype == MOSAIC_BSA_BF16;
    bsa::Geom& g = out->g;
    g.heads = p->heads;
    g.grid_w = p->grid_w;
    g.block_h = p->block_h;
    g.block_w = p->block_w;
    g.blocks_per_row = p->grid_w / p->block_w;
    g.n_blocks = (int32_t)m;
    g.block_tokens = (int32_t)b;
    g.n_select = p->n_select;
    g.n_tokens = N;
    g.scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
    g.kv_group = p->heads / kv_heads;
    return MOSAIC_BSA_OK;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

size_t select_workspace(const Checked& c)
{
    return 2 * align_up((size_t)c.BH * c.g.n_blocks * c.D * sizeof(float));
}

size_t bwd_workspace(const Checked& c)
{
    // delta, then lse * log2(e) (the second half is used by the matrix-core path)
    return 2 * align_up((size_t)c.BH * (size_t)c.g.n_tokens * sizeof(float));
}

}  // namespace

extern "C" size_t mosaic_bsa_workspace_bytes(const mosaic_bsa_params* params, int op)
{
    Checked c;
    if (check_params(params, &c) != MOSAIC_BSA_OK) return 0;
    switch (op) {
    case MOSAIC_BSA_OP_SELECT: return select_workspace(c);
    case MOSAIC_BSA_OP_FWD: return 0;
    case MOSAIC_BSA_OP_BWD: return bwd_workspace(c);
    }
    return 0;
}

extern "C" int mosaic_bsa_select(const mosaic_bsa_params* params, const void* q, const void* k,
                                 int32_t* sel_idx, void* workspace, size_t workspace_bytes,
                                 void* hip_stream)
{
    Checked c;
    if (int rc = check_params(params, &c)) return rc;
    if (!q || !k) return MOSAIC_BSA_ERR_NULL;
    if (c.g.n_select > 0 && !sel_idx) return MOSAIC_BSA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(workspace)) return MOSAIC_BSA_ERR_ALIGN;
    if (!workspace || workspace_bytes < select_workspace(c)) return MOSAIC_BSA_ERR_WORKSPACE;
    if (bsa::select_group_size(c.g.n_blocks, c.D) == 0) return MOSAIC_BSA_ERR_SHAPE;

    hipStream_t stream = (hipStream_t)hip_stream;
    float* qbar = (float*)workspace;
    float* kbar = (float*)((char*)workspace + select_workspace(c) / 2);
    if (bsa::launch_pool(c.is_bf16, q, k, qbar, kbar, c.g, c.D, c.BH, stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    if (c.g.n_select == 0) return MOSAIC_BSA_OK;
    if (bsa::launch_select(qbar, kbar, sel_idx, c.g, c.D, c.BH, stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    return MOSAIC_BSA_OK;
}

extern "C" int mosaic_bsa_fwd(const mosaic_bsa_params* params, const void* q, const void* k,
                              const void* v, const int32_t* sel_idx, void* out, float* lse,
                              void* workspace, size_t workspace_bytes, void* hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    Checked c;
    if (int rc = check_params(params, &c)) return rc;
    if (!q || !k || !v || !out) return MOSAIC_BSA_ERR_NULL;
    if (c.g.n_select > 0 && !sel_idx) return MOSAIC_BSA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out))
        return MOSAIC_BSA_ERR_ALIGN;

    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e;
    if (bsa::fwd_mfma_supported(c.is_bf16, c.g, c.D))
        e = bsa::launch_fwd_mfma(q, k, v, sel_idx, out, lse, c.g, c.D, c.BH, stream);
    else if (bsa::fwd_mfma_d128_supported(c.is_bf16, c.g, c.D))
        e = bsa::launch_fwd_mfma_d128(q, k, v, sel_idx, out, lse, c.g, c.BH, stream);
    else
        e = bsa::launch_fwd_generic(c.is_bf16, q, k, v, sel_idx, out, lse, c.g, c.D, c.BH,
                                    stream);
    return e == hipSuccess ? MOSAIC_BSA_OK : MOSAIC_BSA_ERR_LAUNCH;
}

extern "C" int mosaic_bsa_bwd(const mosaic_bsa_params* params, const void* q, const void* k,
                              const void* v, const void* out, const float* lse, const void* dout,
                              const int32_t* sel_idx, void* dq, void* dk, void* dv,
                              void* workspace, size_t workspace_bytes, void* hip_stream)
{
    Checked c;
    if (int rc = check_params(params, &c)) return rc;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv) return MOSAIC_BSA_ERR_NULL;
    if (c.g.n_select > 0 && !sel_idx) return MOSAIC_BSA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(dout) ||
        misaligned(dq) || misaligned(dk) || misaligned(dv) || misaligned(workspace))
        return MOSAIC_BSA_ERR_ALIGN;
    if (!workspace || workspace_bytes < bwd_workspace(c)) return MOSAIC_BSA_ERR_WORKSPACE;

    hipStream_t stream = (hipStream_t)hip_stream;
    float* delta = (float*)workspace;
    float* lse2 = (float*)((char*)workspace + bwd_workspace(c) / 2);
    const hipError_t e =
        bsa::bwd_mfma_supported(c.is_bf16, c.g, c.D)
            ? bsa::launch_bwd_mfma(q, k, v, out, lse, dout, sel_idx, dq, dk, dv, delta, lse2, c.g,
                                   c.D, c.BH, stream)
            : bsa::launch_bwd(c.is_bf16, q, k, v, out, lse, dout, sel_idx, dq, dk, dv, delta, c.g,
                              c.D, c.BH, stream);
    return e == hipSuccess ? MOSAIC_BSA_OK : MOSAIC_BSA_ERR_LAUNCH;
}

extern "C" const char* mosaic_bsa_strerror(int code)
{
    switch (code) {
    case MOSAIC_BSA_OK: return "success";
    case MOSAIC_BSA_ERR_NULL: return "a required pointer is NULL";
    case MOSAIC_BSA_ERR_SHAPE:
        return "invalid shape: sizes must be positive, the tile must divide the grid, "
               "b <= 1024 and the problem must fit the launch limits";
    case MOSAIC_BSA_ERR_NSELECT: return "n_select must satisfy 0 <= n_select <= m - 1";
    case MOSAIC_BSA_ERR_HEAD_DIM: return "head_dim must be 32, 64 or 128";
    case MOSAIC_BSA_ERR_DTYPE: return "dtype must be MOSAIC_BSA_F32 or MOSAIC_BSA_BF16";
    case MOSAIC_BSA_ERR_WORKSPACE: return "workspace is NULL or smaller than required";
    case MOSAIC_BSA_ERR_ALIGN: return "tensor base pointers must be 16-byte aligned";
    case MOSAIC_BSA_ERR_LAUNCH: return "HIP kernel launch failed";
    case MOSAIC_BSA_ERR_OP: return "operation not available";
    }
    return "unknown error code";
}
