// C ABI of the block-sparse attention library: argument validation on the host,
// then kernel launches on the caller's stream.  Declarations and the contract
// of every entry point are in include/mosaic_bsa.h.
#include "mosaic_bsa.h"

#include <math.h>

#include <mutex>

#include "bsa_launch.h"

// Device memory of mosaic_bsa_select_static, which may not take a workspace from
// its caller nor allocate one: every GPU the library runs on holds this array
// from the moment the code object is loaded until the process ends.  In host
// code the name is only a handle; the array's address on a device comes from
// hipGetSymbolAddress (static_scratch() below).
static __device__ __align__(256) unsigned char scratch[MOSAIC_BSA_STATIC_SCRATCH_BYTES];

namespace {

struct Checked {
    bsa::Geom g;
    int D;
    int64_t BH;       // batch * heads: query slices
    int64_t BKV;      // batch * kv_heads: key/value slices
    bool is_bf16;
};

// own_is_candidate: the three-branch form, where the top-n runs over all m
// blocks (1 <= n <= m); otherwise 0 <= n <= m - 1.
int check_params(const mosaic_bsa_params* p, Checked* out, bool own_is_candidate = false)
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
    if (own_is_candidate ? (p->n_select < 1 || p->n_select > m)
                         : (p->n_select < 0 || p->n_select > m - 1))
        return MOSAIC_BSA_ERR_NSELECT;
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
    g.list_only = 0;
    g.add_dq = g.add_dk = g.add_dv = nullptr;
    g.own_is_candidate = own_is_candidate ? 1 : 0;
    return MOSAIC_BSA_OK;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// pooled q | pooled k | the ranking's channel-interleaved copy of the pooled k
size_t pooled_bytes(const Checked& c)
{
    return align_up((size_t)c.BH * c.g.n_blocks * c.D * sizeof(float));
}

size_t select_workspace(const Checked& c)
{
    return 2 * pooled_bytes(c) + align_up(bsa::select_scratch_bytes(c.g.n_blocks, c.D, c.BH, c.BKV));
}

// delta | lse * log2(e) | connection map (the last two: matrix-core path only)
size_t bwd_rows_bytes(const Checked& c)
{
    return align_up((size_t)c.BH * (size_t)c.g.n_tokens * sizeof(float));
}

size_t bwd_workspace(const Checked& c)
{
    return 2 * bwd_rows_bytes(c) +
           align_up((size_t)bsa::bwd_connection_words(c.g.n_blocks, c.BH) * sizeof(uint32_t));
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

namespace {

// Pooling, block scores and top-n with the selection workspace at `workspace`
// (select_workspace(c) bytes, 256-byte aligned, contents arbitrary: every part
// is written before it is read).
int select_impl(const Checked& c, const void* q, const void* k, int32_t* sel_idx, void* workspace,
                hipStream_t stream)
{
    float* qbar = (float*)workspace;
    float* kbar = (float*)((char*)workspace + pooled_bytes(c));
    void* rest = (char*)workspace + 2 * pooled_bytes(c);
    const hipError_t e =
        c.g.n_select > 0
            ? bsa::launch_pool_select(c.is_bf16, q, k, qbar, kbar, rest, sel_idx, c.g, c.D, c.BH,
                                      stream)
            : bsa::launch_pool(c.is_bf16, q, k, qbar, kbar, c.g, c.D, c.BH, stream);
    return e == hipSuccess ? MOSAIC_BSA_OK : MOSAIC_BSA_ERR_LAUNCH;
}

// Address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_on_device[kMaxDevices];

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return MOSAIC_BSA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_on_device[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return MOSAIC_BSA_ERR_LAUNCH;
        scratch_on_device[dev] = p;
    }
    *out = scratch_on_device[dev];
    return MOSAIC_BSA_OK;
}

}  // namespace

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
    return select_impl(c, q, k, sel_idx, workspace, (hipStream_t)hip_stream);
}

extern "C" int mosaic_bsa_select_static(const mosaic_bsa_params* params, const void* q,
                                        const void* k, int32_t* sel_idx, void* hip_stream)
{
    Checked c;
    if (int rc = check_params(params, &c)) return rc;
    if (!q || !k) return MOSAIC_BSA_ERR_NULL;
    if (c.g.n_select > 0 && !sel_idx) return MOSAIC_BSA_ERR_NULL;
    if (misaligned(q) || misaligned(k)) return MOSAIC_BSA_ERR_ALIGN;
    if (bsa::select_group_size(c.g.n_blocks, c.D) == 0) return MOSAIC_BSA_ERR_SHAPE;
    if (select_workspace(c) > (size_t)MOSAIC_BSA_STATIC_SCRATCH_BYTES)
        return MOSAIC_BSA_ERR_WORKSPACE;
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return select_impl(c, q, k, sel_idx, ws, (hipStream_t)hip_stream);
}

namespace {

// The attention forward for geometry g (which may differ from the checked one
// in its block lists): matrix-core kernels where they apply.
hipError_t forward(const Checked& c, const bsa::Geom& g, const void* q, const void* k,
                   const void* v, const int32_t* lists, void* out, float* lse,
                   hipStream_t stream)
{
    if (bsa::fwd_mfma_supported(c.is_bf16, g, c.D))
        return bsa::launch_fwd_mfma(q, k, v, lists, out, lse, g, c.D, c.BH, stream);
    if (bsa::fwd_mfma_d128_supported(c.is_bf16, g, c.D))
        return bsa::launch_fwd_mfma_d128(q, k, v, lists, out, lse, g, c.BH, stream);
    return bsa::launch_fwd_generic(c.is_bf16, q, k, v, lists, out, lse, g, c.D, c.BH, stream);
}

}  // namespace

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

    return forward(c, c.g, q, k, v, sel_idx, out, lse, (hipStream_t)hip_stream) == hipSuccess
               ? MOSAIC_BSA_OK
               : MOSAIC_BSA_ERR_LAUNCH;
}

namespace {

// Workspace of the three-branch forward: 256-byte aligned parts in this order.
struct ThreeBranchLayout {
    size_t qbar, kbar, vbar, obar, keys, lists, o_fg, o_l, lse_fg, lse_l, total;
};

ThreeBranchLayout three_branch_layout(const Checked& c, int local_tiles)
{
    const size_t m = (size_t)c.g.n_blocks, esz = c.is_bf16 ? 2 : 4;
    ThreeBranchLayout w;
    size_t at = 0;
    auto take = [&](size_t bytes) {
        const size_t start = at;
        at += align_up(bytes);
        return start;
    };
    w.qbar = take((size_t)c.BH * m * c.D * 4);
    w.kbar = take((size_t)c.BKV * m * c.D * 4);
    w.vbar = take((size_t)c.BKV * m * c.D * 4);
    w.obar = take((size_t)c.BH * m * c.D * 4);
    w.keys = take(bsa::select_scratch_bytes(c.g.n_blocks, c.D, c.BH, c.BKV));
    w.lists = take((size_t)c.BH * m * (size_t)(local_tiles - 1) * 4);
    w.o_fg = take((size_t)c.BH * (size_t)c.g.n_tokens * c.D * esz);
    w.o_l = take((size_t)c.BH * (size_t)c.g.n_tokens * c.D * esz);
    w.lse_fg = take((size_t)c.BH * (size_t)c.g.n_tokens * 4);
    w.lse_l = take((size_t)c.BH * (size_t)c.g.n_tokens * 4);
    w.total = at;
    return w;
}

int check_local(const mosaic_bsa_params* p, int local_h, int local_w)
{
    if (local_h <= 0 || local_w <= 0) return MOSAIC_BSA_ERR_SHAPE;
    if ((p->grid_h / p->block_h) % local_h || (p->grid_w / p->block_w) % local_w)
        return MOSAIC_BSA_ERR_SHAPE;
    return MOSAIC_BSA_OK;
}

}  // namespace

extern "C" size_t mosaic_bsa_three_branch_workspace_bytes(const mosaic_bsa_params* params,
                                                          int32_t local_h, int32_t local_w)
{
    Checked c;
    if (check_params(params, &c, true) || check_local(params, local_h, local_w)) return 0;
    if (bsa::select_group_size(c.g.n_blocks, c.D) == 0 ||
        bsa::coarse_group_size(c.g.n_blocks, c.D) == 0)
        return 0;
    return three_branch_layout(c, local_h * local_w).total;
}

extern "C" int mosaic_bsa_fwd_three_branch(const mosaic_bsa_params* params, int32_t local_h,
                                           int32_t local_w, const void* q, const void* k,
                                           const void* v, const float* gates, void* out,
                                           int32_t* sel_idx, void* workspace,
                                           size_t workspace_bytes, void* hip_stream)
{
    Checked c;
    if (int rc = check_params(params, &c, true)) return rc;
    if (int rc = check_local(params, local_h, local_w)) return rc;
    if (!q || !k || !v || !gates || !out || !sel_idx) return MOSAIC_BSA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) ||
        misaligned(workspace))
        return MOSAIC_BSA_ERR_ALIGN;
    if (bsa::select_group_size(c.g.n_blocks, c.D) == 0 ||
        bsa::coarse_group_size(c.g.n_blocks, c.D) == 0)
        return MOSAIC_BSA_ERR_SHAPE;
    const int local_tiles = local_h * local_w;
    const ThreeBranchLayout w = three_branch_layout(c, local_tiles);
    if (!workspace || workspace_bytes < w.total) return MOSAIC_BSA_ERR_WORKSPACE;

    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    float* qbar = (float*)(ws + w.qbar);
    float* kbar = (float*)(ws + w.kbar);
    float* vbar = (float*)(ws + w.vbar);
    float* obar = (float*)(ws + w.obar);
    int32_t* lists = (int32_t*)(ws + w.lists);
    void* o_fg = ws + w.o_fg;
    void* o_l = ws + w.o_l;

    // compression (pooled q, k, v), the coarse branch, and the ranking it shares
    // with the selection branch
    if (bsa::launch_pool_select(c.is_bf16, q, k, qbar, kbar, ws + w.keys, sel_idx, c.g, c.D, c.BH,
                                stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    if (bsa::launch_pool_one(c.is_bf16, v, vbar, c.g, c.D, c.BKV, stream) != hipSuccess ||
        bsa::launch_coarse(qbar, kbar,
                           bsa::select_interleaves_keys(c.g.n_blocks) ? (const float*)(ws + w.keys)
                                                                      : nullptr,
                           vbar, obar, c.g, c.D, c.BH, stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    // selection branch: one softmax over the selected blocks only
    bsa::Geom g_fg = c.g;
    g_fg.list_only = 1;
    if (forward(c, g_fg, q, k, v, sel_idx, o_fg, (float*)(ws + w.lse_fg), stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    // local branch: the tile and the other tiles of its large block
    bsa::Geom g_l = c.g;
    g_l.n_select = local_tiles - 1;
    if (bsa::launch_local_lists(lists, c.g, local_h, local_w, c.BH, stream) != hipSuccess ||
        forward(c, g_l, q, k, v, lists, o_l, (float*)(ws + w.lse_l), stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    // gated sum
    if (bsa::launch_combine(c.is_bf16, obar, o_fg, o_l, gates, out, c.g, c.D, c.BH, stream) !=
        hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    return MOSAIC_BSA_OK;
}

namespace {

// The attention backward for geometry g (selection or lists held fixed);
// scratch: bwd_workspace(c) bytes.
hipError_t backward(const Checked& c, const bsa::Geom& g, const void* q, const void* k,
                    const void* v, const void* out, const float* lse, const void* dout,
                    const int32_t* lists, void* dq, void* dk, void* dv, void* scratch,
                    hipStream_t stream)
{
    float* delta = (float*)scratch;
    float* lse2 = (float*)((char*)scratch + bwd_rows_bytes(c));
    uint32_t* conn = (uint32_t*)((char*)scratch + 2 * bwd_rows_bytes(c));
    return bsa::bwd_mfma_supported(c.is_bf16, g, c.D)
               ? bsa::launch_bwd_mfma(q, k, v, out, lse, dout, lists, dq, dk, dv, delta, lse2,
                                      conn, g, c.D, c.BH, stream)
               : bsa::launch_bwd(c.is_bf16, q, k, v, out, lse, dout, lists, dq, dk, dv, delta, g,
                                 c.D, c.BH, stream);
}

}  // namespace

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

    return backward(c, c.g, q, k, v, out, lse, dout, sel_idx, dq, dk, dv, workspace,
                    (hipStream_t)hip_stream) == hipSuccess
               ? MOSAIC_BSA_OK
               : MOSAIC_BSA_ERR_LAUNCH;
}

namespace {

// Workspace of the three-branch backward: 256-byte aligned parts in this order.
struct ThreeBranchBwdLayout {
    size_t attn, do_fg, do_l, dobar, a_mat, ds_mat, dqbar, dkbar, dvbar, total;
    int chunk_rows;        // query blocks per pass of the coarse branch's backward
};

// The coarse branch's backward keeps the block attention and its gradient of
// chunk_rows query blocks of every slice at a time: as many as fit this many
// bytes per matrix, at least 8.
constexpr size_t kCoarseBwdMatrixBytes = (size_t)64 << 20;

int coarse_bwd_chunk_rows(const Checked& c)
{
    const size_t m = (size_t)c.g.n_blocks;
    size_t rows = kCoarseBwdMatrixBytes / ((size_t)c.BH * m * 4);
    rows = rows / 8 * 8;
    if (rows < 8) rows = 8;
    return (int)(rows < m ? rows : m);
}

ThreeBranchBwdLayout three_branch_bwd_layout(const Checked& c)
{
    const size_t m = (size_t)c.g.n_blocks, N = (size_t)c.g.n_tokens, esz = c.is_bf16 ? 2 : 4;
    ThreeBranchBwdLayout w;
    size_t at = 0;
    auto take = [&](size_t bytes) {
        const size_t start = at;
        at += align_up(bytes);
        return start;
    };
    w.attn = take(bwd_workspace(c));                 // scratch of the attention backward kernels
    w.do_fg = take((size_t)c.BH * N * c.D * esz);
    w.do_l = take((size_t)c.BH * N * c.D * esz);
    w.dobar = take((size_t)c.BH * m * c.D * 4);
    w.chunk_rows = coarse_bwd_chunk_rows(c);
    w.a_mat = take((size_t)c.BH * w.chunk_rows * m * 4);
    w.ds_mat = take((size_t)c.BH * w.chunk_rows * m * 4);
    w.dqbar = take((size_t)c.BH * m * c.D * 4);
    w.dkbar = take((size_t)c.BKV * m * c.D * 4);
    w.dvbar = take((size_t)c.BKV * m * c.D * 4);
    w.total = at;
    return w;
}

}  // namespace

extern "C" size_t mosaic_bsa_three_branch_bwd_workspace_bytes(const mosaic_bsa_params* params,
                                                              int32_t local_h, int32_t local_w)
{
    Checked c;
    if (check_params(params, &c, true) || check_local(params, local_h, local_w)) return 0;
    if (bsa::coarse_bwd_group_size(c.g.n_blocks, c.D) == 0) return 0;
    return three_branch_bwd_layout(c).total;
}

extern "C" int mosaic_bsa_bwd_three_branch(const mosaic_bsa_params* params, int32_t local_h,
                                           int32_t local_w, const void* q, const void* k,
                                           const void* v, const float* gates, const void* dout,
                                           const int32_t* sel_idx, const void* fwd_workspace,
                                           void* dq, void* dk, void* dv, float* dgates,
                                           void* workspace, size_t workspace_bytes,
                                           void* hip_stream)
{
    Checked c;
    if (int rc = check_params(params, &c, true)) return rc;
    if (int rc = check_local(params, local_h, local_w)) return rc;
    if (!q || !k || !v || !gates || !dout || !sel_idx || !fwd_workspace || !dq || !dk || !dv ||
        !dgates)
        return MOSAIC_BSA_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(dout) || misaligned(dq) ||
        misaligned(dk) || misaligned(dv) || misaligned(fwd_workspace) || misaligned(workspace))
        return MOSAIC_BSA_ERR_ALIGN;
    if (bsa::coarse_bwd_group_size(c.g.n_blocks, c.D) == 0) return MOSAIC_BSA_ERR_SHAPE;
    const int local_tiles = local_h * local_w;
    const ThreeBranchLayout f = three_branch_layout(c, local_tiles);
    const ThreeBranchBwdLayout w = three_branch_bwd_layout(c);
    if (!workspace || workspace_bytes < w.total) return MOSAIC_BSA_ERR_WORKSPACE;

    hipStream_t stream = (hipStream_t)hip_stream;
    const char* fw = (const char*)fwd_workspace;
    char* ws = (char*)workspace;
    const float* qbar = (const float*)(fw + f.qbar);
    const float* kbar = (const float*)(fw + f.kbar);
    const float* vbar = (const float*)(fw + f.vbar);
    const float* obar = (const float*)(fw + f.obar);
    const int32_t* lists = (const int32_t*)(fw + f.lists);
    float* dobar = (float*)(ws + w.dobar);

    // upstream gradients of the two attention branches, gate gradients, and the
    // coarse rows' gradient (gated block sums of dout)
    if (bsa::launch_branch_grads(c.is_bf16, obar, fw + f.o_fg, fw + f.o_l, gates, dout,
                                 ws + w.do_fg, ws + w.do_l, dgates, dobar, c.g, c.D, c.BH,
                                 stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    // selection branch -> dq, dk, dv
    bsa::Geom g_fg = c.g;
    g_fg.list_only = 1;
    if (backward(c, g_fg, q, k, v, fw + f.o_fg, (const float*)(fw + f.lse_fg), ws + w.do_fg,
                 sel_idx, dq, dk, dv, ws + w.attn, stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    // coarse branch on the pooled tensors
    if (bsa::launch_coarse_bwd(qbar, kbar,
                               bsa::select_interleaves_keys(c.g.n_blocks)
                                   ? (const float*)(fw + f.keys) : nullptr,
                               vbar, dobar, (float*)(ws + w.a_mat),
                               (float*)(ws + w.ds_mat), (float*)(ws + w.dqbar),
                               (float*)(ws + w.dkbar), (float*)(ws + w.dvbar), c.g, c.D, c.BH,
                               w.chunk_rows, stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    // local branch, added in place together with the block's pooled gradient / b:
    // dx = selection branch + local branch + coarse branch
    bsa::Geom g_l = c.g;
    g_l.n_select = local_tiles - 1;
    g_l.add_dq = (const float*)(ws + w.dqbar);
    g_l.add_dk = (const float*)(ws + w.dkbar);
    g_l.add_dv = (const float*)(ws + w.dvbar);
    if (backward(c, g_l, q, k, v, fw + f.o_l, (const float*)(fw + f.lse_l), ws + w.do_l, lists,
                 dq, dk, dv, ws + w.attn, stream) != hipSuccess)
        return MOSAIC_BSA_ERR_LAUNCH;
    return MOSAIC_BSA_OK;
}

extern "C" int mosaic_bsa_check_selection(const mosaic_bsa_params* params,
                                          const int32_t* sel_idx, int32_t own_block_allowed,
                                          int32_t* n_bad, void* hip_stream)
{
    Checked c;
    if (int rc = check_params(params, &c, own_block_allowed != 0)) return rc;
    if (!n_bad || (c.g.n_select > 0 && !sel_idx)) return MOSAIC_BSA_ERR_NULL;
    return bsa::launch_check_selection(sel_idx, n_bad, c.g, own_block_allowed != 0, c.BH,
                                       (hipStream_t)hip_stream) == hipSuccess
               ? MOSAIC_BSA_OK
               : MOSAIC_BSA_ERR_LAUNCH;
}

extern "C" int mosaic_bsa_probe_mfma(float* sink, int32_t workgroups, int32_t iters,
                                     void* hip_stream)
{
    if (!sink) return MOSAIC_BSA_ERR_NULL;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return MOSAIC_BSA_ERR_SHAPE;
    return bsa::launch_mfma_probe(sink, workgroups, iters, (hipStream_t)hip_stream) == hipSuccess
               ? MOSAIC_BSA_OK
               : MOSAIC_BSA_ERR_LAUNCH;
}

extern "C" const char* mosaic_bsa_strerror(int code)
{
    switch (code) {
    case MOSAIC_BSA_OK: return "success";
    case MOSAIC_BSA_ERR_NULL: return "a required pointer is NULL";
    case MOSAIC_BSA_ERR_SHAPE:
        return "invalid shape: sizes must be positive, the tile must divide the grid, "
               "b <= 1024 and the problem must fit the launch limits";
    case MOSAIC_BSA_ERR_NSELECT:
        return "n_select must satisfy 0 <= n_select <= m - 1 (1 <= n_select <= m in the "
               "three-branch form)";
    case MOSAIC_BSA_ERR_HEAD_DIM: return "head_dim must be 32, 64 or 128";
    case MOSAIC_BSA_ERR_DTYPE: return "dtype must be MOSAIC_BSA_F32 or MOSAIC_BSA_BF16";
    case MOSAIC_BSA_ERR_WORKSPACE:
        return "workspace is NULL or smaller than required (mosaic_bsa_select_static: the "
               "problem needs more than MOSAIC_BSA_STATIC_SCRATCH_BYTES of selection workspace)";
    case MOSAIC_BSA_ERR_ALIGN: return "tensor base pointers must be 16-byte aligned";
    case MOSAIC_BSA_ERR_LAUNCH: return "HIP kernel launch failed";
    case MOSAIC_BSA_ERR_OP: return "operation not available";
    }
    return "unknown error code";
}
