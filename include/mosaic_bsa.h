/*
 * mosaic_bsa.h -- C ABI of the MI355X (gfx950) block-sparse attention library.
 *
 * The library implements the hot path of the paper's Block-Sparse Attention
 * (Section "Mosaic", subsection "Block-Sparse Attention") on a row-major
 * lat-lon grid:
 *
 *   - N = H*W tokens are partitioned into m = N/b non-overlapping blocks
 *     (Compression paragraph).  A block is a block_h x block_w tile of the
 *     grid, b = block_h*block_w.  Token t = r*W + c lies in block
 *     beta = (r / block_h)*(W / block_w) + (c / block_w); inside a block,
 *     tokens are ordered row-major, tau = (r % block_h)*block_w + (c % block_w).
 *   - mosaic_bsa_select: mean-pools Q and K per block (pooling equation,
 *     phi = mean), scores every pair of blocks with the pooled dot product
 *     (block-level attention equation; its softmax and 1/sqrt(d_k) are
 *     monotone per row, so they do not change the ranking and are skipped)
 *     and keeps the top-n key blocks of every query block (Selection
 *     paragraph).
 *   - mosaic_bsa_fwd: every token of query block i attends, in one softmax,
 *     to all tokens of block i (Local Attention paragraph) and of the n
 *     selected blocks (fine-grained attention equation).
 *   - mosaic_bsa_bwd: gradients of that attention with the selection held
 *     fixed (Appendix "Block-sparse attention implementation", kernel design).
 *   - mosaic_bsa_fwd_three_branch / mosaic_bsa_bwd_three_branch: the
 *     subsection's own output form, three branches (coarse-grained attention
 *     over the pooled blocks, selection, local attention inside large blocks)
 *     with a softmax each, summed with gate values that the caller supplies
 *     (aggregation equation of the Native Sparse Attention subsection), and
 *     its gradients.
 *   - mosaic_bsa_check_selection, mosaic_bsa_probe_mfma: a checker for
 *     caller-made selections and a measurement aid; neither is on the hot path.
 *
 * Conventions common to all entry points
 *   Pointers  q, k, v, out, dout, dq, dk, dv, sel_idx, lse and the workspace
 *             are DEVICE pointers; `params` is a HOST pointer.  The caller
 *             owns every buffer; the library never allocates, frees or keeps
 *             device memory and never synchronises.  All work is enqueued on
 *             `hip_stream` (a hipStream_t passed as void*, NULL = default
 *             stream); buffers must stay valid until that work has finished.
 *   Layout    q, out, dout, dq: [batch, heads, N, head_dim]; k, v, dk, dv:
 *             [batch, kv_heads, N, head_dim] (kv_heads = heads unless grouped
 *             query attention is asked for); contiguous, head_dim fastest,
 *             element type given by params->dtype, base pointers 16-byte
 *             aligned.
 *             sel_idx: int32 [batch, heads, m, n_select].
 *             lse: fp32 [batch, heads, N], natural-log sum of
 *             exp(softmax_scale * q.k) over the attended keys.
 *   Errors    0 on success, a negative MOSAIC_BSA_ERR_* code otherwise.  All
 *             argument checks run on the host before anything is enqueued;
 *             on error nothing has been launched.  Inputs must be finite.
 */
#ifndef MOSAIC_BSA_H
#define MOSAIC_BSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOSAIC_BSA_OK = 0,
    MOSAIC_BSA_ERR_NULL = -1,      /* a required pointer is NULL */
    MOSAIC_BSA_ERR_SHAPE = -2,     /* non-positive size, tile does not divide grid, or
                                      kv_heads does not divide heads */
    MOSAIC_BSA_ERR_NSELECT = -3,   /* n_select outside [0, m - 1] ([1, m] in the
                                      three-branch form) */
    MOSAIC_BSA_ERR_HEAD_DIM = -4,  /* head_dim not in {32, 64, 128} */
    MOSAIC_BSA_ERR_DTYPE = -5,     /* dtype not MOSAIC_BSA_F32 / MOSAIC_BSA_BF16 */
    MOSAIC_BSA_ERR_WORKSPACE = -6, /* workspace missing or too small */
    MOSAIC_BSA_ERR_ALIGN = -7,     /* a tensor base pointer is not 16-byte aligned */
    MOSAIC_BSA_ERR_LAUNCH = -8,    /* HIP refused a launch (see hipGetLastError) */
    MOSAIC_BSA_ERR_OP = -9         /* unknown op for mosaic_bsa_workspace_bytes */
};

enum { MOSAIC_BSA_F32 = 0, MOSAIC_BSA_BF16 = 1 };
enum { MOSAIC_BSA_OP_SELECT = 0, MOSAIC_BSA_OP_FWD = 1, MOSAIC_BSA_OP_BWD = 2 };

/* Statement of the problem, in the paper's terms. */
typedef struct {
    int32_t batch;          /* B */
    int32_t heads;          /* query heads (key/value heads: kv_heads below) */
    int32_t grid_h, grid_w; /* H, W: lat-lon grid, N = H*W tokens */
    int32_t block_h, block_w; /* tile shape; must divide H and W; b <= 1024 */
    int32_t head_dim;       /* d_k, one of 32, 64, 128 */
    int32_t n_select;       /* n selected blocks per query block, 0 <= n <= m-1 */
    int32_t dtype;          /* element type of q/k/v/out/...: MOSAIC_BSA_F32 or _BF16;
                               accumulation and softmax are fp32 in both cases */
    float softmax_scale;    /* <= 0 selects 1/sqrt(head_dim) (fine-grained
                               attention equation) */
    int32_t kv_heads;       /* key/value heads for grouped query attention (the
                               paper's Attention paragraph: queries attend to a
                               number of shared key-value heads); 0 = heads.
                               Must divide heads: query head a uses key/value
                               head a / (heads / kv_heads).  Selection stays
                               per query head. */
} mosaic_bsa_params;

/* Bytes of device workspace that `op` needs for `params`; 0 if none.
 * Returns 0 as well when params is invalid (the op itself reports why). */
size_t mosaic_bsa_workspace_bytes(const mosaic_bsa_params *params, int op);

/*
 * Block selection (pooling equation, block-level attention equation,
 * Selection paragraph).
 *   q         in   device, [B, heads, N, D]
 *   k         in   device, [B, kv_heads, N, D]
 *   sel_idx   out  device, int32 [B, heads, m, n]: for every query block the
 *                  n key blocks j != i with the largest pooled score, ordered
 *                  by (score descending, block index ascending).
 *   workspace      device scratch of mosaic_bsa_workspace_bytes(.., OP_SELECT)
 *                  bytes; on return it holds the pooled q, fp32
 *                  [B, heads, m, D], at its start and the pooled k, fp32
 *                  [B, kv_heads, m, D], at the byte offset of the pooled
 *                  q's size rounded up to a multiple of 256; the rest is
 *                  scratch.
 * Arithmetic is fixed so that indices are reproducible bit for bit: pooled
 * sums are fp32 adds in in-tile row-major order followed by one multiply by
 * 1/b; a score is the fp32 chain acc = fma(qbar[d], kbar[d], acc), d ascending.
 * n_select == 0 is valid and writes nothing.
 */
int mosaic_bsa_select(const mosaic_bsa_params *params, const void *q, const void *k,
                      int32_t *sel_idx, void *workspace, size_t workspace_bytes,
                      void *hip_stream);

/*
 * mosaic_bsa_select for callers that can neither allocate device memory nor
 * hand over a workspace: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same results (bit
 * for bit) as mosaic_bsa_select, but the selection workspace is a fixed array
 * inside the library, MOSAIC_BSA_STATIC_SCRATCH_BYTES per GPU, that lives from
 * the loading of the library to the end of the process; the call allocates
 * and frees nothing.
 *   - A problem whose selection workspace (mosaic_bsa_workspace_bytes(..,
 *     OP_SELECT)) exceeds MOSAIC_BSA_STATIC_SCRATCH_BYTES is rejected with
 *     MOSAIC_BSA_ERR_WORKSPACE before anything is enqueued.
 *   - All calls on one GPU share that GPU's array: calls whose stream work can
 *     overlap on one GPU race with each other.  Nothing in the array has to
 *     start at zero (every part is written before it is read), so consecutive
 *     calls on one stream need nothing between them.
 *   - The first call on a device looks up the array's address
 *     (hipGetSymbolAddress, with that device current); make it outside graph
 *     capture.  The pooled tensors are not handed back to the caller.
 */
#define MOSAIC_BSA_STATIC_SCRATCH_BYTES (32u << 20)
int mosaic_bsa_select_static(const mosaic_bsa_params *params, const void *q, const void *k,
                             int32_t *sel_idx, void *hip_stream);

/*
 * Block-sparse attention forward (fine-grained attention equation over the
 * union of the query block itself and its selected blocks, one softmax).
 *   q         in   device, [B, heads, N, D]
 *   k, v      in   device, [B, kv_heads, N, D]
 *   sel_idx   in   device, int32 [B, heads, m, n]; every entry in [0, m),
 *                  no duplicates within a row, never the row's own block;
 *                  any order.  Entries are trusted: an out-of-range index is
 *                  undefined behaviour.
 *   out       out  device, [B, heads, N, D], same element type as q; must not
 *                  alias an input.
 *   lse       out  device, fp32 [B, heads, N]; may be NULL.
 *   workspace      unused by this op (may be NULL with workspace_bytes 0).
 */
int mosaic_bsa_fwd(const mosaic_bsa_params *params, const void *q, const void *k,
                   const void *v, const int32_t *sel_idx, void *out, float *lse,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward of mosaic_bsa_fwd with sel_idx held fixed (no gradient flows
 * through the top-n choice).
 *   q, out, dout        in   device, [B, heads, N, D]
 *   k, v                in   device, [B, kv_heads, N, D]
 *   lse                 in   device, fp32 [B, heads, N] as written by fwd
 *   sel_idx             in   device, same contract as in mosaic_bsa_fwd
 *   dq                  out  device, [B, heads, N, D], element type of q
 *   dk, dv              out  device, [B, kv_heads, N, D] (summed over the query
 *                            heads that share a key/value head)
 *   workspace                device scratch of
 *                            mosaic_bsa_workspace_bytes(.., OP_BWD) bytes; on
 *                            return its start holds delta_l = dout_l . out_l,
 *                            fp32 [B, heads, N] (the rest is scratch: the
 *                            log-sum-exps in base 2 and the reverse map of the
 *                            selection, one bit per (query slice, key block,
 *                            query block)).
 * dk/dv of a key block are reduced over the query blocks that attend to it in
 * a fixed order (no floating-point atomics): results are run-to-run identical.
 */
int mosaic_bsa_bwd(const mosaic_bsa_params *params, const void *q, const void *k,
                   const void *v, const void *out, const float *lse, const void *dout,
                   const int32_t *sel_idx, void *dq, void *dk, void *dv,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The paper's three-branch output (Block-Sparse Attention subsection:
 * Compression, Selection and Local Attention paragraphs; gated sum of the
 * aggregation equation in the Native Sparse Attention subsection):
 *
 *   o_l = g_cg(l) * o_cg(l) + g_fg(l) * o_fg(l) + g_loc(l) * o_loc(l)
 *
 *   coarse     o_cg(l) = sum_j abar_ij vbar_j for every token l of block i,
 *              abar_i = softmax over ALL m blocks of qbar_i . kbar_j * scale,
 *              vbar_j the mean-pooled values;
 *   selection  S_i = the n largest entries of row i over all m blocks (the
 *              block itself is a candidate; 1 <= n_select <= m; ranked by the
 *              pinned fp32 pooled dot product, ties to the smaller index);
 *              o_fg = one softmax over the tokens of the blocks in S_i only;
 *   local      one softmax over the tokens of the large block that contains
 *              l: the aligned group of local_h x local_w mesh tiles
 *              (local_h divides grid_h / block_h, local_w divides
 *              grid_w / block_w; 1 x 1 = the tile itself);
 *   gates      caller-supplied values, one per token, head and branch.
 *
 *   q             in   device, [B, heads, N, D]
 *   k, v          in   device, [B, kv_heads, N, D]
 *   gates         in   device, fp32 [B, heads, N, 3] in the order (coarse,
 *                      selection, local)
 *   out           out  device, [B, heads, N, D], element type of q
 *   sel_idx       out  device, int32 [B, heads, m, n]: S_i in ranking order
 *   workspace          device scratch of
 *                      mosaic_bsa_three_branch_workspace_bytes(..) bytes (pooled
 *                      tensors, block lists, the two attention branches'
 *                      outputs in the element type of q and their
 *                      log-sum-exps); on return it holds what
 *                      mosaic_bsa_bwd_three_branch needs from the forward.
 * The branch outputs are rounded to the element type of q before the gated
 * sum, which runs in fp32.  Errors as for the other entry points; a local
 * group that does not divide the grid of tiles is MOSAIC_BSA_ERR_SHAPE.
 * mosaic_bsa_three_branch_workspace_bytes returns 0 for invalid arguments.
 */
size_t mosaic_bsa_three_branch_workspace_bytes(const mosaic_bsa_params *params,
                                               int32_t local_h, int32_t local_w);
int mosaic_bsa_fwd_three_branch(const mosaic_bsa_params *params, int32_t local_h,
                                int32_t local_w, const void *q, const void *k,
                                const void *v, const float *gates, void *out,
                                int32_t *sel_idx, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * Backward of mosaic_bsa_fwd_three_branch with sel_idx held fixed: no gradient
 * flows through the top-n choice; the coarse branch's block softmax, the mean
 * pooling and the gates are differentiated.
 *   q, k, v, gates   in   device, as in the forward
 *   dout             in   device, [B, heads, N, D], element type of q
 *   sel_idx          in   device, as written by the forward
 *   fwd_workspace    in   device, the forward's workspace after the forward
 *                         call on the same inputs, contents intact
 *   dq               out  device, [B, heads, N, D], element type of q
 *   dk, dv           out  device, [B, kv_heads, N, D]
 *   dgates           out  device, fp32 [B, heads, N, 3]: dout . branch output
 *   workspace             device scratch of
 *                         mosaic_bsa_three_branch_bwd_workspace_bytes(..) bytes
 * The upstream gradients of the two attention branches (gate * dout) and the
 * branches' partial gradients are rounded to the element type of q; every sum
 * runs in a fixed order (no floating-point atomics).
 */
size_t mosaic_bsa_three_branch_bwd_workspace_bytes(const mosaic_bsa_params *params,
                                                   int32_t local_h, int32_t local_w);
int mosaic_bsa_bwd_three_branch(const mosaic_bsa_params *params, int32_t local_h,
                                int32_t local_w, const void *q, const void *k,
                                const void *v, const float *gates, const void *dout,
                                const int32_t *sel_idx, const void *fwd_workspace,
                                void *dq, void *dk, void *dv, float *dgates,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Checker for selections that were not produced by mosaic_bsa_select: the
 * attention entry points trust sel_idx (an out-of-range index is undefined
 * behaviour), so a caller that builds its own lists can have them counted
 * first.  Not part of the hot path.
 *   sel_idx             in   device, int32 [B, heads, m, n]
 *   own_block_allowed        0: the contract of mosaic_bsa_fwd / _bwd (a row
 *                            never names its own block, n <= m - 1); non-zero:
 *                            the three-branch form's lists (it may, n <= m)
 *   n_bad               out  device, one int32: the number of entries that are
 *                            outside [0, m), repeat an earlier entry of their
 *                            row, or name the own block when that is not
 *                            allowed; 0 means the lists are safe to use.
 */
int mosaic_bsa_check_selection(const mosaic_bsa_params *params, const int32_t *sel_idx,
                               int32_t own_block_allowed, int32_t *n_bad, void *hip_stream);

/*
 * Measurement aid, not part of the attention path: a register-resident bf16
 * matrix-core loop (no loads, no LDS, no vector work) whose rate is the most
 * the matrix pipe sustains on the device at hand.  `workgroups` workgroups of
 * 4 wavefronts each issue 16 * iters 32x32x16 bf16 MFMAs, i.e.
 * workgroups * 4 * 16 * iters * 32768 flop in total; the caller times it.
 *   sink   out  device, workgroups * 256 floats (keeps the loop alive)
 */
int mosaic_bsa_probe_mfma(float *sink, int32_t workgroups, int32_t iters, void *hip_stream);

/* Static, human-readable text for a return code. */
const char *mosaic_bsa_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_BSA_H */
