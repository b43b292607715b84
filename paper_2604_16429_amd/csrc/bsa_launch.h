// Host-side launch entry points of the individual kernels; called only by the
// C-ABI layer after it has validated the arguments.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bsa_device.h"

namespace bsa {

// Query blocks ranked per workgroup by the selection kernel; 0 = m too large.
int select_group_size(int m, int D);

hipError_t launch_pool(bool is_bf16, const void* q, const void* k, float* qbar, float* kbar,
                       const Geom& g, int D, int64_t BH, hipStream_t stream);

// Counts, into *n_bad (device), the entries of sel_idx that the attention
// kernels must not be given: out of [0, m), repeated within a row, or (unless
// own_ok) the row's own block.
hipError_t launch_check_selection(const int32_t* sel_idx, int32_t* n_bad, const Geom& g,
                                  bool own_ok, int64_t BH, hipStream_t stream);

// Pooled means of one key/value-shaped tensor (slices = batch * kv_heads).
hipError_t launch_pool_one(bool is_bf16, const void* x, float* xbar, const Geom& g, int D,
                           int64_t slices, hipStream_t stream);

// Pooling of Q and K, block scores and top-n as one sequence of launches in
// which the pooling of one part of the batch runs beside the ranking of the part
// before.  The scores of a query block stay in LDS; `scratch` is device memory
// of select_scratch_bytes(...) bytes (BKV = batch * kv_heads): a second copy of
// the pooled keys, per slice [D/4][m][4], which the ranking's threads (one key
// block each) read as consecutive 16-byte groups and launch_pool_select leaves
// there (select_interleaves_keys(m)).
size_t select_scratch_bytes(int m, int D, int64_t BH, int64_t BKV);
bool select_interleaves_keys(int m);
hipError_t launch_pool_select(bool is_bf16, const void* q, const void* k, float* qbar,
                              float* kbar, void* scratch, int32_t* sel_idx, const Geom& g, int D,
                              int64_t BH, hipStream_t stream);

// Any tile shape / head dim in {32, 64, 128} / dtype; fp32 vector arithmetic.
hipError_t launch_fwd_generic(bool is_bf16, const void* q, const void* k, const void* v,
                              const int32_t* sel_idx, void* out, float* lse, const Geom& g, int D,
                              int64_t BH, hipStream_t stream);

// bf16 MFMA forward; covers the shapes fwd_mfma_supported() accepts.
bool fwd_mfma_supported(bool is_bf16, const Geom& g, int D);
hipError_t launch_fwd_mfma(const void* q, const void* k, const void* v, const int32_t* sel_idx,
                           void* out, float* lse, const Geom& g, int D, int64_t BH,
                           hipStream_t stream);

// bf16 MFMA forward for head dim 128 (query blocks of 64, 128 or 256 tokens, one
// workgroup of 2, 4 or 8 wavefronts each, K/V tiles shared through LDS).
bool fwd_mfma_d128_supported(bool is_bf16, const Geom& g, int D);
hipError_t launch_fwd_mfma_d128(const void* q, const void* k, const void* v,
                                const int32_t* sel_idx, void* out, float* lse, const Geom& g,
                                int64_t BH, hipStream_t stream);

// Backward with the selection fixed; `delta` is fp32 scratch of B*heads*N floats.
hipError_t launch_bwd(bool is_bf16, const void* q, const void* k, const void* v, const void* out,
                      const float* lse, const void* dout, const int32_t* sel_idx, void* dq,
                      void* dk, void* dv, float* delta, const Geom& g, int D, int64_t BH,
                      hipStream_t stream);

// bf16 MFMA backward (head dim 64 or 128, blocks of 64, 128 or 256 tokens);
// `delta` and `lse2` are fp32 scratch of B*heads*N floats each, `conn` scratch of
// bwd_connection_words(...) 32-bit words (the reverse map of the selection: one
// bit per (query slice, key block, query block)).
bool bwd_mfma_supported(bool is_bf16, const Geom& g, int D);
inline int64_t bwd_connection_words(int m, int64_t BH) { return BH * m * (int64_t)((m + 31) >> 5); }
hipError_t launch_bwd_mfma(const void* q, const void* k, const void* v, const void* out,
                           const float* lse, const void* dout, const int32_t* sel_idx, void* dq,
                           void* dk, void* dv, float* delta, float* lse2, uint32_t* conn,
                           const Geom& g, int D, int64_t BH, hipStream_t stream);

// Three-branch output: coarse branch (softmax over all pooled key blocks times
// pooled values, fp32 [B*heads, m, D]), the block lists of the local branch
// (int32 [B*heads, m, local_h*local_w - 1]) and the gated sum of the branches.
// kbar_il: the channel-interleaved copy of the pooled keys that
// launch_pool_select leaves in its scratch for m <= 512, or NULL.
int coarse_group_size(int m, int D);
hipError_t launch_coarse(const float* qbar, const float* kbar, const float* kbar_il,
                         const float* vbar, float* obar, const Geom& g, int D, int64_t BH,
                         hipStream_t stream);
hipError_t launch_local_lists(int32_t* lists, const Geom& g, int local_h, int local_w,
                              int64_t BH, hipStream_t stream);
hipError_t launch_combine(bool is_bf16, const float* obar, const void* o_fg, const void* o_l,
                          const float* gates, void* out, const Geom& g, int D, int64_t BH,
                          hipStream_t stream);

// Backward of the three-branch output: upstream gradients of the two attention
// branches and the gate gradients; the coarse branch's gradients on the pooled
// tensors, chunk_rows query blocks at a time (a_mat, ds_mat: fp32 scratch
// [B*heads, chunk_rows, m]).
int coarse_bwd_group_size(int m, int D);
hipError_t launch_branch_grads(bool is_bf16, const float* obar, const void* o_fg, const void* o_l,
                               const float* gates, const void* dout, void* do_fg, void* do_l,
                               float* dgates, float* dobar, const Geom& g, int D, int64_t BH,
                               hipStream_t stream);
hipError_t launch_coarse_bwd(const float* qbar, const float* kbar, const float* kbar_il,
                             const float* vbar, const float* dobar, float* a_mat, float* ds_mat, float* dqbar,
                             float* dkbar, float* dvbar, const Geom& g, int D, int64_t BH,
                             int chunk_rows, hipStream_t stream);

// Measurement aid: `workgroups` x 4 wavefronts, each issuing 16 * iters
// v_mfma_f32_32x32x16_bf16 on register operands; sink: workgroups * 256 floats.
hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, hipStream_t stream);

}  // namespace bsa
