"""ctypes front end of the CPU oracle (oracle/bsa_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module,
and this module never imports the product package.

All tensors are numpy arrays: fp32 [B, heads, N, D] inputs (bf16 data widened
exactly to fp32 by the caller), int32 [B, heads, m, n] selections, float64
outputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bsa_oracle.c")
_LIB = os.path.join(_HERE, "libbsa_oracle.so")
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in (
        "batch", "heads", "grid_h", "grid_w", "block_h", "block_w",
        "head_dim", "n_select")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call([
            "gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fopenmp",
            "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_token_of.restype = ctypes.c_int64
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def _shape(batch, heads, grid_h, grid_w, block_h, block_w, head_dim, n_select,
           own_is_candidate=False):
    if grid_h % block_h or grid_w % block_w:
        raise ValueError("tile must divide the grid")
    m = (grid_h // block_h) * (grid_w // block_w)
    if own_is_candidate:          # three-branch form: top-n over all m blocks
        if not 1 <= n_select <= m:
            raise ValueError("n_select must be in [1, m]")
    elif not 0 <= n_select <= m - 1:
        raise ValueError("n_select must be in [0, m-1]")
    return _Shape(batch, heads, grid_h, grid_w, block_h, block_w, head_dim,
                  n_select)


def shape_of(cfg, n_select=None, own_is_candidate=False):
    """oracle shape from any object with the grid-configuration attributes."""
    return _shape(cfg.batch, cfg.heads, cfg.grid_h, cfg.grid_w, cfg.block_h,
                  cfg.block_w, cfg.head_dim,
                  cfg.n_select if n_select is None else n_select, own_is_candidate)


def _f32(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x, x.ctypes.data_as(ctypes.c_void_p)


def _i32(x):
    x = np.ascontiguousarray(x, dtype=np.int32)
    return x, x.ctypes.data_as(ctypes.c_void_p)


def _dims(s):
    N = s.grid_h * s.grid_w
    b = s.block_h * s.block_w
    return s.batch, s.heads, N, s.head_dim, b, N // b


def _check(s, *tensors):
    B, h, N, D, _, _ = _dims(s)
    for t in tensors:
        if t.shape != (B, h, N, D):
            raise ValueError(f"expected {(B, h, N, D)}, got {t.shape}")


def threads() -> int:
    return int(_load().oracle_threads())


def token_of(s, beta: int, tau: int) -> int:
    return int(_load().oracle_token_of(ctypes.byref(s), int(beta), int(tau)))


def pool(s, x):
    """Mean-pooled block representations, fp32 [B, heads, m, D]."""
    B, h, N, D, b, m = _dims(s)
    x, px = _f32(x)
    _check(s, x)
    out = np.empty((B, h, m, D), dtype=np.float32)
    _load().oracle_pool(ctypes.byref(s), px, out.ctypes.data_as(ctypes.c_void_p))
    return out


def scores(s, qbar, kbar):
    """Block-level scores, fp32 [B, heads, m, m] (diagonal included)."""
    B, h, N, D, b, m = _dims(s)
    qbar, pq = _f32(qbar)
    kbar, pk = _f32(kbar)
    out = np.empty((B, h, m, m), dtype=np.float32)
    _load().oracle_scores(ctypes.byref(s), pq, pk,
                          out.ctypes.data_as(ctypes.c_void_p))
    return out


def select_from_pooled(s, qbar, kbar):
    B, h, N, D, b, m = _dims(s)
    qbar, pq = _f32(qbar)
    kbar, pk = _f32(kbar)
    assert qbar.shape == (B, h, m, D) and kbar.shape == (B, h, m, D)
    idx = np.empty((B, h, m, s.n_select), dtype=np.int32)
    _load().oracle_select_from_pooled(ctypes.byref(s), pq, pk,
                                      idx.ctypes.data_as(ctypes.c_void_p))
    return idx


def select(s, q, k):
    """Selected block indices, int32 [B, heads, m, n]."""
    B, h, N, D, b, m = _dims(s)
    q, pq = _f32(q)
    k, pk = _f32(k)
    _check(s, q, k)
    idx = np.empty((B, h, m, s.n_select), dtype=np.int32)
    _load().oracle_select(ctypes.byref(s), pq, pk,
                          idx.ctypes.data_as(ctypes.c_void_p))
    return idx


def fwd(s, q, k, v, sel_idx, scale: float = 0.0):
    """Attention output and log-sum-exp, float64 ([B,h,N,D], [B,h,N])."""
    B, h, N, D, b, m = _dims(s)
    q, pq = _f32(q)
    k, pk = _f32(k)
    v, pv = _f32(v)
    _check(s, q, k, v)
    sel_idx, pi = _i32(sel_idx)
    assert sel_idx.shape == (B, h, m, s.n_select)
    out = np.empty((B, h, N, D), dtype=np.float64)
    lse = np.empty((B, h, N), dtype=np.float64)
    _load().oracle_fwd(ctypes.byref(s), pq, pk, pv, pi, ctypes.c_double(scale),
                       out.ctypes.data_as(ctypes.c_void_p),
                       lse.ctypes.data_as(ctypes.c_void_p))
    return out, lse


def fwd_blocks(s, q, k, v, sel_idx, pairs, scale: float = 0.0):
    """Forward for the listed (batch*head, block) pairs only.

    Returns (out [cnt, b, D], lse [cnt, b]) float64 with rows in in-tile order.
    Works slice by slice on views of the inputs (no copies of the tensors).
    k, v may carry fewer heads than q (grouped query attention: query head a
    reads head a // group).
    """
    B, h, N, D, b, m = _dims(s)
    q, _ = _f32(q)
    k, _ = _f32(k)
    v, _ = _f32(v)
    _check(s, q)
    kv_heads = k.shape[1]
    assert k.shape == v.shape == (B, kv_heads, N, D) and h % kv_heads == 0
    sel_idx, _ = _i32(sel_idx)
    pairs = np.ascontiguousarray(pairs, dtype=np.int64).reshape(-1, 2)
    q3 = q.reshape(B * h, N, D)
    k3, v3 = (x.reshape(B * kv_heads, N, D) for x in (k, v))

    def kv_slice(g):
        e, a = divmod(int(g), h)
        return e * kv_heads + a // (h // kv_heads)
    i3 = sel_idx.reshape(B * h, m, s.n_select)
    sub = _shape(1, 1, s.grid_h, s.grid_w, s.block_h, s.block_w, D, s.n_select)
    out = np.empty((len(pairs), b, D), dtype=np.float64)
    lse = np.empty((len(pairs), b), dtype=np.float64)
    full_o = np.zeros((N, D), dtype=np.float64)
    full_l = np.zeros((N,), dtype=np.float64)
    for g in np.unique(pairs[:, 0]):
        where = np.nonzero(pairs[:, 0] == g)[0]
        blocks = pairs[where, 1]
        p_s = np.ascontiguousarray(np.stack([np.zeros_like(blocks), blocks], axis=1))
        _load().oracle_fwd_blocks(
            ctypes.byref(sub), q3[g].ctypes.data_as(ctypes.c_void_p),
            k3[kv_slice(g)].ctypes.data_as(ctypes.c_void_p),
            v3[kv_slice(g)].ctypes.data_as(ctypes.c_void_p),
            i3[g].ctypes.data_as(ctypes.c_void_p), ctypes.c_double(scale),
            p_s.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(len(p_s)),
            full_o.ctypes.data_as(ctypes.c_void_p), full_l.ctypes.data_as(ctypes.c_void_p))
        for w, i in zip(where, blocks):
            rows = np.array([token_of(s, int(i), t) for t in range(b)], dtype=np.int64)
            out[w] = full_o[rows]
            lse[w] = full_l[rows]
    return out, lse


def block_weights(s, q, k, v, sel_idx, g: int, i: int, scale: float = 0.0):
    """Attention weights P [b, (n+1)*b] of query block i of batch*head g;
    column c*b + tau is token tau of the c-th attended block (c = 0: itself)."""
    B, h, N, D, b, m = _dims(s)
    q, pq = _f32(q)
    k, pk = _f32(k)
    v, pv = _f32(v)
    sel_idx, pi = _i32(sel_idx)
    P = np.empty((b, (s.n_select + 1) * b), dtype=np.float64)
    _load().oracle_block_weights(ctypes.byref(s), pq, pk, pv, pi,
                                 ctypes.c_double(scale), ctypes.c_int64(g),
                                 ctypes.c_int(i),
                                 P.ctypes.data_as(ctypes.c_void_p))
    return P


def bwd(s, q, k, v, dout, sel_idx, scale: float = 0.0):
    """dQ, dK, dV (float64 [B,h,N,D]) with the selection held fixed."""
    B, h, N, D, b, m = _dims(s)
    q, pq = _f32(q)
    k, pk = _f32(k)
    v, pv = _f32(v)
    dout, pd = _f32(dout)
    _check(s, q, k, v, dout)
    sel_idx, pi = _i32(sel_idx)
    dq = np.empty((B, h, N, D), dtype=np.float64)
    dk = np.empty_like(dq)
    dv = np.empty_like(dq)
    _load().oracle_bwd(ctypes.byref(s), pq, pk, pv, pd, pi,
                       ctypes.c_double(scale),
                       dq.ctypes.data_as(ctypes.c_void_p),
                       dk.ctypes.data_as(ctypes.c_void_p),
                       dv.ctypes.data_as(ctypes.c_void_p))
    return dq, dk, dv


def bwd_blocks(s, q, k, v, dout, sel_idx, pairs, scale: float = 0.0):
    """Gradients on sampled blocks, for problems too large for a full pass:
    pairs int64 [cnt, 2] = (batch*heads + head, block).  Returns (dq, dk, dv),
    float64 [cnt, b, D] each, in in-tile token order: dq of the block as a query
    block, dk and dv of the block as a key block (summed over every query block
    of the slice that attends to it)."""
    B, h, N, D, b, m = _dims(s)
    q, pq = _f32(q)
    k, pk = _f32(k)
    v, pv = _f32(v)
    dout, pd = _f32(dout)
    _check(s, q, k, v, dout)
    sel_idx, pi = _i32(sel_idx)
    pairs = np.ascontiguousarray(pairs, dtype=np.int64).reshape(-1, 2)
    assert pairs[:, 0].min() >= 0 and pairs[:, 0].max() < B * h
    assert pairs[:, 1].min() >= 0 and pairs[:, 1].max() < m
    cnt = pairs.shape[0]
    dq = np.empty((cnt, b, D), dtype=np.float64)
    dk = np.empty_like(dq)
    dv = np.empty_like(dq)
    _load().oracle_bwd_blocks(ctypes.byref(s), pq, pk, pv, pd, pi, ctypes.c_double(scale),
                              pairs.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(cnt),
                              dq.ctypes.data_as(ctypes.c_void_p),
                              dk.ctypes.data_as(ctypes.c_void_p),
                              dv.ctypes.data_as(ctypes.c_void_p))
    return dq, dk, dv


# ---------------------------------------------------------------------------
# Grouped query attention (the paper's Attention paragraph: the queries attend
# to a smaller number of shared key-value heads).  Reading taken here: query
# head a reads key/value head a // (heads / kv_heads); pooling, scoring and
# selection stay per query head, on the key head that the query head reads.
# Written out as the definition: give every query head its own copy of the
# key/value head it reads and run the one-head-each path; the gradient of a
# shared head is the sum of the gradients of its copies.
# ---------------------------------------------------------------------------
def expand_kv(x, heads: int):
    """[B, kv_heads, N, D] -> [B, heads, N, D], head a <- x[:, a // group]."""
    kv_heads = x.shape[1]
    if heads % kv_heads:
        raise ValueError("kv_heads must divide heads")
    return np.repeat(np.asarray(x), heads // kv_heads, axis=1)


def reduce_kv(dx, kv_heads: int):
    """[B, heads, N, D] -> [B, kv_heads, N, D]: sum over each group, in
    ascending head order."""
    B, h, N, D = dx.shape
    group = h // kv_heads
    out = np.zeros((B, kv_heads, N, D), dtype=dx.dtype)
    for a in range(h):
        out[:, a // group] += dx[:, a]
    return out


def select_gqa(s, q, k):
    return select(s, q, expand_kv(k, s.heads))


def fwd_gqa(s, q, k, v, sel_idx, scale: float = 0.0):
    return fwd(s, q, expand_kv(k, s.heads), expand_kv(v, s.heads), sel_idx, scale)


def bwd_gqa(s, q, k, v, dout, sel_idx, scale: float = 0.0):
    kv_heads = k.shape[1]
    dq, dk, dv = bwd(s, q, expand_kv(k, s.heads), expand_kv(v, s.heads), dout,
                     sel_idx, scale)
    return dq, reduce_kv(dk, kv_heads), reduce_kv(dv, kv_heads)


# ---------------------------------------------------------------------------
# The paper's three branches (Block-Sparse Attention subsection), summed with
# caller-supplied gate values (aggregation equation of the Native Sparse
# Attention subsection).  Readings taken where the text leaves a choice:
#   * coarse branch: softmax over ALL m blocks of qbar_i . kbar_j / sqrt(d_k)
#     (the printed sum runs over l = 1..m, own block included), applied to the
#     mean-pooled values, the result handed to every token of the block;
#   * selection branch: top-n of that row over all m blocks (own block is a
#     candidate), ranked by the raw pooled dot product (same order), then ONE
#     softmax over the tokens of the selected blocks only;
#   * local branch: plain attention inside "large blocks": aligned groups of
#     local_h x local_w mesh tiles;
#   * gates: values g[B, heads, N, 3] in the order (coarse, selection, local),
#     one scalar per token, head and branch; how they are produced from the
#     layer input is outside the path.
# ---------------------------------------------------------------------------
def select_all(s, q, k):
    """Top-n key blocks per query block over all m blocks, int32 [B,h,m,n]."""
    B, h, N, D, b, m = _dims(s)
    if not 1 <= s.n_select <= m:
        raise ValueError("three-branch selection needs 1 <= n <= m")
    qbar, pq = _f32(pool(s, q))
    kbar, pk = _f32(pool(s, k))
    idx = np.empty((B, h, m, s.n_select), dtype=np.int32)
    _load().oracle_select_all_from_pooled(ctypes.byref(s), pq, pk,
                                          idx.ctypes.data_as(ctypes.c_void_p))
    return idx


def attend_lists(s, q, k, v, lists, scale: float = 0.0):
    """One softmax per token over exactly the listed blocks of its query block;
    lists int32 [B, h, m, cnt].  Returns (out, lse) float64."""
    B, h, N, D, b, m = _dims(s)
    q, pq = _f32(q)
    k, pk = _f32(k)
    v, pv = _f32(v)
    _check(s, q, k, v)
    lists, pl = _i32(lists)
    cnt = lists.shape[-1]
    assert lists.shape == (B, h, m, cnt) and cnt >= 1
    assert lists.min() >= 0 and lists.max() < m
    out = np.empty((B, h, N, D), dtype=np.float64)
    lse = np.empty((B, h, N), dtype=np.float64)
    _load().oracle_attend_lists(ctypes.byref(s), pq, pk, pv, pl, ctypes.c_int(cnt),
                                ctypes.c_double(scale),
                                out.ctypes.data_as(ctypes.c_void_p),
                                lse.ctypes.data_as(ctypes.c_void_p))
    return out, lse


def local_lists(s, local_h: int, local_w: int):
    """Blocks of the large local block that contains block i, ascending;
    int32 [m, local_h*local_w].  Large blocks are aligned groups of
    local_h x local_w mesh tiles."""
    rows, cols = s.grid_h // s.block_h, s.grid_w // s.block_w
    if rows % local_h or cols % local_w:
        raise ValueError("the local group must divide the grid of tiles")
    out = np.empty((rows * cols, local_h * local_w), dtype=np.int32)
    for r in range(rows):
        for c in range(cols):
            r0, c0 = r - r % local_h, c - c % local_w
            out[r * cols + c] = [(r0 + dr) * cols + (c0 + dc)
                                 for dr in range(local_h) for dc in range(local_w)]
    return out


def coarse(s, q, k, v, scale: float = 0.0):
    """Coarse-grained branch: (block outputs float64 [B,h,m,D], block-level
    attention float64 [B,h,m,m]).  Pooled means are the fp32 ones of pool()."""
    D = s.head_dim
    qbar = pool(s, q).astype(np.float64)
    kbar = pool(s, k).astype(np.float64)
    vbar = pool(s, v).astype(np.float64)
    sc = scale if scale > 0 else 1.0 / np.sqrt(D)
    z = sc * np.einsum("ghid,ghjd->ghij", qbar, kbar)
    z -= z.max(axis=-1, keepdims=True)
    a = np.exp(z)
    a /= a.sum(axis=-1, keepdims=True)
    return np.einsum("ghij,ghjd->ghid", a, vbar), a


def block_of_token(s):
    """Block index of every token, int64 [N] (inverse of token_of)."""
    B, h, N, D, b, m = _dims(s)
    out = np.empty(N, dtype=np.int64)
    for beta in range(m):
        for tau in range(b):
            out[token_of(s, beta, tau)] = beta
    return out


def fwd_three_branch(s, q, k, v, gates, local_h: int, local_w: int, scale: float = 0.0,
                     sel=None):
    """out = g_cg * o_cg + g_fg * o_fg + g_l * o_l, float64 [B,h,N,D]; also
    returns the selection and the three branch outputs.  k, v may carry fewer
    heads than q (grouped query attention).  A given `sel` replaces the
    ranking (used to hold the selection fixed)."""
    k, v = expand_kv(k, s.heads), expand_kv(v, s.heads)
    B, h, N, D, b, m = _dims(s)
    gates = np.asarray(gates, dtype=np.float64)
    assert gates.shape == (B, h, N, 3)
    o_blocks, _ = coarse(s, q, k, v, scale)
    o_cg = o_blocks[:, :, block_of_token(s), :]
    if sel is None:
        sel = select_all(s, q, k)
    o_fg, _ = attend_lists(s, q, k, v, sel, scale)
    win = np.broadcast_to(local_lists(s, local_h, local_w), (B, h, m, local_h * local_w))
    o_l, _ = attend_lists(s, q, k, v, win, scale)
    out = gates[..., 0:1] * o_cg + gates[..., 1:2] * o_fg + gates[..., 2:3] * o_l
    return out, sel, (o_cg, o_fg, o_l)


def tile_tokens(s):
    """Token index of every (block, in-tile position), int64 [m, b]."""
    B, h, N, D, b, m = _dims(s)
    return np.array([[token_of(s, beta, tau) for tau in range(b)] for beta in range(m)],
                    dtype=np.int64)


def bwd_three_branch(s, q, k, v, gates, dout, sel, local_h: int, local_w: int,
                     scale: float = 0.0):
    """Gradients of sum(out * dout) with respect to q, k, v and the gates, the
    selection held fixed (no gradient through the top-n; the coarse branch's
    softmax and the pooling are differentiated).  The three-branch definition
    is written out once more with float64 tensor operations (tile means,
    softmax, matrix products over gathered tiles) and differentiated by the
    library's reverse mode.  Returns (dq [B,h,N,D], dk, dv [B,kv_heads,N,D],
    dgates [B,h,N,3], out [B,h,N,D]) as float64 numpy arrays."""
    import torch
    B, h, N, D, b, m = _dims(s)
    kv_heads = k.shape[1]
    group = h // kv_heads
    sc = scale if scale > 0 else 1.0 / np.sqrt(D)
    perm = torch.from_numpy(tile_tokens(s))                         # [m, b]
    tq, tk, tv, tg = (torch.tensor(np.asarray(x), dtype=torch.float64, requires_grad=True)
                      for x in (q, k, v, gates))
    td = torch.tensor(np.asarray(dout), dtype=torch.float64)
    qt = tq[:, :, perm]                                             # [B, h, m, b, D]
    kt = tk[:, :, perm].repeat_interleave(group, dim=1)             # head a <- a // group
    vt = tv[:, :, perm].repeat_interleave(group, dim=1)
    gt, dt = tg[:, :, perm], td[:, :, perm]                         # [B, h, m, b, 3 / D]

    # coarse branch: block-level attention over all m blocks on the tile means
    qbar, kbar, vbar = qt.mean(dim=3), kt.mean(dim=3), vt.mean(dim=3)
    abar = torch.softmax(sc * qbar @ kbar.transpose(-1, -2), dim=-1)
    o_cg = (abar @ vbar)[:, :, :, None, :]                          # same row for the whole tile

    def attend(lists):                                              # lists [B, h, m, cnt]
        idx = torch.from_numpy(np.ascontiguousarray(lists, dtype=np.int64))
        e = torch.arange(B)[:, None, None, None]
        a = torch.arange(h)[None, :, None, None]
        kk = kt[e, a, idx].reshape(B, h, m, -1, D)                  # gathered tiles
        vv = vt[e, a, idx].reshape(B, h, m, -1, D)
        p = torch.softmax(sc * qt @ kk.transpose(-1, -2), dim=-1)
        return p @ vv

    o_fg = attend(sel)
    win = np.broadcast_to(local_lists(s, local_h, local_w), (B, h, m, local_h * local_w))
    o_l = attend(win)
    out_t = gt[..., 0:1] * o_cg + gt[..., 1:2] * o_fg + gt[..., 2:3] * o_l
    (out_t * dt).sum().backward()
    out = np.empty((B, h, N, D), dtype=np.float64)
    out[:, :, perm.numpy()] = out_t.detach().numpy()
    return (tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy(), tg.grad.numpy(), out)
