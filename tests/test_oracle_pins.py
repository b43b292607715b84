"""Pins of the CPU oracle against facts fixed by the paper and by mathematics.

None of these tests touches the GPU library.  Each one is chosen so that a
plausible mistake in the oracle (wrong tile index, dropped block, missing
scale, wrong sign in the gradient, transposed operand, wrong tie-break ...)
fails it.  Citations name the paper's Block-Sparse Attention subsection.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from tests.helpers import (from_tiles, rand_qkv, random_selection, shape_ns,
                           to_tiles)

torch.set_num_threads(4)


# --------------------------------------------------------------------------
# partition (Compression paragraph: m non-overlapping blocks)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("H,W,bh,bw", [(16, 24, 8, 8), (8, 32, 4, 16), (6, 6, 2, 3)])
def test_partition_is_a_bijection_and_matches_reshape(oracle, H, W, bh, bw):
    c = shape_ns(1, 1, H, W, bh, bw, 1, 0)
    s = oracle.shape_of(c)
    toks = np.array([[oracle.token_of(s, i, t) for t in range(c.block_tokens)]
                     for i in range(c.n_blocks)])
    assert sorted(toks.ravel().tolist()) == list(range(H * W))
    grid = np.arange(H * W, dtype=np.float32).reshape(1, 1, H * W, 1)
    assert np.array_equal(to_tiles(grid, c)[0, 0, :, :, 0].astype(np.int64), toks)
    # tokens of a block are spatial neighbours: a bh x bw rectangle
    r, col = toks // W, toks % W
    assert np.all(r.max(1) - r.min(1) == bh - 1)
    assert np.all(col.max(1) - col.min(1) == bw - 1)


# --------------------------------------------------------------------------
# pooling equation (phi = mean)
# --------------------------------------------------------------------------
def test_pool_constant_and_block_id_fields(oracle):
    c = shape_ns(2, 2, 16, 32, 8, 8, 4, 0)
    s = oracle.shape_of(c)
    x = np.full((2, 2, c.n_tokens, 4), 0.3, dtype=np.float32)
    # 64 adds of 0.3f are not exact, but a power-of-two constant is
    x[:] = 0.375
    assert np.all(oracle.pool(s, x) == np.float32(0.375))
    ids = np.arange(c.n_blocks, dtype=np.float32)
    tiles = np.broadcast_to(ids[None, None, :, None, None],
                            (2, 2, c.n_blocks, c.block_tokens, 4))
    pooled = oracle.pool(s, from_tiles(np.ascontiguousarray(tiles), c))
    assert np.array_equal(pooled, np.broadcast_to(ids[None, None, :, None],
                                                  pooled.shape))


def test_pool_plus_minus_pairs_vanish_and_matches_float64_mean(oracle):
    c = shape_ns(1, 3, 24, 16, 8, 8, 5, 0)
    s = oracle.shape_of(c)
    rng = np.random.default_rng(1)
    tiles = rng.standard_normal((1, 3, c.n_blocks, c.block_tokens, 5)).astype(np.float32)
    tiles[..., 1::2, :] = -tiles[..., 0::2, :]
    assert np.all(oracle.pool(s, from_tiles(tiles, c)) == 0.0)
    x = rng.standard_normal((1, 3, c.n_tokens, 5)).astype(np.float32)
    ref = to_tiles(x, c).astype(np.float64).mean(axis=3)
    np.testing.assert_allclose(oracle.pool(s, x), ref, rtol=0, atol=2e-6)


def test_pool_and_scores_exact_in_the_quantised_regime(oracle):
    """Inputs on a 1/4 grid in [-2, 2], b = 64, D = 32: every partial sum,
    mean and partial score fits fp32 exactly, so the oracle must reproduce
    integer arithmetic bit for bit, whatever the summation order."""
    c = shape_ns(1, 2, 32, 64, 8, 8, 32, 4)
    s = oracle.shape_of(c)
    rng = np.random.default_rng(2)
    qi = rng.integers(-8, 9, size=(1, 2, c.n_tokens, 32))
    ki = rng.integers(-8, 9, size=(1, 2, c.n_tokens, 32))
    q, k = (qi / 4).astype(np.float32), (ki / 4).astype(np.float32)
    qsum = to_tiles(qi, c).sum(axis=3)          # integers, units of 1/4
    ksum = to_tiles(ki, c).sum(axis=3)
    qbar, kbar = oracle.pool(s, q), oracle.pool(s, k)
    assert np.array_equal(qbar.astype(np.float64) * 256, qsum)   # mean = sum/(4*64)
    assert np.array_equal(kbar.astype(np.float64) * 256, ksum)
    sc = oracle.scores(s, qbar, kbar)
    exact = np.einsum("ghid,ghjd->ghij", qsum, ksum)             # units of 2^-16
    assert np.array_equal(sc.astype(np.float64) * 65536, exact)
    # ranking by exact integers == oracle selection, with the tie-break rule
    idx = oracle.select(s, q, k)
    for a in range(2):
        for i in range(c.n_blocks):
            cand = [j for j in range(c.n_blocks) if j != i]
            cand.sort(key=lambda j: (-int(exact[0, a, i, j]), j))
            assert idx[0, a, i].tolist() == cand[:4]


def test_scores_agree_with_exact_rational_arithmetic(oracle):
    c = shape_ns(1, 1, 8, 16, 2, 4, 8, 3)
    s = oracle.shape_of(c)
    q, k, _ = rand_qkv(c, 3)
    qbar, kbar = oracle.pool(s, q), oracle.pool(s, k)
    sc = oracle.scores(s, qbar, kbar)[0, 0]
    idx = oracle.select(s, q, k)[0, 0]
    m = c.n_blocks
    fq = [[Fraction(float(x)) for x in row] for row in qbar[0, 0]]
    fk = [[Fraction(float(x)) for x in row] for row in kbar[0, 0]]
    for i in range(m):
        ex = [sum(a * b for a, b in zip(fq[i], fk[j])) for j in range(m)]
        mag = [sum(abs(a * b) for a, b in zip(fq[i], fk[j])) for j in range(m)]
        for j in range(m):
            # fused chain of D terms: error <= D * 2^-24 * sum |terms|
            assert abs(Fraction(float(sc[i, j])) - ex[j]) <= 8 * Fraction(1, 2 ** 24) * mag[j]
        cand = sorted((j for j in range(m) if j != i), key=lambda j: (-ex[j], j))
        gap = min(ex[cand[r]] - ex[cand[r + 1]] for r in range(3))
        if gap > 16 * Fraction(1, 2 ** 24) * max(mag):
            assert idx[i].tolist() == cand[:3]


# --------------------------------------------------------------------------
# selection (Selection paragraph: top-n of the block-level scores)
# --------------------------------------------------------------------------
def test_planted_selection_follows_the_planted_ranking(oracle):
    c = shape_ns(1, 2, 16, 32, 4, 4, 8, 5)
    s = oracle.shape_of(c)
    m = c.n_blocks
    rng = np.random.default_rng(4)
    u = rng.integers(1, 4, size=8).astype(np.float32)            # positive direction
    alpha = rng.permutation(m).astype(np.float32) - 7.0          # distinct integers
    ktiles = np.broadcast_to((alpha[:, None, None] * u)[None, None],
                             (1, 2, m, c.block_tokens, 8))
    qtiles = np.broadcast_to(u[None, None, None, None, :], (1, 2, m, c.block_tokens, 8))
    k = from_tiles(np.ascontiguousarray(ktiles, dtype=np.float32), c)
    q = from_tiles(np.ascontiguousarray(qtiles, dtype=np.float32), c)
    idx = oracle.select(s, q, k)
    order = np.argsort(-alpha, kind="stable")
    for i in range(m):
        want = [j for j in order if j != i][:5]
        assert idx[0, 0, i].tolist() == want and idx[0, 1, i].tolist() == want
    # flipping the sign of Q reverses the ranking (a lost sign would not)
    idx_neg = oracle.select(s, -q, k)
    order_neg = np.argsort(alpha, kind="stable")
    for i in range(m):
        assert idx_neg[0, 0, i].tolist() == [j for j in order_neg if j != i][:5]


def test_all_ties_give_smallest_indices_excluding_self(oracle):
    c = shape_ns(1, 1, 16, 16, 4, 4, 4, 6)
    s = oracle.shape_of(c)
    q, _, _ = rand_qkv(c, 5)
    k = np.ones_like(q)
    idx = oracle.select(s, q, k)[0, 0]
    for i in range(c.n_blocks):
        assert idx[i].tolist() == [j for j in range(c.n_blocks) if j != i][:6]


def test_selection_invariances(oracle):
    c = shape_ns(1, 2, 32, 32, 8, 8, 16, 4)
    s = oracle.shape_of(c)
    q, k, _ = rand_qkv(c, 6)
    idx = oracle.select(s, q, k)
    # power-of-two scaling of Q is exact in fp32: ranking unchanged
    assert np.array_equal(oracle.select(s, q * 8.0, k), idx)
    assert np.array_equal(oracle.select(s, q, k * 0.25), idx)
    # rows: n distinct indices, never the block itself, all in range
    m = c.n_blocks
    assert idx.min() >= 0 and idx.max() < m
    for a in range(2):
        for i in range(m):
            row = idx[0, a, i].tolist()
            assert i not in row and len(set(row)) == 4
    # only pooled means matter: quantised data + zero-mean pattern per tile
    rng = np.random.default_rng(7)
    qq = (rng.integers(-8, 9, size=q.shape) / 4).astype(np.float32)
    kq = (rng.integers(-8, 9, size=q.shape) / 4).astype(np.float32)
    pat = (rng.integers(-4, 5, size=(1, 2, m, 32, 16)) / 4).astype(np.float32)
    pat = np.concatenate([pat, -pat], axis=3)                    # sums to 0 per tile
    base = oracle.select(s, qq, kq)
    assert np.array_equal(oracle.select(s, qq, kq + from_tiles(pat, c)), base)


def test_select_equals_sorting_the_oracle_scores(oracle):
    """Top-n emitted == full sort of every candidate by (score desc, index asc)."""
    c = shape_ns(2, 2, 16, 32, 4, 4, 8, 7)
    s = oracle.shape_of(c)
    q, k, _ = rand_qkv(c, 8)
    sc = oracle.scores(s, oracle.pool(s, q), oracle.pool(s, k))
    idx = oracle.select(s, q, k)
    for e in range(2):
        for a in range(2):
            for i in range(c.n_blocks):
                js = np.array([j for j in range(c.n_blocks) if j != i])
                order = np.lexsort((js, -sc[e, a, i, js].astype(np.float64)))
                assert idx[e, a, i].tolist() == js[order][:7].tolist()


# --------------------------------------------------------------------------
# attention (fine-grained attention equation + local block, one softmax)
# --------------------------------------------------------------------------
def _sdpa(q, k, v, scale=None):
    return torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(),
        torch.from_numpy(v).double(), scale=scale).numpy()


def test_all_blocks_selected_is_dense_attention(oracle):
    c = shape_ns(2, 2, 8, 16, 4, 4, 16, 7)     # m = 8, n = m - 1
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 9)
    idx = oracle.select(s, q, k)
    out, lse = oracle.fwd(s, q, k, v, idx)
    np.testing.assert_allclose(out, _sdpa(q, k, v), rtol=0, atol=1e-12)
    z = np.einsum("ghld,ghtd->ghlt", q.astype(np.float64), k.astype(np.float64)) / 4.0
    np.testing.assert_allclose(
        lse, torch.logsumexp(torch.from_numpy(z), dim=-1).numpy(), rtol=0, atol=1e-12)
    # any order of the selected blocks gives the same result
    out2, _ = oracle.fwd(s, q, k, v, random_selection(c, 10))
    np.testing.assert_allclose(out2, out, rtol=0, atol=1e-13)
    # explicit scale argument is honoured
    out3, _ = oracle.fwd(s, q, k, v, idx, scale=0.7)
    np.testing.assert_allclose(out3, _sdpa(q, k, v, scale=0.7), rtol=0, atol=1e-12)


def test_no_selection_is_block_diagonal_attention(oracle):
    c = shape_ns(1, 2, 8, 12, 4, 3, 8, 0)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 11)
    idx = np.zeros((1, 2, c.n_blocks, 0), dtype=np.int32)
    out, _ = oracle.fwd(s, q, k, v, idx)
    ref = _sdpa(to_tiles(q, c), to_tiles(k, c), to_tiles(v, c))
    np.testing.assert_allclose(to_tiles(out, c), ref, rtol=0, atol=1e-12)


def test_sparse_attention_equals_library_attention_over_gathered_tiles(oracle):
    """For an arbitrary valid selection, each query tile's result equals plain
    softmax attention over the concatenation of its own and its selected
    tiles (gathered here by reshape, not by the oracle's index formula)."""
    c = shape_ns(2, 2, 12, 16, 4, 4, 8, 3)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 12, scale=1.5)
    idx = random_selection(c, 13)
    out, lse = oracle.fwd(s, q, k, v, idx)
    qt, kt, vt, ot = (to_tiles(x, c) for x in (q, k, v, out))
    lt = to_tiles(lse[..., None], c)[..., 0]
    for e in range(2):
        for a in range(2):
            for i in range(c.n_blocks):
                blocks = [i] + idx[e, a, i].tolist()
                kk = np.concatenate([kt[e, a, j] for j in blocks])
                vv = np.concatenate([vt[e, a, j] for j in blocks])
                np.testing.assert_allclose(ot[e, a, i], _sdpa(qt[e, a, i], kk, vv),
                                           rtol=0, atol=1e-12)
                z = qt[e, a, i].astype(np.float64) @ kk.astype(np.float64).T / np.sqrt(8.0)
                ref_lse = torch.logsumexp(torch.from_numpy(z), dim=-1).numpy()
                np.testing.assert_allclose(lt[e, a, i], ref_lse, rtol=0, atol=1e-12)


def test_rows_sum_to_one(oracle):
    c = shape_ns(1, 2, 16, 16, 4, 4, 8, 5)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 14, scale=2.0)
    idx = oracle.select(s, q, k)
    const = np.linspace(-1, 1, 8).astype(np.float32)
    out, _ = oracle.fwd(s, q, k, np.broadcast_to(const, v.shape).copy(), idx)
    np.testing.assert_allclose(out, np.broadcast_to(const.astype(np.float64), out.shape),
                               rtol=0, atol=1e-14)
    P = oracle.block_weights(s, q, k, v, idx, 1, 3)
    assert P.shape == (16, 6 * 16) and np.all(P >= 0)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-14)


def test_backward_on_sampled_blocks(oracle):
    """bwd_blocks (gradients of single blocks, for full-size checks) against the
    library's reverse mode over the gathered-tile attention written with float64
    tensor operations, and against the full closed-form pass."""
    import torch
    c = shape_ns(2, 2, 12, 16, 3, 4, 8, 3)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 2121)
    dout = rand_qkv(c, 2122)[0]
    idx = random_selection(c, 9)
    pairs = np.array([[0, 0], [1, 5], [3, 15], [2, 7], [3, 0]])
    dq, dk, dv = oracle.bwd_blocks(s, q, k, v, dout, idx, pairs)
    # library autograd on the definition: per query block, softmax over its gathered tiles
    tq, tk, tv = (torch.tensor(to_tiles(x, c).astype(np.float64), requires_grad=True)
                  for x in (q, k, v))
    td = torch.tensor(to_tiles(dout, c).astype(np.float64))
    B, h, m, b, D = tq.shape
    loss = 0.0
    for e in range(B):
        for a in range(h):
            for i in range(m):
                blocks = [i] + idx[e, a, i].tolist()
                kk = torch.cat([tk[e, a, j] for j in blocks])
                vv = torch.cat([tv[e, a, j] for j in blocks])
                o = torch.softmax(tq[e, a, i] @ kk.T / np.sqrt(D), dim=-1) @ vv
                loss = loss + (o * td[e, a, i]).sum()
    loss.backward()
    for w, (g, x) in enumerate(pairs):
        e, a = divmod(int(g), h)
        np.testing.assert_allclose(dq[w], tq.grad[e, a, x].numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(dk[w], tk.grad[e, a, x].numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(dv[w], tv.grad[e, a, x].numpy(), rtol=0, atol=1e-12)
    # and the full pass
    fq, fk, fv = oracle.bwd(s, q, k, v, dout, idx)
    for w, (g, x) in enumerate(pairs):
        e, a = divmod(int(g), h)
        for got, full in ((dq, fq), (dk, fk), (dv, fv)):
            np.testing.assert_allclose(got[w], to_tiles(full, c)[e, a, x], rtol=0, atol=1e-13)


def test_block_weights_columns_follow_the_gathered_tiles(oracle):
    """Column c * b + tau of the weights of query block i belongs to in-tile
    position tau of the c-th attended block (block i itself, then its selected
    blocks in the order given): pinned against the library softmax over the
    tiles gathered in exactly that order, and against the output they imply."""
    import torch
    c = shape_ns(1, 2, 12, 20, 3, 4, 8, 4)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 1717)
    idx = random_selection(c, 5)
    g, i = 1, 7
    P = oracle.block_weights(s, q, k, v, idx, g, i)
    b, D = c.block_tokens, c.head_dim
    qt, kt, vt = (torch.from_numpy(to_tiles(x, c)[0, g].astype(np.float64)) for x in (q, k, v))
    blocks = [i] + idx[0, g, i].tolist()
    kk = torch.cat([kt[j] for j in blocks])            # [(n+1) b, D], block-major, tau inside
    vv = torch.cat([vt[j] for j in blocks])
    w = torch.softmax(qt[i] @ kk.T / np.sqrt(D), dim=-1).numpy()
    assert P.shape == (b, len(blocks) * b)
    np.testing.assert_allclose(P, w, rtol=0, atol=1e-14)
    out, _ = oracle.fwd(s, q, k, v, idx)
    np.testing.assert_allclose(P @ vv.numpy(), to_tiles(out, c)[0, g, i], rtol=0, atol=1e-13)
    # a column order that ignores the selection's order would fail here
    assert np.abs(P[:, b:2 * b] - w[:, 2 * b:3 * b]).max() > 1e-6


def test_unselected_blocks_do_not_matter(oracle):
    c = shape_ns(1, 1, 16, 16, 4, 4, 8, 3)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 15)
    idx = oracle.select(s, q, k)
    out, lse = oracle.fwd(s, q, k, v, idx)
    i = 5
    untouched = [j for j in range(c.n_blocks) if j != i and j not in idx[0, 0, i]]
    kt, vt = to_tiles(k, c).copy(), to_tiles(v, c).copy()
    kt[0, 0, untouched] = 7.0
    vt[0, 0, untouched] = -3.0
    out2, lse2 = oracle.fwd(s, q, from_tiles(kt, c), from_tiles(vt, c), idx)
    assert np.array_equal(to_tiles(out, c)[0, 0, i], to_tiles(out2, c)[0, 0, i])
    # ... while a selected block does
    kt2 = to_tiles(k, c).copy()
    kt2[0, 0, idx[0, 0, i, 0]] += 1.0
    out3, _ = oracle.fwd(s, q, from_tiles(kt2, c), v, idx)
    assert not np.array_equal(to_tiles(out, c)[0, 0, i], to_tiles(out3, c)[0, 0, i])


def test_single_token_blocks_without_selection_return_v(oracle):
    c = shape_ns(1, 1, 4, 4, 1, 1, 8, 0)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 16)
    out, lse = oracle.fwd(s, q, k, v, np.zeros((1, 1, 16, 0), np.int32))
    assert np.array_equal(out, v.astype(np.float64))
    z = (q.astype(np.float64) * k.astype(np.float64)).sum(-1) / np.sqrt(8.0)
    np.testing.assert_allclose(lse, z, rtol=0, atol=1e-14)


def test_fwd_blocks_matches_full_forward(oracle):
    c = shape_ns(2, 2, 16, 16, 4, 4, 8, 3)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 17)
    idx = oracle.select(s, q, k)
    out, lse = oracle.fwd(s, q, k, v, idx)
    pairs = np.array([[0, 0], [3, 5], [1, 15], [3, 2]])
    o_s, l_s = oracle.fwd_blocks(s, q, k, v, idx, pairs)
    ot = to_tiles(out, c).reshape(4, 16, 16, 8)
    lt = to_tiles(lse[..., None], c).reshape(4, 16, 16)
    for w, (g, i) in enumerate(pairs):
        assert np.array_equal(o_s[w], ot[g, i]) and np.array_equal(l_s[w], lt[g, i])


# --------------------------------------------------------------------------
# backward with the selection held fixed (Appendix, kernel design paragraph)
# --------------------------------------------------------------------------
def _torch_sparse_loss(q, k, v, dout, idx, c):
    """sum(O * dO) of the block-sparse attention, built from torch fp64 ops on
    reshape-gathered tiles; autograd supplies the reference gradients."""
    gh, gw = c.grid_h // c.block_h, c.grid_w // c.block_w

    def tiles(x):
        B, h, N, D = x.shape
        t = x.reshape(B, h, gh, c.block_h, gw, c.block_w, D).permute(0, 1, 2, 4, 3, 5, 6)
        return t.reshape(B, h, gh * gw, c.block_tokens, D)

    qt, kt, vt, dt = tiles(q), tiles(k), tiles(v), tiles(dout)
    loss = 0.0
    for e in range(c.batch):
        for a in range(c.heads):
            for i in range(c.n_blocks):
                blocks = [i] + idx[e, a, i].tolist()
                kk = torch.cat([kt[e, a, j] for j in blocks])
                vv = torch.cat([vt[e, a, j] for j in blocks])
                p = torch.softmax(qt[e, a, i] @ kk.T / np.sqrt(c.head_dim), dim=-1)
                loss = loss + ((p @ vv) * dt[e, a, i]).sum()
    return loss


@pytest.mark.parametrize("n_select", [2, 5])       # 5 = m - 1: dense gradient
def test_bwd_matches_autograd_of_gathered_attention(oracle, n_select):
    c = shape_ns(1, 2, 6, 8, 3, 2, 8, n_select)    # m = 8, b = 6
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 18)
    dout = rand_qkv(c, 19)[0]
    idx = random_selection(c, 20)
    dq, dk, dv = oracle.bwd(s, q, k, v, dout, idx)
    tq, tk, tv = (torch.from_numpy(x).double().requires_grad_() for x in (q, k, v))
    _torch_sparse_loss(tq, tk, tv, torch.from_numpy(dout).double(), idx, c).backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-12)


def test_bwd_matches_central_differences_of_the_oracle_forward(oracle):
    c = shape_ns(1, 1, 4, 8, 2, 2, 4, 2)
    s = oracle.shape_of(c)
    rng = np.random.default_rng(21)
    # values on a 2^-6 grid so that x +- 2^-9 is exact in fp32
    q, k, v, dout = ((rng.integers(-96, 97, size=(1, 1, 32, 4)) / 64).astype(np.float32)
                     for _ in range(4))
    idx = random_selection(c, 22)
    dq, dk, dv = oracle.bwd(s, q, k, v, dout, idx)
    hstep = 2.0 ** -9

    def loss(qq, kk, vv):
        return float((oracle.fwd(s, qq, kk, vv, idx)[0] * dout).sum())

    for name, grad in (("q", dq), ("k", dk), ("v", dv)):
        for pos in [(0, 0, 0, 0), (0, 0, 13, 2), (0, 0, 31, 3), (0, 0, 6, 1)]:
            args = {"q": q.copy(), "k": k.copy(), "v": v.copy()}
            args[name][pos] += hstep
            up = loss(args["q"], args["k"], args["v"])
            args[name][pos] -= 2 * hstep
            dn = loss(args["q"], args["k"], args["v"])
            fd = (up - dn) / (2 * hstep)
            assert abs(fd - grad[pos]) <= 1e-5 * max(1.0, abs(fd)), (name, pos)


def test_softmax_jacobian_rows_vanish(oracle):
    """sum_t dS_lt = 0 for every query row, hence sum_t dK_t = 0: adding one
    vector to every key changes no attention weight."""
    c = shape_ns(1, 1, 8, 16, 4, 4, 8, 3)      # m = 8, sparse
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 23)
    dout = rand_qkv(c, 24)[0]
    idx = oracle.select(s, q, k)
    dq, dk, dv = oracle.bwd(s, q, k, v, dout, idx)
    np.testing.assert_allclose(dk.sum(axis=2), 0.0, rtol=0, atol=1e-12)
    # dV is P^T dO: column sums of P are recovered with dO = 1
    ones = np.ones_like(dout)
    _, _, dv1 = oracle.bwd(s, q, k, v, ones, idx)
    np.testing.assert_allclose(dv1.sum(axis=2), c.n_tokens, rtol=0, atol=1e-10)


# --------------------------------------------------------------------------
# grouped query attention (Attention paragraph: shared key-value heads)
# --------------------------------------------------------------------------
def _kv(c, seed, kv_heads):
    """Key/value tensors [B, kv_heads, N, D]."""
    rng = np.random.default_rng(seed)
    shp = (c.batch, kv_heads, c.n_tokens, c.head_dim)
    return tuple(rng.standard_normal(shp).astype(np.float32) for _ in range(2))


def test_gqa_all_blocks_selected_is_library_grouped_attention(oracle):
    """n = m - 1: the result is dense attention, which the library computes
    with its own grouped-head convention (query head a reads head a // group)."""
    c = shape_ns(2, 6, 8, 8, 4, 4, 16, 3)       # m = 4, 6 query heads on 2 kv heads
    s = oracle.shape_of(c)
    q = rand_qkv(c, 40)[0]
    k, v = _kv(c, 41, 2)
    idx = oracle.select_gqa(s, q, k)
    out, _ = oracle.fwd_gqa(s, q, k, v, idx)
    tq, tk, tv = (torch.from_numpy(x).double() for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, enable_gqa=True)
    np.testing.assert_allclose(out, ref.numpy(), rtol=0, atol=1e-12)
    # gradients of sum(O * dO) against the library's autograd
    dout = rand_qkv(c, 42)[0]
    dq, dk, dv = oracle.bwd_gqa(s, q, k, v, dout, idx)
    tq, tk, tv = (t.requires_grad_() for t in (tq, tk, tv))
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, enable_gqa=True)
    (o * torch.from_numpy(dout).double()).sum().backward()
    assert dk.shape == k.shape and dv.shape == v.shape
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-12)


def test_gqa_head_by_head_equals_single_head_problems(oracle):
    """Sparse case: query head a of the grouped problem is the one-head
    problem on (q[:, a], k[:, a // group], v[:, a // group]), picked out here by
    indexing; the gradient of a shared head is the sum over its query heads."""
    c = shape_ns(1, 4, 12, 16, 4, 4, 8, 3)      # m = 12
    s = oracle.shape_of(c)
    q = rand_qkv(c, 43)[0]
    k, v = _kv(c, 44, 2)
    dout = rand_qkv(c, 45)[0]
    idx = oracle.select_gqa(s, q, k)
    out, lse = oracle.fwd_gqa(s, q, k, v, idx)
    dq, dk, dv = oracle.bwd_gqa(s, q, k, v, dout, idx)
    c1 = shape_ns(1, 1, 12, 16, 4, 4, 8, 3)
    s1 = oracle.shape_of(c1)
    dk_sum, dv_sum = np.zeros_like(dk), np.zeros_like(dv)
    for a in range(4):
        u = a // 2
        q1, k1, v1, d1 = q[:, a:a + 1], k[:, u:u + 1], v[:, u:u + 1], dout[:, a:a + 1]
        idx1 = oracle.select(s1, q1, k1)
        assert np.array_equal(idx1, idx[:, a:a + 1])
        o1, l1 = oracle.fwd(s1, q1, k1, v1, idx1)
        np.testing.assert_array_equal(o1, out[:, a:a + 1])
        np.testing.assert_array_equal(l1, lse[:, a:a + 1])
        g = oracle.bwd(s1, q1, k1, v1, d1, idx1)
        np.testing.assert_array_equal(g[0], dq[:, a:a + 1])
        dk_sum[:, u:u + 1] += g[1]
        dv_sum[:, u:u + 1] += g[2]
    np.testing.assert_allclose(dk, dk_sum, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv, dv_sum, rtol=0, atol=1e-13)
    # the two query heads of a group see the same keys but select differently
    assert not np.array_equal(idx[:, 0], idx[:, 1])
    # the sampled forward reads the shared heads in place
    pairs = np.array([[0, 3], [1, 0], [2, 11], [3, 7]])
    o_s, l_s = oracle.fwd_blocks(s, q, k, v, idx, pairs)
    ot, lt = to_tiles(out, c), to_tiles(lse[..., None], c)[..., 0]
    for w, (g, i) in enumerate(pairs):
        np.testing.assert_array_equal(o_s[w], ot[0, g, i])
        np.testing.assert_array_equal(l_s[w], lt[0, g, i])


def test_gqa_with_one_head_per_group_is_the_plain_path(oracle):
    c = shape_ns(1, 3, 8, 8, 4, 4, 8, 2)
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 46)
    idx = oracle.select(s, q, k)
    assert np.array_equal(oracle.select_gqa(s, q, k), idx)
    np.testing.assert_array_equal(oracle.fwd_gqa(s, q, k, v, idx)[0],
                                  oracle.fwd(s, q, k, v, idx)[0])


# --------------------------------------------------------------------------
# the three branches and their gated sum (Block-Sparse Attention subsection;
# aggregation equation of the Native Sparse Attention subsection)
# --------------------------------------------------------------------------
def test_coarse_branch_with_single_token_blocks_is_dense_attention(oracle):
    c = shape_ns(1, 2, 4, 6, 1, 1, 8, 1)
    s = oracle.shape_of(c, own_is_candidate=True)
    q, k, v = rand_qkv(c, 50)
    o_blocks, a = oracle.coarse(s, q, k, v)
    np.testing.assert_allclose(o_blocks, _sdpa(q, k, v), rtol=0, atol=1e-12)
    np.testing.assert_allclose(a.sum(-1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.coarse(s, q, k, v, scale=0.3)[0],
                               _sdpa(q, k, v, scale=0.3), rtol=0, atol=1e-12)


def test_coarse_branch_is_library_attention_of_the_tile_means(oracle):
    c = shape_ns(2, 2, 8, 12, 4, 3, 8, 1)
    s = oracle.shape_of(c, own_is_candidate=True)
    q, k, v = rand_qkv(c, 51)
    qb, kb, vb = (to_tiles(x, c).astype(np.float64).mean(axis=3) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(qb), torch.from_numpy(kb), torch.from_numpy(vb),
        scale=1.0 / np.sqrt(8.0)).numpy()       # scale uses d_k, not the block size
    np.testing.assert_allclose(oracle.coarse(s, q, k, v)[0], ref, rtol=0, atol=2e-6)


def test_select_all_ranks_every_block_own_included(oracle):
    c = shape_ns(1, 2, 8, 16, 4, 4, 16, 8)      # m = 8 = n
    s = oracle.shape_of(c, own_is_candidate=True)
    q, k, v = rand_qkv(c, 52)
    full = oracle.select_all(s, q, k)
    sc = oracle.scores(s, oracle.pool(s, q), oracle.pool(s, k))
    for a in range(2):
        for i in range(8):
            order = np.lexsort((np.arange(8), -sc[0, a, i].astype(np.float64)))
            assert np.array_equal(full[0, a, i], order)
    # a shorter list is a prefix of the full ranking
    s3 = oracle.shape_of(c, n_select=3, own_is_candidate=True)
    assert np.array_equal(oracle.select_all(s3, q, k), full[..., :3])
    # dropping the own block gives the ranking of the single-softmax form
    s7 = oracle.shape_of(c, n_select=7)
    others = oracle.select(s7, q, k)
    for a in range(2):
        for i in range(8):
            assert np.array_equal(full[0, a, i][full[0, a, i] != i], others[0, a, i])
    # a query block whose own key block scores highest selects itself first
    assert (full[..., 0] == np.arange(8)).sum() < 16      # ... but not always: no special case


def test_attend_lists_reduces_to_known_cases(oracle):
    c = shape_ns(1, 2, 8, 12, 4, 4, 8, 2)       # m = 6
    s = oracle.shape_of(c)
    q, k, v = rand_qkv(c, 53, scale=1.3)
    idx = random_selection(c, 54)
    own = np.broadcast_to(np.arange(6, dtype=np.int32)[None, None, :, None], (1, 2, 6, 1))
    # own block in front of the selection: the single-softmax forward
    out, lse = oracle.attend_lists(s, q, k, v, np.concatenate([own, idx], axis=-1))
    ref, ref_lse = oracle.fwd(s, q, k, v, idx)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-13)
    # every block listed (any order): dense attention
    rng = np.random.default_rng(55)
    everything = np.stack([rng.permutation(6) for _ in range(12)]).reshape(1, 2, 6, 6)
    np.testing.assert_allclose(oracle.attend_lists(s, q, k, v, everything)[0], _sdpa(q, k, v),
                               rtol=0, atol=1e-12)
    # the selection alone: library attention over the gathered tiles, own block absent
    out, _ = oracle.attend_lists(s, q, k, v, idx)
    qt, kt, vt, ot = (to_tiles(x, c) for x in (q, k, v, out))
    for a in range(2):
        for i in range(6):
            kk = np.concatenate([kt[0, a, j] for j in idx[0, a, i]])
            vv = np.concatenate([vt[0, a, j] for j in idx[0, a, i]])
            np.testing.assert_allclose(ot[0, a, i], _sdpa(qt[0, a, i], kk, vv), rtol=0, atol=1e-12)


def test_local_branch_is_block_diagonal_attention_of_the_large_blocks(oracle):
    c = shape_ns(1, 2, 8, 24, 2, 4, 8, 1)       # tiles 2 x 4, large blocks of 2 x 3 tiles
    s = oracle.shape_of(c, own_is_candidate=True)
    q, k, v = rand_qkv(c, 56)
    win = oracle.local_lists(s, 2, 3)
    assert win.shape == (c.n_blocks, 6)
    for i in range(c.n_blocks):
        assert i in win[i] and len(set(win[i])) == 6
    out, _ = oracle.attend_lists(s, q, k, v, np.broadcast_to(win, (1, 2) + win.shape))
    big = shape_ns(1, 2, 8, 24, 4, 12, 8, 0)    # the same large blocks as tiles of their own
    ref = _sdpa(to_tiles(q, big), to_tiles(k, big), to_tiles(v, big))
    np.testing.assert_allclose(to_tiles(out, big), ref, rtol=0, atol=1e-12)


def test_three_branch_sum_follows_the_gates(oracle):
    c = shape_ns(2, 4, 8, 16, 2, 4, 8, 3, kv_heads=2)     # grouped: 4 query heads on 2
    s = oracle.shape_of(c, own_is_candidate=True)
    q = rand_qkv(c, 57)[0]
    k, v = _kv(c, 58, 2)
    rng = np.random.default_rng(59)
    gates = rng.uniform(0.0, 1.0, size=(2, 4, c.n_tokens, 3))
    out, sel, (o_cg, o_fg, o_l) = oracle.fwd_three_branch(s, q, k, v, gates, 2, 2)
    # one-hot gates isolate each branch
    for br, o in enumerate((o_cg, o_fg, o_l)):
        g1 = np.zeros_like(gates)
        g1[..., br] = 1.0
        np.testing.assert_array_equal(oracle.fwd_three_branch(s, q, k, v, g1, 2, 2)[0], o)
    np.testing.assert_allclose(
        out, gates[..., 0:1] * o_cg + gates[..., 1:2] * o_fg + gates[..., 2:3] * o_l,
        rtol=0, atol=1e-14)
    # the coarse output is constant inside a tile and differs between tiles
    t = to_tiles(o_cg, c)
    assert np.array_equal(t, np.broadcast_to(t[:, :, :, :1], t.shape))
    assert np.abs(t[:, :, 0, 0] - t[:, :, 1, 0]).max() > 1e-3
    # branches of query head a are those of the one-head problem on kv head a // 2
    c1 = shape_ns(2, 1, 8, 16, 2, 4, 8, 3)
    s1 = oracle.shape_of(c1, own_is_candidate=True)
    for a in range(4):
        u = a // 2
        o1, sel1, _ = oracle.fwd_three_branch(s1, q[:, a:a + 1], k[:, u:u + 1], v[:, u:u + 1],
                                              gates[:, a:a + 1], 2, 2)
        assert np.array_equal(sel1, sel[:, a:a + 1])
        np.testing.assert_array_equal(o1, out[:, a:a + 1])
    # values that do not depend on the token come back scaled by the sum of the gates
    vc = np.broadcast_to(rng.standard_normal((2, 2, 1, 8)).astype(np.float32), v.shape)
    outc = oracle.fwd_three_branch(s, q, k, vc, gates, 2, 2)[0]
    np.testing.assert_allclose(outc, gates.sum(-1, keepdims=True) * np.repeat(vc, 2, axis=1),
                               rtol=0, atol=1e-6)


def test_three_branch_gradients(oracle):
    """The reverse-mode gradients of the three-branch form: its forward value
    equals the loop-written forward, and the gradients match central
    differences of THAT forward (selection held fixed) for every input."""
    c = shape_ns(1, 4, 8, 16, 2, 4, 8, 3, kv_heads=2)      # m = 8, b = 8
    s = oracle.shape_of(c, own_is_candidate=True)
    rng = np.random.default_rng(60)
    # values on a 2^-6 grid so that x +- 2^-9 is exact in fp32
    q, dout = ((rng.integers(-96, 97, size=(1, 4, 128, 8)) / 64).astype(np.float32)
               for _ in range(2))
    k, v = ((rng.integers(-96, 97, size=(1, 2, 128, 8)) / 64).astype(np.float32)
            for _ in range(2))
    gates = (rng.integers(8, 65, size=(1, 4, 128, 3)) / 64).astype(np.float32)
    out_ref, sel, _ = oracle.fwd_three_branch(s, q, k, v, gates, 2, 2)
    dq, dk, dv, dg, out = oracle.bwd_three_branch(s, q, k, v, gates, dout, sel, 2, 2)
    np.testing.assert_allclose(out, out_ref, rtol=0, atol=1e-6)   # fp32 pooled means vs float64
    assert dk.shape == k.shape and dv.shape == v.shape and dg.shape == gates.shape
    hstep = 2.0 ** -9

    def loss(**kw):
        a = dict(q=q, k=k, v=v, gates=gates)
        a.update(kw)
        o = oracle.fwd_three_branch(s, a["q"], a["k"], a["v"], a["gates"], 2, 2, sel=sel)[0]
        return float((o * dout).sum())

    for name, x, grad, spots in (
            ("q", q, dq, [(0, 0, 0, 0), (0, 3, 77, 5), (0, 1, 127, 7)]),
            ("k", k, dk, [(0, 0, 5, 1), (0, 1, 64, 3), (0, 1, 127, 0)]),
            ("v", v, dv, [(0, 0, 9, 2), (0, 1, 100, 6)]),
            ("gates", gates, dg, [(0, 0, 0, 0), (0, 2, 50, 1), (0, 3, 127, 2)])):
        for pos in spots:
            up, dn = x.copy(), x.copy()
            up[pos] += hstep
            dn[pos] -= hstep
            fd = (loss(**{name: up}) - loss(**{name: dn})) / (2 * hstep)
            assert abs(fd - grad[pos]) <= 2e-5 * max(1.0, abs(fd)), (name, pos, fd, grad[pos])
    # gradient of a gate is the branch output dotted with the upstream gradient
    _, _, (o_cg, o_fg, o_l) = oracle.fwd_three_branch(s, q, k, v, gates, 2, 2, sel=sel)
    for br, o in enumerate((o_cg, o_fg, o_l)):
        np.testing.assert_allclose(dg[..., br], (o * dout).sum(-1), rtol=0, atol=1e-6)
