"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on the same seeded inputs.

Bars: selected indices bit-exact (element for element, in the emitted order);
outputs within 1e-5 of max|O| in fp32 mode and within 2e-2 max-abs in bf16
mode; lse within 1e-3 (bf16) / 1e-5 relative (fp32).  The matrix-core kernels
round the attention weights to bf16 (nearest even) for the PV product and sum
the normaliser from the fp32 weights, so lse carries fp32 noise only."""
import dataclasses

import numpy as np
import pytest
import torch

from inputs.fields import get_config, make_problem, round_to_bf16
from tests.helpers import rand_qkv, random_selection, shape_ns, to_tiles

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_util
    return gpu_util


def check_out(cfg, out_gpu, lse_gpu, out_ref, lse_ref):
    if cfg.dtype == "bf16":
        err = np.abs(out_gpu - out_ref).max()
        assert err <= 2e-2, f"bf16 max-abs error {err}"
        assert np.abs(lse_gpu - lse_ref).max() <= 1e-3
    else:
        rel = np.abs(out_gpu - out_ref).max() / max(np.abs(out_ref).max(), 1e-30)
        assert rel <= 1e-5, f"fp32 relative error {rel}"
        assert np.abs(lse_gpu - lse_ref).max() <= 1e-5 * max(1.0, np.abs(lse_ref).max())


def full_parity(G, oracle, cfg, q, k, v):
    s = oracle.shape_of(cfg)
    idx_ref = oracle.select(s, q, k)
    idx_gpu = G.gpu_select(cfg, q, k)
    assert np.array_equal(idx_gpu, idx_ref)
    out_ref, lse_ref = oracle.fwd(s, q, k, v, idx_ref)
    out_gpu, lse_gpu = G.gpu_fwd(cfg, q, k, v, idx_gpu)
    check_out(cfg, out_gpu, lse_gpu, out_ref, lse_ref)


def test_config1_tiny_grid_fp32(G, oracle):
    p = make_problem(1)
    full_parity(G, oracle, p.cfg, p.q, p.k, p.v)


def test_config2_global_grid_bf16(G, oracle):
    p = make_problem(2)
    full_parity(G, oracle, p.cfg, p.q, p.k, p.v)


def test_config3_ensemble_reduced_batch(G, oracle):
    p = make_problem(3, batch=2, heads=2)
    full_parity(G, oracle, p.cfg, p.q, p.k, p.v)


def test_config5_forward_reduced_batch(G, oracle):
    p = make_problem(5, batch=1, heads=2)
    full_parity(G, oracle, p.cfg, p.q, p.k, p.v)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("H,W,bh,bw,D,n", [
    (12, 18, 6, 6, 32, 3),      # b = 36: ragged against the 64-row chunk
    (16, 48, 8, 12, 64, 5),     # b = 96: one full chunk + a tail
    (8, 8, 8, 8, 64, 0),        # a single block, nothing to select
    (32, 64, 32, 32, 32, 1),    # b = 1024, the largest tile
    (16, 16, 2, 2, 128, 63),    # every block selected: dense attention
    (24, 40, 8, 8, 128, 7),
])
def test_edge_shapes(G, oracle, dtype, H, W, bh, bw, D, n):
    cfg = shape_ns(2, 3, H, W, bh, bw, D, n, dtype)
    q, k, v = rand_qkv(cfg, 100 + H + W)
    if dtype == "bf16":
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    full_parity(G, oracle, cfg, q, k, v)


@pytest.mark.parametrize("H,W,bh,bw,n", [
    (64, 96, 16, 16, 5),     # 256-token tiles (the 0.25 degree configuration's tile)
    (32, 64, 4, 32, 3),      # 128-token tiles, wide
    (32, 64, 16, 4, 6),      # 64-token tiles, narrow
    (48, 64, 24, 8, 2),      # 192-token tiles: three sub-blocks
    (24, 128, 1, 64, 4),     # block-contiguous layout: a block is 64 consecutive tokens
    (12, 256, 1, 128, 3),    # block-contiguous, 128-token blocks
    (8, 256, 2, 128, 2),     # two rows of 128: sub-tiles are halves of a tile row
])
def test_mfma_tile_shapes(G, oracle, H, W, bh, bw, n):
    """bf16, D = 64 tiles of 64*T tokens (matrix-core forward kernel)."""
    cfg = shape_ns(2, 2, H, W, bh, bw, 64, n, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 500 + bh + bw))
    full_parity(G, oracle, cfg, q, k, v)


@pytest.mark.parametrize("H,W,bh,bw,n", [
    (32, 64, 8, 16, 4),      # the gradient configuration's tile
    (32, 64, 4, 32, 0),      # block-diagonal
    (32, 64, 16, 8, 15),     # n = m - 1: dense attention
    (16, 128, 2, 64, 3),
    (64, 32, 32, 4, 5),      # 4-token load slabs, the narrowest supported tile
    (8, 64, 8, 16, 1),       # one row of tiles
    (16, 256, 1, 128, 4),    # block-contiguous layout: a block is 128 consecutive tokens
    (32, 64, 8, 8, 5),       # 64-token tiles: workgroups of two wavefronts
    (32, 32, 16, 4, 3),      # 64-token tiles, the narrowest supported width
    (64, 64, 16, 16, 4),     # 256-token tiles: workgroups of eight wavefronts
    (8, 512, 1, 256, 0),     # block-contiguous 256-token blocks, block-diagonal
])
def test_mfma_d128_tile_shapes(G, oracle, H, W, bh, bw, n):
    """bf16, D = 128, tiles of 64, 128 or 256 tokens (matrix-core kernel with 32
    query rows per wavefront)."""
    cfg = shape_ns(2, 2, H, W, bh, bw, 128, n, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 700 + bh + bw))
    full_parity(G, oracle, cfg, q, k, v)


@pytest.mark.parametrize("H,W,bh,bw,D,n", [
    (80, 80, 8, 8, 64, 70),      # m = 100
    (72, 128, 8, 16, 128, 68),   # m = 72
])
def test_mfma_more_than_64_attended_blocks(G, oracle, H, W, bh, bw, D, n):
    """Above 64 attended blocks the matrix-core kernels visit the selection in
    the given order instead of sorting it inside a wavefront."""
    cfg = shape_ns(1, 2, H, W, bh, bw, D, n, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 600 + D))
    full_parity(G, oracle, cfg, q, k, v)


def test_mfma_d128_is_deterministic_and_order_invariant(G, oracle):
    cfg = shape_ns(1, 2, 32, 64, 8, 16, 128, 5, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 77))
    idx = oracle.select(oracle.shape_of(cfg), q, k)
    o1, l1 = G.gpu_fwd(cfg, q, k, v, idx)
    o2, l2 = G.gpu_fwd(cfg, q, k, v, idx)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    o3, _ = G.gpu_fwd(cfg, q, k, v, idx[..., ::-1].copy())
    assert np.abs(o3 - o1).max() <= 2e-2


def test_config4_quarter_degree_reduced(G, oracle):
    """The 0.25 degree configuration's tiles, head dim and n on a reduced grid
    (full forward against the oracle), seeded smooth fields."""
    p = make_problem(4, heads=2, grid_h=144, grid_w=288)
    full_parity(G, oracle, p.cfg, p.q, p.k, p.v)


def test_ties_and_exact_arithmetic_selection(G, oracle):
    """Constant keys (all scores tie) and quantised data (exact arithmetic):
    the tie-break and the never-select-yourself rule must match bit for bit."""
    cfg = shape_ns(1, 2, 32, 64, 8, 8, 32, 6, "fp32")
    s = oracle.shape_of(cfg)
    q, _, _ = rand_qkv(cfg, 7)
    k = np.ones_like(q)
    idx = G.gpu_select(cfg, q, k)
    assert np.array_equal(idx, oracle.select(s, q, k))
    for i in range(cfg.n_blocks):
        assert idx[0, 0, i].tolist() == [j for j in range(cfg.n_blocks) if j != i][:6]
    rng = np.random.default_rng(8)
    qq = (rng.integers(-8, 9, size=q.shape) / 4).astype(np.float32)
    kq = (rng.integers(-2, 3, size=q.shape) / 4).astype(np.float32)   # many ties
    assert np.array_equal(G.gpu_select(cfg, qq, kq), oracle.select(s, qq, kq))


@pytest.mark.parametrize("H,W,bh,bw,D,n,dtype", [
    (80, 120, 4, 4, 32, 9, "fp32"),      # m = 600
    (64, 128, 2, 2, 64, 40, "bf16"),     # m = 2048
    (64, 256, 2, 2, 128, 5, "bf16"),     # m = 4096, the most the register path holds
])
def test_selection_with_many_blocks(G, oracle, H, W, bh, bw, D, n, dtype):
    """512 < m <= 4096: ranking keys go through a global scratch matrix and the
    top-n runs from registers; indices must still match bit for bit, ties
    included."""
    cfg = shape_ns(1, 2, H, W, bh, bw, D, n, dtype)
    s = oracle.shape_of(cfg)
    q, k, _ = rand_qkv(cfg, 900 + D)
    if dtype == "bf16":
        q, k = round_to_bf16(q), round_to_bf16(k)
    assert np.array_equal(G.gpu_select(cfg, q, k), oracle.select(s, q, k))
    rng = np.random.default_rng(901)
    qq = (rng.integers(-8, 9, size=q.shape) / 4).astype(np.float32)
    kq = (rng.integers(-2, 3, size=q.shape) / 4).astype(np.float32)   # many exact ties
    assert np.array_equal(G.gpu_select(cfg, qq, kq), oracle.select(s, qq, kq))
    ones = np.ones_like(k)                                            # every score ties
    idx = G.gpu_select(cfg, q, ones)
    for i in (0, 1, n, cfg.n_blocks - 1):
        assert idx[0, 1, i].tolist() == [j for j in range(cfg.n_blocks) if j != i][:n]


def test_selection_with_more_blocks_than_registers_hold(G, oracle):
    """m > 4096: the fused kernel again, with fewer query blocks per workgroup
    and a top-n that rescans LDS after every pick."""
    cfg = shape_ns(1, 2, 96, 96, 1, 2, 32, 3, "fp32")          # m = 4608
    assert cfg.n_blocks == 4608
    s = oracle.shape_of(cfg)
    q, k, _ = rand_qkv(cfg, 950)
    assert np.array_equal(G.gpu_select(cfg, q, k), oracle.select(s, q, k))
    rng = np.random.default_rng(951)
    qq = (rng.integers(-8, 9, size=q.shape) / 4).astype(np.float32)
    kq = (rng.integers(-2, 3, size=q.shape) / 4).astype(np.float32)   # many exact ties
    assert np.array_equal(G.gpu_select(cfg, qq, kq), oracle.select(s, qq, kq))


def test_selection_at_the_largest_number_of_blocks(G, oracle):
    """m = 36,864: the most blocks whose scores of ONE query block fit the
    workgroup's LDS (one query block per workgroup); every row against the
    oracle.  (The next larger grid is rejected on the host: test_abi.)"""
    cfg = shape_ns(1, 1, 192, 192, 1, 1, 32, 3, "fp32")
    assert cfg.n_blocks == 36864
    s = oracle.shape_of(cfg)
    q, k, _ = rand_qkv(cfg, 960)
    assert np.array_equal(G.gpu_select(cfg, q, k), oracle.select(s, q, k))


@pytest.mark.parametrize("dtype,B,heads,kv_heads,H,W,bh,bw,D,n", [
    ("fp32", 1, 1, 1, 32, 64, 8, 8, 32, 5),       # one slice: a single part
    ("fp32", 1, 3, 3, 32, 64, 8, 8, 32, 5),       # three slices: three parts
    ("bf16", 5, 2, 1, 32, 64, 8, 8, 64, 7),       # 5 key/value slices in 4 parts, 2 query heads each
    ("bf16", 3, 6, 2, 64, 64, 8, 8, 128, 4),      # 6 key/value slices, head dim 128
    ("bf16", 5, 8, 8, 120, 240, 8, 8, 64, 16),    # 300 pooling blocks per part: the 256 resident
                                                  # pooling workgroups take more than one block
    ("bf16", 2, 4, 2, 64, 128, 2, 4, 64, 9),      # m = 1024 (64 candidates per lane), grouped heads
    ("fp32", 3, 2, 1, 48, 100, 2, 2, 32, 70),     # m = 1200, n > 64, odd number of key blocks per thread pair
])
def test_selection_over_parts_of_the_batch(G, oracle, dtype, B, heads, kv_heads, H, W, bh, bw, D, n):
    """mosaic_bsa_select pools one part of the batch beside the ranking of the
    part before: every way the slices fall into parts must give the indices
    and the pooled means of the one-pass definition, bit for bit."""
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    cfg = shape_ns(B, heads, H, W, bh, bw, D, n, dtype, kv_heads=kv_heads)
    rng = np.random.default_rng(8100 + B + heads + D)
    q = rng.standard_normal((B, heads, H * W, D)).astype(np.float32)
    k = rng.standard_normal((B, kv_heads, H * W, D)).astype(np.float32)
    if dtype == "bf16":
        q, k = round_to_bf16(q), round_to_bf16(k)
    s = oracle.shape_of(cfg)
    prm = G.params_of(cfg)
    ws = torch.full((M.mosaic_bsa_workspace_bytes(prm, binding.OP_SELECT),), 0xff,
                    dtype=torch.uint8, device="cuda")
    idx = torch.full((B, heads, cfg.n_blocks, n), -1, dtype=torch.int32, device="cuda")
    M.mosaic_bsa_select(prm, G.to_dev(q, cfg), G.to_dev(k, cfg), idx, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), oracle.select_gqa(s, q, k))
    wsf = ws.view(torch.float32).cpu().numpy()
    cnt_q = B * heads * cfg.n_blocks * D
    cnt_k = B * kv_heads * cfg.n_blocks * D
    k_at = (cnt_q * 4 + 255) // 256 * 256 // 4
    s_kv = oracle.shape_of(shape_ns(B, kv_heads, H, W, bh, bw, D, n, dtype))
    assert np.array_equal(wsf[:cnt_q], oracle.pool(s, q).reshape(-1))
    assert np.array_equal(wsf[k_at:k_at + cnt_k], oracle.pool(s_kv, k).reshape(-1))


def test_pooled_means_in_workspace_are_bit_exact(G, oracle):
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    p = make_problem(2)
    cfg = p.cfg
    s = oracle.shape_of(cfg)
    prm = G.params_of(cfg)
    q_d, k_d = G.to_dev(p.q, cfg), G.to_dev(p.k, cfg)
    nbytes = M.mosaic_bsa_workspace_bytes(prm, binding.OP_SELECT)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    idx = torch.empty((cfg.batch, cfg.heads, cfg.n_blocks, cfg.n_select), dtype=torch.int32,
                      device="cuda")
    M.mosaic_bsa_select(prm, q_d, k_d, idx, ws)
    torch.cuda.synchronize()
    cnt = cfg.batch * cfg.heads * cfg.n_blocks * cfg.head_dim
    wsf = ws.view(torch.float32).cpu().numpy()
    assert np.array_equal(wsf[:cnt].reshape(oracle.pool(s, p.q).shape), oracle.pool(s, p.q))
    half = (cnt * 4 + 255) // 256 * 256 // 4      # pooled q rounded up to 256 bytes
    assert np.array_equal(wsf[half:half + cnt].reshape(-1), oracle.pool(s, p.k).reshape(-1))


def test_forward_properties_on_gpu(G, oracle):
    cfg = get_config(2, heads=2)
    p = make_problem(2, heads=2)
    s = oracle.shape_of(cfg)
    idx = oracle.select(s, p.q, p.k)
    out, lse = G.gpu_fwd(cfg, p.q, p.k, p.v, idx)
    # deterministic: bitwise equal reruns
    out2, lse2 = G.gpu_fwd(cfg, p.q, p.k, p.v, idx)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
    # rows of the attention matrix sum to one: constant V comes back
    const = round_to_bf16(np.linspace(-1, 1, 64).astype(np.float32))
    outc, _ = G.gpu_fwd(cfg, p.q, p.k, np.broadcast_to(const, p.v.shape).copy(), idx)
    assert np.abs(outc - const).max() <= 1e-2
    # order of the selected blocks does not matter (up to rounding)
    rng = np.random.default_rng(3)
    perm = np.stack([rng.permutation(cfg.n_select) for _ in range(cfg.n_blocks)])
    idx_p = np.take_along_axis(idx, np.broadcast_to(perm, idx.shape), axis=3)
    outp, lsep = G.gpu_fwd(cfg, p.q, p.k, p.v, idx_p)
    assert np.abs(outp - out).max() <= 2e-2 and np.abs(lsep - lse).max() <= 4e-3
    # blocks that query block i did not select cannot influence its rows
    i = 77
    untouched = [j for j in range(cfg.n_blocks) if j != i and j not in idx[0, 0, i]]
    kt, vt = to_tiles(p.k, cfg).copy(), to_tiles(p.v, cfg).copy()
    kt[0, 0, untouched] = 3.0
    vt[0, 0, untouched] = -2.0
    from tests.helpers import from_tiles
    out3, _ = G.gpu_fwd(cfg, p.q, from_tiles(kt, cfg), from_tiles(vt, cfg), idx)
    assert np.array_equal(to_tiles(out, cfg)[0, 0, i], to_tiles(out3, cfg)[0, 0, i])


def test_arbitrary_selection_and_explicit_scale(G, oracle):
    cfg = shape_ns(1, 2, 32, 48, 8, 8, 64, 6, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 11))
    s = oracle.shape_of(cfg)
    idx = random_selection(cfg, 12)
    out_ref, lse_ref = oracle.fwd(s, q, k, v, idx, scale=0.2)
    out, lse = G.gpu_fwd(cfg, q, k, v, idx, softmax_scale=0.2)
    check_out(cfg, out, lse, out_ref, lse_ref)


# --------------------------------------------------------------------------
# full sizes, in the launch configuration the benchmark times
# --------------------------------------------------------------------------
def full_size_check(G, oracle, p, pairs):
    """Selection compared in full (bit-exact); forward compared on sampled query
    blocks that the oracle computes one by one."""
    cfg = p.cfg
    s = oracle.shape_of(cfg)
    q_d, k_d, v_d = (G.to_dev(x, cfg) for x in (p.q, p.k, p.v))
    idx_d = G.select_dev(cfg, q_d, k_d)
    out_d, lse_d = G.fwd_dev(cfg, q_d, k_d, v_d, idx_d)
    torch.cuda.synchronize()
    idx = idx_d.cpu().numpy()
    assert np.array_equal(idx, oracle.select_gqa(s, p.q, p.k))
    out_ref, lse_ref = oracle.fwd_blocks(s, p.q, p.k, p.v, idx, pairs)
    bh = cfg.batch * cfg.heads
    out_t = out_d.view(bh, cfg.n_tokens, cfg.head_dim)
    lse_t = lse_d.view(bh, cfg.n_tokens)
    for w, (g, i) in enumerate(pairs):
        rows = torch.tensor([oracle.token_of(s, int(i), t) for t in range(cfg.block_tokens)],
                            device="cuda")
        o = out_t[int(g)][rows].float().cpu().numpy()
        l = lse_t[int(g)][rows].cpu().numpy()
        assert np.isfinite(o).all()
        assert np.abs(o - out_ref[w]).max() <= 2e-2, (g, i)
        assert np.abs(l - lse_ref[w]).max() <= 1e-3, (g, i)
    # every output row was written (the buffers were pre-filled with NaN)
    assert bool(torch.isfinite(out_d.float()).all()) and bool(torch.isfinite(lse_d).all())


def test_config3_full_size_sampled(G, oracle):
    p = make_problem(3)
    cfg = p.cfg
    rng = np.random.default_rng(33)
    pairs = [[0, i] for i in range(cfg.n_blocks)]                 # member 0, head 0: all blocks
    for g in rng.choice(cfg.batch * cfg.heads, size=12, replace=False):
        pairs += [[int(g), int(i)] for i in rng.choice(cfg.n_blocks, size=24, replace=False)]
    full_size_check(G, oracle, p, np.array(pairs))


def test_config4_full_size_sampled(G, oracle):
    p = make_problem(4)
    cfg = p.cfg
    rng = np.random.default_rng(44)
    pairs = [[int(g), int(i)] for g in range(cfg.batch * cfg.heads)
             for i in rng.choice(cfg.n_blocks, size=41, replace=False)]   # 1 % of the query blocks
    full_size_check(G, oracle, p, np.array(pairs))


def test_config5_full_size_forward_sampled(G, oracle):
    p = make_problem(5)
    cfg = p.cfg
    rng = np.random.default_rng(55)
    pairs = [[int(g), int(i)] for g in rng.choice(cfg.batch * cfg.heads, size=8, replace=False)
             for i in rng.choice(cfg.n_blocks, size=20, replace=False)]
    full_size_check(G, oracle, p, np.array(pairs))


def test_config8_grouped_heads_full_size_sampled(G, oracle):
    """Configuration 3's shape with 4 query heads per key/value head."""
    p = make_problem(8)
    cfg = p.cfg
    rng = np.random.default_rng(88)
    pairs = [[int(g), int(i)] for g in rng.choice(cfg.batch * cfg.heads, size=24, replace=False)
             for i in rng.choice(cfg.n_blocks, size=12, replace=False)]
    full_size_check(G, oracle, p, np.array(pairs))


def test_config9_paper_stage1_shape_full_size_sampled(G, oracle):
    """49,152 tokens as 384 contiguous blocks of 128, 24 selected, grouped heads."""
    p = make_problem(9)
    cfg = p.cfg
    rng = np.random.default_rng(99)
    pairs = [[int(g), int(i)] for g in rng.choice(cfg.batch * cfg.heads, size=12, replace=False)
             for i in rng.choice(cfg.n_blocks, size=6, replace=False)]
    full_size_check(G, oracle, p, np.array(pairs))


# --------------------------------------------------------------------------
# backward (selection held fixed)
# --------------------------------------------------------------------------
def check_grads(cfg, got, ref):
    """fp32 mode: 1e-4 of the largest gradient entry.  bf16 mode: 2e-2 of
    max(1, largest entry) -- inputs, O and the stored gradients are bf16."""
    for name, g, r in zip(("dq", "dk", "dv"), got, ref):
        scale = max(1.0, np.abs(r).max()) if cfg.dtype == "bf16" else np.abs(r).max()
        tol = (2e-2 if cfg.dtype == "bf16" else 1e-4) * scale
        err = np.abs(g - r).max()
        assert err <= tol, f"{name}: max error {err} > {tol}"


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("H,W,bh,bw,D,n", [
    (32, 64, 8, 8, 32, 4),      # the tiny-grid configuration
    (48, 96, 8, 16, 128, 12),   # tile and head dim of the gradient configuration
    (12, 18, 6, 6, 32, 3),      # b = 36: ragged against the 64-row chunk
    (16, 48, 8, 12, 64, 5),     # b = 96
    (8, 8, 8, 8, 64, 0),        # single block
    (16, 16, 4, 4, 64, 15),     # every block selected: dense gradient
])
def test_backward_matches_oracle(G, oracle, dtype, H, W, bh, bw, D, n):
    cfg = shape_ns(1, 2, H, W, bh, bw, D, n, dtype)
    q, k, v = rand_qkv(cfg, 300 + H + D)
    dout = rand_qkv(cfg, 301 + H + D)[0]
    if dtype == "bf16":
        q, k, v, dout = (round_to_bf16(x) for x in (q, k, v, dout))
    s = oracle.shape_of(cfg)
    idx = oracle.select(s, q, k)
    ref = oracle.bwd(s, q, k, v, dout, idx)
    got = G.gpu_bwd(cfg, q, k, v, dout, idx)
    check_grads(cfg, got, ref)


@pytest.mark.parametrize("H,W,bh,bw,D,n", [
    (32, 64, 8, 8, 64, 4),       # 64-token blocks, two wavefronts per block
    (32, 64, 8, 16, 64, 3),      # 128-token blocks
    (32, 64, 16, 16, 64, 2),     # 256-token blocks, eight wavefronts per block
    (16, 128, 4, 32, 128, 0),    # head dim 128, block-diagonal
    (32, 32, 16, 16, 128, 3),    # head dim 128, 256-token blocks, n = m - 1: dense gradient
    (24, 64, 8, 16, 128, 5),
    (16, 128, 1, 128, 128, 3),   # block-contiguous layout, 128-token blocks
    (8, 256, 1, 256, 64, 2),     # block-contiguous layout, 256-token blocks
])
def test_backward_matrix_core_shapes(G, oracle, H, W, bh, bw, D, n):
    """bf16 shapes that run on the matrix-core backward kernels."""
    cfg = shape_ns(1, 3, H, W, bh, bw, D, n, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 900 + bh + D))
    dout = round_to_bf16(rand_qkv(cfg, 901 + bh + D)[0])
    s = oracle.shape_of(cfg)
    idx = random_selection(cfg, 41) if n else oracle.select(s, q, k)
    ref = oracle.bwd(s, q, k, v, dout, idx)
    got = G.gpu_bwd(cfg, q, k, v, dout, idx)
    check_grads(cfg, got, ref)


@pytest.mark.parametrize("H,W,bh,bw,D,n,sel_seed", [
    (96, 128, 8, 8, 64, 5, 43),      # 64-token blocks: rounds of 128 query blocks, m = 192
    (136, 256, 8, 16, 128, 3, 44),   # 128-token blocks, head dim 128: rounds of 256, m = 272
    (34, 1024, 1, 128, 64, 4, 45),   # block-contiguous 128-token blocks, head dim 64, m = 272
    (384, 384, 16, 16, 64, 1, 46),   # 256-token blocks: rounds of 512, m = 576
    (72, 80, 8, 8, 64, 70, 47),      # n > 64: the attended blocks do not fit one wavefront
    (40, 128, 8, 8, 64, 0, 0),       # n = 0 with several rounds: only the own block is connected
])
def test_backward_with_more_query_blocks_than_one_scan_round(G, oracle, H, W, bh, bw, D, n,
                                                             sel_seed):
    """The dK/dV kernels collect the query blocks connected to a key block in
    rounds of 64 x (wavefronts per workgroup) candidates; these shapes need two
    or more rounds per key block (the benchmark configurations need four to
    eight), and one of them has more attended blocks than a wavefront has
    lanes.  Arbitrary valid selections in random order."""
    cfg = shape_ns(1, 2, H, W, bh, bw, D, n, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 950 + bh + D + n))
    dout = round_to_bf16(rand_qkv(cfg, 951 + bh + D + n)[0])
    s = oracle.shape_of(cfg)
    idx = random_selection(cfg, sel_seed) if n else oracle.select(s, q, k)
    ref = oracle.bwd(s, q, k, v, dout, idx)
    got = G.gpu_bwd(cfg, q, k, v, dout, idx)
    check_grads(cfg, got, ref)


def slices_against_oracle_bwd(G, oracle, p, slices, idx_d=None):
    """Forward + backward of the whole problem on the GPU (the launch
    configuration the benchmark times); the gradients of the given (batch, head)
    slices against the oracle, which treats them as the heads of one entry."""
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    cfg = p.cfg
    prm = G.params_of(cfg)
    q_d, k_d, v_d, do_d = (G.to_dev(x, cfg) for x in (p.q, p.k, p.v, p.dout))
    if idx_d is None:
        idx_d = G.select_dev(cfg, q_d, k_d)
    out, lse = G.fwd_dev(cfg, q_d, k_d, v_d, idx_d)
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q_d, k_d, v_d))
    ws = torch.empty(M.mosaic_bsa_workspace_bytes(prm, binding.OP_BWD), dtype=torch.uint8,
                     device="cuda")
    M.mosaic_bsa_bwd(prm, q_d, k_d, v_d, out, lse, do_d, idx_d, dq, dk, dv, ws)
    torch.cuda.synchronize()
    for t in (dq, dk, dv):
        assert bool(torch.isfinite(t.float()).all())        # every row was written
    idx = idx_d.cpu().numpy()
    pick = lambda x: np.stack([x[e, a] for e, a in slices])[None]
    sub = dataclasses.replace(cfg, batch=1, heads=len(slices))
    ref = oracle.bwd(oracle.shape_of(sub), pick(p.q), pick(p.k), pick(p.v), pick(p.dout),
                     pick(idx))
    got = tuple(pick(t.float().cpu().numpy()) for t in (dq, dk, dv))
    check_grads(cfg, got, ref)
    return idx_d, (dq, dk, dv)


def test_backward_gradient_configuration_full_grid(G, oracle):
    """The gradient configuration at its full size (120 x 240 grid, batch 4, 16
    heads, head dim 128, tiles of 8 x 16, 12 selected blocks, dO white): the
    GPU's own selection, forward and backward of the whole problem; dQ, dK, dV
    of two whole (batch, head) slices against the oracle's closed forms."""
    p = make_problem(5)
    slices_against_oracle_bwd(G, oracle, p, [(1, 3), (3, 14)])


def test_backward_ensemble_shape_full_grid(G, oracle):
    """The 1.5 degree ensemble shape (m = 450 blocks of 64 tokens, head dim 64,
    16 selected blocks: four scan rounds per key block) at a reduced batch, dO
    white; two whole slices against the oracle; reruns are bitwise identical."""
    p = make_problem(3, batch=2, heads=4)
    rng = np.random.default_rng(35)
    p.dout = round_to_bf16(rng.standard_normal(p.q.shape).astype(np.float32))
    idx_d, first = slices_against_oracle_bwd(G, oracle, p, [(0, 1), (1, 2)])
    _, second = slices_against_oracle_bwd(G, oracle, p, [(1, 3)], idx_d)
    for a, b in zip(first, second):
        assert torch.equal(a, b)


def sampled_blocks_against_oracle_bwd(G, oracle, p, pairs):
    """Selection, forward and backward of the whole problem on the GPU (the
    launch configuration the benchmark times); dQ of the sampled blocks as query
    blocks and dK, dV of the same blocks as key blocks against the oracle."""
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    cfg = p.cfg
    prm = G.params_of(cfg)
    q_d, k_d, v_d, do_d = (G.to_dev(x, cfg) for x in (p.q, p.k, p.v, p.dout))
    idx_d = G.select_dev(cfg, q_d, k_d)
    out, lse = G.fwd_dev(cfg, q_d, k_d, v_d, idx_d)
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q_d, k_d, v_d))
    ws = torch.empty(M.mosaic_bsa_workspace_bytes(prm, binding.OP_BWD), dtype=torch.uint8,
                     device="cuda")
    M.mosaic_bsa_bwd(prm, q_d, k_d, v_d, out, lse, do_d, idx_d, dq, dk, dv, ws)
    torch.cuda.synchronize()
    del out, lse, ws
    s = oracle.shape_of(cfg)
    ref = oracle.bwd_blocks(s, p.q, p.k, p.v, p.dout, idx_d.cpu().numpy(), pairs)
    bh = cfg.batch * cfg.heads
    for w, (g, x) in enumerate(pairs):
        rows = torch.tensor([oracle.token_of(s, int(x), t) for t in range(cfg.block_tokens)],
                            device="cuda")
        got = tuple(t.view(bh, cfg.n_tokens, cfg.head_dim)[int(g)][rows].float().cpu().numpy()
                    for t in (dq, dk, dv))
        check_grads(cfg, got, tuple(r[w] for r in ref))
    for t in (dq, dk, dv):
        assert bool(torch.isfinite(t.float()).all())        # every row was written


def test_backward_quarter_degree_full_size_sampled(G, oracle):
    """The 0.25 degree configuration at its full size (m = 4050 blocks of 256
    tokens: eight scan rounds per key block), dO white: gradients of sampled
    blocks against the oracle."""
    p = make_problem(4)
    rng = np.random.default_rng(46)
    p.dout = round_to_bf16(rng.standard_normal(p.q.shape, dtype=np.float32))
    cfg = p.cfg
    pairs = np.array([[int(g), int(x)] for g in rng.choice(cfg.batch * cfg.heads, size=8,
                                                            replace=False)
                      for x in rng.choice(cfg.n_blocks, size=2, replace=False)])
    sampled_blocks_against_oracle_bwd(G, oracle, p, pairs)


def test_backward_ensemble_full_size_sampled(G, oracle):
    """The 1.5 degree ensemble configuration at its full size (batch 24, 16
    heads), dO white: gradients of sampled blocks against the oracle."""
    p = make_problem(3)
    rng = np.random.default_rng(36)
    p.dout = round_to_bf16(rng.standard_normal(p.q.shape, dtype=np.float32))
    cfg = p.cfg
    pairs = np.array([[int(g), int(x)] for g in rng.choice(cfg.batch * cfg.heads, size=16,
                                                            replace=False)
                      for x in rng.choice(cfg.n_blocks, size=3, replace=False)])
    sampled_blocks_against_oracle_bwd(G, oracle, p, pairs)


def test_backward_gradient_configuration_fields(G, oracle):
    """Seeded smooth fields of the gradient configuration (tile 8x16, D = 128,
    n = 12, dO white) on a reduced grid, arbitrary selection order; reruns are
    bitwise identical (fixed-order reduction, no float atomics)."""
    p = make_problem(5, batch=1, heads=2, grid_h=48, grid_w=96)
    cfg = p.cfg
    s = oracle.shape_of(cfg)
    idx = random_selection(cfg, 31)
    ref = oracle.bwd(s, p.q, p.k, p.v, p.dout, idx)
    got = G.gpu_bwd(cfg, p.q, p.k, p.v, p.dout, idx)
    check_grads(cfg, got, ref)
    again = G.gpu_bwd(cfg, p.q, p.k, p.v, p.dout, idx)
    for a, b in zip(got, again):
        assert np.array_equal(a, b)


# --------------------------------------------------------------------------
# grouped query attention: shared key/value heads, selection per query head
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,heads,kv_heads,H,W,bh,bw,D,n", [
    ("fp32", 2, 4, 2, 16, 32, 8, 8, 32, 3),      # general kernels
    ("bf16", 2, 6, 2, 12, 18, 6, 6, 64, 2),      # general kernels, bf16, b = 36
    ("bf16", 3, 6, 2, 16, 32, 8, 8, 64, 3),      # head dim 64 matrix-core path, 6 kv slices
    ("bf16", 5, 4, 2, 16, 32, 8, 8, 64, 3),      # 10 kv slices: 8 dealt to XCDs, 2 linear
    ("bf16", 1, 8, 1, 32, 32, 16, 16, 64, 2),    # 256-token blocks, one shared kv head
    ("bf16", 3, 8, 4, 16, 64, 8, 16, 128, 3),    # head dim 128 matrix-core path, 12 kv slices
    ("bf16", 2, 4, 4, 16, 32, 8, 8, 64, 3),      # kv_heads = heads, given explicitly
    ("bf16", 1, 4, 2, 96, 128, 8, 8, 64, 3),     # m = 192: two scan rounds per key block and head of a group
])
def test_grouped_query_attention(G, oracle, dtype, B, heads, kv_heads, H, W, bh, bw, D, n):
    cfg = shape_ns(B, heads, H, W, bh, bw, D, n, dtype, kv_heads=kv_heads)
    rng = np.random.default_rng(7000 + B + heads + D)
    q, dout = (rng.standard_normal((B, heads, H * W, D)).astype(np.float32) for _ in range(2))
    k, v = (rng.standard_normal((B, kv_heads, H * W, D)).astype(np.float32) for _ in range(2))
    if dtype == "bf16":
        q, k, v, dout = (round_to_bf16(x) for x in (q, k, v, dout))
    s = oracle.shape_of(cfg)
    idx_ref = oracle.select_gqa(s, q, k)
    idx_gpu = G.gpu_select(cfg, q, k)
    assert np.array_equal(idx_gpu, idx_ref)
    out_ref, lse_ref = oracle.fwd_gqa(s, q, k, v, idx_ref)
    out_gpu, lse_gpu = G.gpu_fwd(cfg, q, k, v, idx_gpu)
    check_out(cfg, out_gpu, lse_gpu, out_ref, lse_ref)
    ref = oracle.bwd_gqa(s, q, k, v, dout, idx_ref)
    got = G.gpu_bwd(cfg, q, k, v, dout, idx_ref)
    assert got[1].shape == k.shape and got[2].shape == v.shape
    check_grads(cfg, got, ref)


# --------------------------------------------------------------------------
# the three branches with their own softmaxes and the gated sum
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,heads,kv_heads,H,W,bh,bw,D,n,lh,lw", [
    ("fp32", 1, 2, 0, 32, 64, 8, 8, 32, 4, 2, 2),     # general kernels
    ("fp32", 2, 4, 2, 12, 18, 6, 6, 32, 6, 1, 3),     # n = m, b = 36, grouped heads
    ("bf16", 2, 4, 0, 32, 64, 8, 8, 64, 4, 2, 4),     # head dim 64 matrix-core kernels
    ("bf16", 1, 4, 1, 32, 64, 8, 8, 64, 1, 1, 1),     # n = 1, local block = the tile itself
    ("bf16", 1, 8, 2, 16, 256, 1, 128, 64, 5, 2, 2),  # block-contiguous 128-token blocks, grouped
    ("bf16", 2, 2, 0, 32, 64, 8, 16, 128, 3, 2, 2),   # head dim 128 matrix-core kernel
    ("bf16", 1, 2, 0, 120, 240, 8, 8, 64, 16, 3, 5),  # the 1.5 degree grid, m = 450
    ("fp32", 1, 2, 0, 80, 120, 4, 4, 32, 6, 2, 2),    # m = 600: ranking through global scratch
])
def test_three_branch_forward(G, oracle, dtype, B, heads, kv_heads, H, W, bh, bw, D, n, lh, lw):
    cfg = shape_ns(B, heads, H, W, bh, bw, D, n, dtype, kv_heads=kv_heads)
    hk = kv_heads or heads
    rng = np.random.default_rng(8000 + H + D + n)
    q = rng.standard_normal((B, heads, H * W, D)).astype(np.float32)
    k, v = (rng.standard_normal((B, hk, H * W, D)).astype(np.float32) for _ in range(2))
    if dtype == "bf16":
        q, k, v = (round_to_bf16(x) for x in (q, k, v))
    gates = rng.uniform(0.0, 1.0, size=(B, heads, H * W, 3)).astype(np.float32)
    s = oracle.shape_of(cfg, own_is_candidate=True)
    ref, sel_ref, _ = oracle.fwd_three_branch(s, q, k, v, gates, lh, lw)
    got, sel = G.gpu_fwd_three_branch(cfg, q, k, v, gates, lh, lw)
    assert np.array_equal(sel, sel_ref)
    if dtype == "bf16":
        err = np.abs(got - ref).max()
        assert err <= 2e-2, f"bf16 max-abs error {err}"
    else:
        rel = np.abs(got - ref).max() / np.abs(ref).max()
        assert rel <= 1e-5, f"fp32 relative error {rel}"


def test_three_branch_gates_isolate_the_branches(G, oracle):
    """One-hot gates: each branch on its own against the oracle's branch."""
    cfg = shape_ns(1, 2, 32, 64, 8, 8, 64, 3, "bf16")
    q, k, v = (round_to_bf16(x) for x in rand_qkv(cfg, 77))
    s = oracle.shape_of(cfg, own_is_candidate=True)
    ones = np.ones((1, 2, cfg.n_tokens, 3), dtype=np.float32)
    _, _, branches = oracle.fwd_three_branch(s, q, k, v, ones, 2, 2)
    for br in range(3):
        gates = np.zeros_like(ones)
        gates[..., br] = 1.0
        got, _ = G.gpu_fwd_three_branch(cfg, q, k, v, gates, 2, 2)
        err = np.abs(got - branches[br]).max()
        assert err <= 2e-2, f"branch {br}: max-abs error {err}"


def test_three_branch_paper_stage2_layer_reduced_batch(G, oracle):
    """The paper's stage-2 attention layer (12,288 pixels in contiguous blocks
    of 128, 12 selected blocks, local blocks of 1024, 4 query heads per
    key/value head) on seeded smooth fields, one batch entry and one group."""
    p = make_problem(11, batch=1, heads=4, kv_heads=1)
    cfg = p.cfg
    rng = np.random.default_rng(1111)
    gates = rng.uniform(0.0, 1.0, size=(1, 4, cfg.n_tokens, 3)).astype(np.float32)
    s = oracle.shape_of(cfg, own_is_candidate=True)
    ref, sel_ref, _ = oracle.fwd_three_branch(s, p.q, p.k, p.v, gates, 8, 1)
    got, sel = G.gpu_fwd_three_branch(cfg, p.q, p.k, p.v, gates, 8, 1)
    assert np.array_equal(sel, sel_ref)
    err = np.abs(got - ref).max()
    assert err <= 2e-2, f"bf16 max-abs error {err}"


@pytest.mark.parametrize("dtype,B,heads,kv_heads,H,W,bh,bw,D,n,lh,lw", [
    ("fp32", 1, 2, 0, 32, 64, 8, 8, 32, 4, 2, 2),     # general kernels
    ("fp32", 2, 4, 2, 12, 18, 6, 6, 32, 6, 1, 3),     # n = m, b = 36, grouped heads
    ("bf16", 2, 4, 0, 32, 64, 8, 8, 64, 4, 2, 4),     # head dim 64 matrix-core kernels
    ("bf16", 1, 4, 1, 32, 64, 8, 8, 64, 1, 1, 1),     # n = 1, local block = the tile itself
    ("bf16", 1, 8, 2, 16, 256, 1, 128, 64, 5, 2, 2),  # block-contiguous 128-token blocks, grouped
    ("bf16", 2, 2, 0, 32, 64, 8, 16, 128, 3, 2, 2),   # head dim 128 matrix-core kernels
    ("fp32", 1, 2, 0, 80, 120, 4, 4, 32, 6, 2, 2),    # m = 600: no interleaved copy of the pooled keys
    ("bf16", 1, 2, 0, 96, 128, 8, 8, 64, 4, 2, 2),    # m = 192: the lists span two scan rounds of dK/dV
    ("bf16", 1, 4, 2, 34, 1024, 1, 128, 64, 3, 2, 4), # m = 272, 128-token blocks, grouped heads
])
def test_three_branch_backward(G, oracle, dtype, B, heads, kv_heads, H, W, bh, bw, D, n, lh, lw):
    """Gradients of the three-branch form with the selection held fixed,
    against the oracle's reverse-mode gradients of the written-out definition."""
    cfg = shape_ns(B, heads, H, W, bh, bw, D, n, dtype, kv_heads=kv_heads)
    hk = kv_heads or heads
    rng = np.random.default_rng(8500 + H + D + n)
    q, dout = (rng.standard_normal((B, heads, H * W, D)).astype(np.float32) for _ in range(2))
    k, v = (rng.standard_normal((B, hk, H * W, D)).astype(np.float32) for _ in range(2))
    if dtype == "bf16":
        q, k, v, dout = (round_to_bf16(x) for x in (q, k, v, dout))
    gates = rng.uniform(0.0, 1.0, size=(B, heads, H * W, 3)).astype(np.float32)
    s = oracle.shape_of(cfg, own_is_candidate=True)
    out, sel, dq, dk, dv, dg = G.gpu_three_branch_fwd_bwd(cfg, q, k, v, gates, dout, lh, lw)
    rq, rk, rv, rg, _ = oracle.bwd_three_branch(s, q, k, v, gates, dout, sel, lh, lw)
    assert np.array_equal(sel, oracle.select_all(s, q, oracle.expand_kv(k, heads)))
    check_grads(cfg, (dq, dk, dv), (rq, rk, rv))
    tol = (2e-2 if dtype == "bf16" else 1e-4) * max(1.0, np.abs(rg).max())
    assert np.abs(dg - rg).max() <= tol


@pytest.mark.parametrize("kv_heads", [0, 4])
def test_three_branch_backward_coarse_branch_in_row_chunks(G, oracle, kv_heads):
    """With this many slices and blocks the block attention of the coarse branch
    and its gradient (B*h*m*m values each) exceed what the backward keeps of
    them, so it walks the query blocks in chunks and carries the column sums
    from chunk to chunk.  Batch entries and key/value heads are independent:
    sampled groups of the big problem against the oracle run on that group alone."""
    B, heads, H, W, D, n = 12, 8, 120, 240, 64, 4
    hk = kv_heads or heads
    group = heads // hk
    cfg = shape_ns(B, heads, H, W, 8, 8, D, n, "bf16", kv_heads=kv_heads)
    assert B * heads * cfg.n_blocks ** 2 * 4 > 64 << 20       # more than one chunk
    rng = np.random.default_rng(9100 + hk)
    q, dout = (round_to_bf16(rng.standard_normal((B, heads, H * W, D), dtype=np.float32))
               for _ in range(2))
    k, v = (round_to_bf16(rng.standard_normal((B, hk, H * W, D), dtype=np.float32))
            for _ in range(2))
    gates = rng.uniform(0.0, 1.0, size=(B, heads, H * W, 3)).astype(np.float32)
    out, sel, dq, dk, dv, dg = G.gpu_three_branch_fwd_bwd(cfg, q, k, v, gates, dout, 3, 3)
    one = shape_ns(1, group, H, W, 8, 8, D, n, "bf16", kv_heads=1 if kv_heads else 0)
    s = oracle.shape_of(one, own_is_candidate=True)
    for e, a in ((0, 0), (7, hk - 1), (11, hk // 2)):          # (batch entry, key/value head)
        qs = slice(a * group, (a + 1) * group)
        sub = lambda x, hs: np.ascontiguousarray(x[e:e + 1, hs])
        ks = slice(a, a + 1)
        rq, rk, rv, rg, _ = oracle.bwd_three_branch(s, sub(q, qs), sub(k, ks), sub(v, ks),
                                                    sub(gates, qs), sub(dout, qs), sub(sel, qs),
                                                    3, 3)
        check_grads(one, (sub(dq, qs), sub(dk, ks), sub(dv, ks)), (rq, rk, rv))
        assert np.abs(sub(dg, qs) - rg).max() <= 2e-2 * max(1.0, np.abs(rg).max())


def test_select_and_forward_replay_from_a_hip_graph(G, oracle):
    """The entry points allocate nothing and launch on the caller's stream, so a
    select + forward step can be captured once and replayed (the small
    configurations are launch-bound).  Every replay, with eager work and
    synchronisations in between, must reproduce the eager result bit for bit."""
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    cfg = shape_ns(1, 4, 32, 64, 8, 8, 64, 4, "bf16")
    prm = G.params_of(cfg)
    qs = [G.to_dev(round_to_bf16(rand_qkv(cfg, 40 + t)[0]), cfg) for t in range(3)]
    ks = [G.to_dev(round_to_bf16(rand_qkv(cfg, 50 + t)[1]), cfg) for t in range(3)]
    vs = [G.to_dev(round_to_bf16(rand_qkv(cfg, 60 + t)[2]), cfg) for t in range(3)]
    q, k, v = (torch.empty_like(qs[0]) for _ in range(3))
    idx = torch.empty((1, 4, cfg.n_blocks, 4), dtype=torch.int32, device="cuda")
    out = torch.empty_like(q)
    lse = torch.empty((1, 4, cfg.n_tokens), dtype=torch.float32, device="cuda")
    ws = torch.empty(M.mosaic_bsa_workspace_bytes(prm, binding.OP_SELECT), dtype=torch.uint8,
                     device="cuda")

    def step():
        M.mosaic_bsa_select(prm, q, k, idx, ws)
        M.mosaic_bsa_fwd(prm, q, k, v, idx, out, lse)

    eager = []
    for t in range(3):                       # eager results (also the warm-up before capture)
        q.copy_(qs[t]); k.copy_(ks[t]); v.copy_(vs[t])
        step()
        torch.cuda.synchronize()
        eager.append((idx.clone(), out.clone(), lse.clone()))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(2):
        for t in range(3):
            q.copy_(qs[t]); k.copy_(ks[t]); v.copy_(vs[t])
            out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(idx, eager[t][0])
            assert torch.equal(out, eager[t][1]) and torch.equal(lse, eager[t][2])


def test_three_branch_results_are_run_to_run_identical(G, oracle):
    """Every sum in the three-branch forward and backward has a fixed order
    (no floating-point atomics): two runs agree bit for bit, grouped heads
    included."""
    cfg = shape_ns(2, 4, 32, 64, 8, 8, 64, 5, "bf16", kv_heads=2)
    rng = np.random.default_rng(4242)
    q, dout = (round_to_bf16(rng.standard_normal((2, 4, 2048, 64)).astype(np.float32))
               for _ in range(2))
    k, v = (round_to_bf16(rng.standard_normal((2, 2, 2048, 64)).astype(np.float32))
            for _ in range(2))
    gates = rng.uniform(0.0, 1.0, size=(2, 4, 2048, 3)).astype(np.float32)
    first = G.gpu_three_branch_fwd_bwd(cfg, q, k, v, gates, dout, 2, 2)
    second = G.gpu_three_branch_fwd_bwd(cfg, q, k, v, gates, dout, 2, 2)
    for a, b in zip(first, second):
        assert np.array_equal(a, b)


def test_selection_checker_counts_what_the_kernels_must_not_get(G, oracle):
    import paper_2604_16429_amd as M
    cfg = shape_ns(2, 3, 32, 64, 8, 8, 64, 5, "bf16")
    prm = G.params_of(cfg)
    q, k, _ = (round_to_bf16(x) for x in rand_qkv(cfg, 321))
    idx = torch.from_numpy(G.gpu_select(cfg, q, k)).to("cuda")
    n_bad = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    M.mosaic_bsa_check_selection(prm, idx, False, n_bad)
    assert int(n_bad.item()) == 0                       # what select emits is clean
    bad = idx.clone()
    bad[0, 0, 3, 2] = cfg.n_blocks                      # out of range
    bad[1, 2, 7, 0] = -1                                # negative
    bad[0, 1, 5, 4] = bad[0, 1, 5, 1]                   # repeats an earlier entry
    bad[1, 0, 9, 3] = 9                                 # the row's own block
    M.mosaic_bsa_check_selection(prm, bad, False, n_bad)
    assert int(n_bad.item()) == 4
    M.mosaic_bsa_check_selection(prm, bad, True, n_bad)     # own block allowed: three left
    assert int(n_bad.item()) == 3


@pytest.mark.parametrize("bh,bw,D", [(8, 8, 64), (8, 16, 64), (8, 16, 128), (6, 6, 32)])
def test_large_logits_with_rising_maxima(G, oracle, bh, bw, D):
    """Logits of magnitude up to about +-80 whose maxima grow with the block
    index: the kernels visit blocks in ascending order, so the running
    reference of the softmax has to be replaced again and again (the slow
    path of the matrix-core kernels); forward and backward must stay within
    the usual bounds (outputs of magnitude up to about 5 here: the plain 2e-2
    bound is 1.25 bf16 half-ulps of the largest entries) and free of NaN / inf."""
    H, W = 4 * bh, 6 * bw
    cfg = shape_ns(1, 2, H, W, bh, bw, D, 9, "bf16")
    q, k, v = rand_qkv(cfg, 1234 + D)
    dout = rand_qkv(cfg, 1235 + D)[0]
    s = oracle.shape_of(cfg)
    # scale keys block by block (1x .. 7x), queries by 3
    grow = 1.0 + 6.0 * np.arange(cfg.n_blocks) / (cfg.n_blocks - 1)
    kt = to_tiles(k, cfg) * grow[None, None, :, None, None].astype(np.float32)
    from tests.helpers import from_tiles
    k = from_tiles(kt, cfg)
    q, k, v, dout = (round_to_bf16(x) for x in (3.0 * q, k, v, dout))
    idx = random_selection(cfg, 77)
    out_ref, lse_ref = oracle.fwd(s, q, k, v, idx)
    assert np.abs(lse_ref).max() > 40.0                 # the logits really are large
    out, lse = G.gpu_fwd(cfg, q, k, v, idx)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    err = np.abs(out - out_ref).max()
    print(f"stress: max|O| {np.abs(out_ref).max():.3f} max-abs error {err:.4f} "
          f"lse error {np.abs(lse - lse_ref).max():.2e}")
    assert err <= 2e-2
    assert np.abs(lse - lse_ref).max() <= 1e-3
    got = G.gpu_bwd(cfg, q, k, v, dout, idx)
    ref = oracle.bwd(s, q, k, v, dout, idx)
    for g_, r_ in zip(got, ref):
        assert np.isfinite(g_).all()
    check_grads(cfg, got, ref)
