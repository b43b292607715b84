"""Seeded synthetic Q/K/V fields on a lat-lon grid.

This module only manufactures inputs.  It holds none of the attention
method's arithmetic (no pooling, scoring, selection or softmax) so that both
the CPU oracle's tests and the GPU path's tests can draw the same bits from it
without sharing any of the code under test.

Recipe (one tensor X in {Q, K, V}, shape [B, heads, N, D], N = H*W, token
t = r*W + c, D fastest):

  * for every (head, channel) draw a white N(0,1) field on the H x W grid;
  * low-pass it with a Gaussian of standard deviation L cells ("correlation
    length L"), reflecting in latitude and periodic in longitude.  The filter
    is applied in the spectral domain: a DCT-II along latitude (its implied
    boundary is the half-sample reflection) and a real FFT along longitude
    (periodic), multiplied by the Gaussian transfer function
    exp(-L^2 w^2 / 2);
  * rescale each field to unit sample variance;
  * add sigma_w * N(0,1) white noise;
  * ensemble configurations share that base field between members and add an
    independent sigma_m * N(0,1) perturbation per member;
  * bf16 configurations are rounded to bf16 (round-to-nearest-even) once, on
    the host, and handed out as fp32 arrays whose values are exactly
    bf16-representable, so every consumer sees identical bits.

Seeds: 16429000 + 100*config_id + tensor_id with tensor_id Q=0, K=1, V=2,
dO=3; heads and ensemble members spawn numbered child streams of that seed.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import scipy.fft

SEED_BASE = 16429000
TENSOR_ID = {"q": 0, "k": 1, "v": 2, "do": 3}


@dataclasses.dataclass(frozen=True)
class GridConfig:
    """Shape of one attention call on the grid (names follow the paper:
    b tokens per block, m blocks, n selected blocks)."""
    config_id: int
    batch: int
    heads: int
    grid_h: int
    grid_w: int
    block_h: int
    block_w: int
    head_dim: int
    n_select: int
    dtype: str            # "fp32" or "bf16"
    corr_len: float       # L, in grid cells
    sigma_white: float    # sigma_w
    sigma_member: float = 0.0   # sigma_m; > 0 means members share a base field
    with_dout: bool = False
    kv_heads: int = 0           # key/value heads; 0 = heads (no grouping)

    @property
    def n_tokens(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def block_tokens(self) -> int:
        return self.block_h * self.block_w

    @property
    def n_blocks(self) -> int:
        return self.n_tokens // self.block_tokens

    def fwd_flops(self) -> int:
        """Multiply-add work of the block products QK^T and PV (2 flops per
        MAC): the O(N n b + N b) term of the paper's cost model."""
        return (4 * self.batch * self.heads * self.n_tokens
                * (self.n_select + 1) * self.block_tokens * self.head_dim)


CONFIGS = {
    1: GridConfig(1, 1, 2, 32, 64, 8, 8, 32, 4, "fp32", 4.0, 0.1),
    2: GridConfig(2, 1, 8, 120, 240, 8, 8, 64, 8, "bf16", 6.0, 0.1),
    3: GridConfig(3, 24, 16, 120, 240, 8, 8, 64, 16, "bf16", 6.0, 0.1,
                  sigma_member=0.05),
    4: GridConfig(4, 1, 16, 720, 1440, 16, 16, 64, 16, "bf16", 24.0, 0.1),
    5: GridConfig(5, 4, 16, 120, 240, 8, 16, 128, 12, "bf16", 6.0, 0.1,
                  with_dout=True),
    # Shapes of the paper's first stage (49,152 tokens, sparse block size 128,
    # 24 selected blocks; architecture table), which the five benchmark
    # configurations do not cover.  6: block-contiguous layout, a block is 128
    # consecutive tokens (what a nested HEALPix ordering gives): 384 tiles one
    # row high.  7: the same token count as 8 x 16 tiles of a 192 x 256 grid,
    # to measure what gathering 2-D tiles costs against contiguous blocks.
    6: GridConfig(6, 8, 16, 384, 128, 1, 128, 64, 24, "bf16", 6.0, 0.1),
    7: GridConfig(7, 8, 16, 192, 256, 8, 16, 64, 24, "bf16", 6.0, 0.1),
    # Grouped query attention at the paper's ratio of 4 query heads per
    # key/value head (architecture table): 8 is configuration 3 and 9 is
    # configuration 6 with K and V of shape [B, heads / 4, N, D].
    8: GridConfig(8, 24, 16, 120, 240, 8, 8, 64, 16, "bf16", 6.0, 0.1,
                  sigma_member=0.05, kv_heads=4),
    9: GridConfig(9, 8, 16, 384, 128, 1, 128, 64, 24, "bf16", 6.0, 0.1, kv_heads=4),
    # The attention layers of the paper's U-Net as the architecture table gives
    # them (pixels, heads = dim / 64, grouped-query ratio 4, sparse block size
    # 128, sparse block count), batch 24, block-contiguous: 10 = stage 1
    # (49,152 pixels, 12 heads, 24 blocks), 11 = stage 2 (12,288 pixels, 16
    # heads, 12 blocks), 12 = bottleneck (3,072 pixels, 20 heads, 4 blocks).
    10: GridConfig(10, 24, 12, 384, 128, 1, 128, 64, 24, "bf16", 6.0, 0.1, kv_heads=3),
    11: GridConfig(11, 24, 16, 96, 128, 1, 128, 64, 12, "bf16", 6.0, 0.1, kv_heads=4),
    12: GridConfig(12, 24, 20, 24, 128, 1, 128, 64, 4, "bf16", 6.0, 0.1, kv_heads=5),
}


def get_config(config_id: int, **overrides) -> GridConfig:
    """A named configuration, optionally with fields replaced (tests use
    reduced batch/heads variants of the large configurations)."""
    return dataclasses.replace(CONFIGS[config_id], **overrides)


# ---------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (data format only)
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs must be finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose values are the bf16 roundings of x."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ---------------------------------------------------------------------------
# smooth random fields
# ---------------------------------------------------------------------------

def _transfer(grid_h: int, grid_w: int, corr_len: float) -> np.ndarray:
    w_lat = np.pi * np.arange(grid_h) / grid_h                 # DCT-II modes
    w_lon = 2.0 * np.pi * np.arange(grid_w // 2 + 1) / grid_w  # rfft modes
    g_lat = np.exp(-0.5 * (corr_len * w_lat) ** 2)
    g_lon = np.exp(-0.5 * (corr_len * w_lon) ** 2)
    return (g_lat[:, None] * g_lon[None, :]).astype(np.float32)


def smooth_fields(rng: np.random.Generator, count: int, grid_h: int,
                  grid_w: int, corr_len: float, workers: int = 1) -> np.ndarray:
    """`count` independent unit-variance Gaussian random fields, [count, H, W]
    fp32, low-passed as described in the module docstring."""
    white = rng.standard_normal((count, grid_h, grid_w), dtype=np.float32)
    spec = scipy.fft.dct(white, type=2, axis=1, norm="ortho", workers=workers)
    spec = scipy.fft.rfft(spec, axis=2, workers=workers)
    spec *= _transfer(grid_h, grid_w, corr_len)[None]
    out = scipy.fft.irfft(spec, n=grid_w, axis=2, workers=workers)
    out = scipy.fft.idct(out, type=2, axis=1, norm="ortho", workers=workers)
    out = out.astype(np.float32, copy=False)
    out /= out.reshape(count, -1).std(axis=1, dtype=np.float64).astype(
        np.float32)[:, None, None]
    return out


def _head_base(seed: int, head: int, cfg: GridConfig) -> np.ndarray:
    """Base field of one head: [N, D] fp32 = smooth + sigma_w * white."""
    ss = np.random.SeedSequence([seed, 0, head])
    rng = np.random.Generator(np.random.PCG64(ss))
    f = smooth_fields(rng, cfg.head_dim, cfg.grid_h, cfg.grid_w, cfg.corr_len)
    f += np.float32(cfg.sigma_white) * rng.standard_normal(
        f.shape, dtype=np.float32)
    # [D, H, W] -> [N, D]
    return np.ascontiguousarray(f.reshape(cfg.head_dim, cfg.n_tokens).T)


def _finish(x: np.ndarray, cfg: GridConfig) -> np.ndarray:
    return round_to_bf16(x) if cfg.dtype == "bf16" else x


def make_tensor(cfg: GridConfig, name: str, workers: int = 8) -> np.ndarray:
    """One of q/k/v/do for `cfg`: fp32 array [B, heads, N, D] ([B, kv_heads,
    N, D] for k and v of a grouped configuration; values bf16-representable
    when cfg.dtype == "bf16")."""
    seed = SEED_BASE + 100 * cfg.config_id + TENSOR_ID[name]
    B, h, N, D = cfg.batch, cfg.heads, cfg.n_tokens, cfg.head_dim
    if name in ("k", "v") and cfg.kv_heads:
        h = cfg.kv_heads
    out = np.empty((B, h, N, D), dtype=np.float32)

    if name == "do":   # upstream gradient: plain white noise
        def fill(e):
            ss = np.random.SeedSequence([seed, 2, e])
            rng = np.random.Generator(np.random.PCG64(ss))
            out[e] = _finish(rng.standard_normal((h, N, D), dtype=np.float32),
                             cfg)
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(fill, range(B)))
        return out

    if cfg.sigma_member > 0.0:
        # ensemble: members share one base field per head
        def fill_head(a):
            base = _head_base(seed, a, cfg)
            for e in range(B):
                ss = np.random.SeedSequence([seed, 1, e, a])
                rng = np.random.Generator(np.random.PCG64(ss))
                eps = rng.standard_normal((N, D), dtype=np.float32)
                eps *= np.float32(cfg.sigma_member)
                eps += base
                out[e, a] = _finish(eps, cfg)
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(fill_head, range(h)))
        return out

    # independent fields per (batch entry, head)
    def fill_one(idx):
        e, a = divmod(idx, h)
        out[e, a] = _finish(_head_base(seed + 7919 * e, a, cfg), cfg)
    with ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(fill_one, range(B * h)))
    return out


@dataclasses.dataclass
class Problem:
    cfg: GridConfig
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    dout: np.ndarray | None = None


def make_problem(config_id: int, workers: int = 8, **overrides) -> Problem:
    """Seeded inputs of configuration `config_id` (see CONFIGS)."""
    cfg = get_config(config_id, **overrides)
    q = make_tensor(cfg, "q", workers)
    k = make_tensor(cfg, "k", workers)
    v = make_tensor(cfg, "v", workers)
    dout = make_tensor(cfg, "do", workers) if cfg.with_dout else None
    return Problem(cfg, q, k, v, dout)
