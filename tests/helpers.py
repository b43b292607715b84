"""Test-side helpers that are independent of both the oracle and the HIP path."""
from __future__ import annotations

import types

import numpy as np


def shape_ns(batch, heads, grid_h, grid_w, block_h, block_w, head_dim, n_select,
             dtype="fp32", kv_heads=0):
    return types.SimpleNamespace(
        kv_heads=kv_heads,
        batch=batch, heads=heads, grid_h=grid_h, grid_w=grid_w, block_h=block_h,
        block_w=block_w, head_dim=head_dim, n_select=n_select, dtype=dtype,
        n_tokens=grid_h * grid_w, block_tokens=block_h * block_w,
        n_blocks=(grid_h // block_h) * (grid_w // block_w))


def to_tiles(x, c):
    """[B,h,N,D] -> [B,h,m,b,D] by reshaping the grid into tiles.  This is a
    second, independent statement of the token partition (no index formula)."""
    B, h, N, D = x.shape
    gh, gw = c.grid_h // c.block_h, c.grid_w // c.block_w
    t = x.reshape(B, h, gh, c.block_h, gw, c.block_w, D)
    t = np.transpose(t, (0, 1, 2, 4, 3, 5, 6))
    return np.ascontiguousarray(t).reshape(B, h, gh * gw, c.block_h * c.block_w, D)


def from_tiles(t, c):
    """Inverse of to_tiles."""
    B, h, m, b, D = t.shape
    gh, gw = c.grid_h // c.block_h, c.grid_w // c.block_w
    x = t.reshape(B, h, gh, gw, c.block_h, c.block_w, D)
    x = np.transpose(x, (0, 1, 2, 4, 3, 5, 6))
    return np.ascontiguousarray(x).reshape(B, h, c.grid_h * c.grid_w, D)


def rand_qkv(c, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    shp = (c.batch, c.heads, c.n_tokens, c.head_dim)
    return tuple((scale * rng.standard_normal(shp)).astype(np.float32)
                 for _ in range(3))


def random_selection(c, seed):
    """A valid but arbitrary selection: n distinct blocks != own, random order."""
    rng = np.random.default_rng(seed)
    m, n = c.n_blocks, c.n_select
    idx = np.empty((c.batch, c.heads, m, n), dtype=np.int32)
    for e in range(c.batch):
        for a in range(c.heads):
            for i in range(m):
                cand = np.delete(np.arange(m), i)
                idx[e, a, i] = rng.permutation(cand)[:n]
    return idx
