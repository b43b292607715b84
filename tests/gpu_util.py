"""Runs the HIP library through its C ABI (via the thin Python binding) on
numpy inputs; used by the GPU parity tests only."""
from __future__ import annotations

import numpy as np
import torch

import paper_2604_16429_amd as M
from paper_2604_16429_amd import binding


def params_of(cfg, n_select=None, softmax_scale=0.0):
    return M.Params(cfg.batch, cfg.heads, cfg.grid_h, cfg.grid_w, cfg.block_h,
                    cfg.block_w, cfg.head_dim,
                    cfg.n_select if n_select is None else n_select,
                    binding.BF16 if cfg.dtype == "bf16" else binding.F32,
                    softmax_scale, getattr(cfg, "kv_heads", 0))


def to_dev(x, cfg):
    """fp32 numpy (bf16-representable when cfg is bf16) -> device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    return t.to(torch.bfloat16) if cfg.dtype == "bf16" else t


def select_dev(cfg, q_d, k_d, n_select=None):
    p = params_of(cfg, n_select)
    n = p.n_select
    idx = torch.full((cfg.batch, cfg.heads, p.n_blocks, n), -1, dtype=torch.int32,
                     device="cuda")
    ws = torch.empty(max(M.mosaic_bsa_workspace_bytes(p, binding.OP_SELECT), 256),
                     dtype=torch.uint8, device="cuda")
    M.mosaic_bsa_select(p, q_d, k_d, idx, ws)
    return idx


def fwd_dev(cfg, q_d, k_d, v_d, idx_d, n_select=None, softmax_scale=0.0, want_lse=True):
    p = params_of(cfg, n_select, softmax_scale)
    out = torch.full_like(q_d, float("nan"))
    lse = (torch.full((cfg.batch, cfg.heads, p.n_tokens), float("nan"),
                      dtype=torch.float32, device="cuda") if want_lse else None)
    M.mosaic_bsa_fwd(p, q_d, k_d, v_d, idx_d, out, lse)
    return out, lse


def gpu_select(cfg, q, k, n_select=None):
    idx = select_dev(cfg, to_dev(q, cfg), to_dev(k, cfg), n_select)
    torch.cuda.synchronize()
    return idx.cpu().numpy()


def gpu_fwd(cfg, q, k, v, idx, n_select=None, softmax_scale=0.0):
    idx_d = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).to("cuda")
    out, lse = fwd_dev(cfg, to_dev(q, cfg), to_dev(k, cfg), to_dev(v, cfg), idx_d,
                       n_select, softmax_scale)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), lse.cpu().numpy()


def gpu_bwd(cfg, q, k, v, dout, idx, n_select=None, softmax_scale=0.0):
    """Forward then backward on the GPU; returns (dq, dk, dv) as fp32 numpy."""
    p = params_of(cfg, n_select, softmax_scale)
    idx_d = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).to("cuda")
    q_d, k_d, v_d, do_d = (to_dev(x, cfg) for x in (q, k, v, dout))
    out, lse = fwd_dev(cfg, q_d, k_d, v_d, idx_d, n_select, softmax_scale)
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q_d, k_d, v_d))
    ws = torch.empty(max(M.mosaic_bsa_workspace_bytes(p, binding.OP_BWD), 256),
                     dtype=torch.uint8, device="cuda")
    M.mosaic_bsa_bwd(p, q_d, k_d, v_d, out, lse, do_d, idx_d, dq, dk, dv, ws)
    torch.cuda.synchronize()
    return tuple(t.float().cpu().numpy() for t in (dq, dk, dv))


def gpu_fwd_three_branch(cfg, q, k, v, gates, local_h, local_w, softmax_scale=0.0):
    """Three-branch forward on the GPU; returns (out fp32 numpy, sel_idx)."""
    p = params_of(cfg, None, softmax_scale)
    q_d, k_d, v_d = (to_dev(x, cfg) for x in (q, k, v))
    g_d = torch.from_numpy(np.ascontiguousarray(gates, dtype=np.float32)).to("cuda")
    out = torch.full_like(q_d, float("nan"))
    idx = torch.full((cfg.batch, cfg.heads, p.n_blocks, p.n_select), -1, dtype=torch.int32,
                     device="cuda")
    nbytes = M.mosaic_bsa_three_branch_workspace_bytes(p, local_h, local_w)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    M.mosaic_bsa_fwd_three_branch(p, local_h, local_w, q_d, k_d, v_d, g_d, out, idx, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), idx.cpu().numpy()


def gpu_three_branch_fwd_bwd(cfg, q, k, v, gates, dout, local_h, local_w):
    """Three-branch forward then backward on the GPU; returns (out, sel, dq, dk,
    dv, dgates) as numpy arrays."""
    p = params_of(cfg)
    q_d, k_d, v_d, do_d = (to_dev(x, cfg) for x in (q, k, v, dout))
    g_d = torch.from_numpy(np.ascontiguousarray(gates, dtype=np.float32)).to("cuda")
    out = torch.full_like(q_d, float("nan"))
    idx = torch.full((cfg.batch, cfg.heads, p.n_blocks, p.n_select), -1, dtype=torch.int32,
                     device="cuda")
    ws_f = torch.empty(M.mosaic_bsa_three_branch_workspace_bytes(p, local_h, local_w),
                       dtype=torch.uint8, device="cuda")
    M.mosaic_bsa_fwd_three_branch(p, local_h, local_w, q_d, k_d, v_d, g_d, out, idx, ws_f)
    nbytes = M.mosaic_bsa_three_branch_bwd_workspace_bytes(p, local_h, local_w)
    assert nbytes > 0
    ws_b = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q_d, k_d, v_d))
    dg = torch.full_like(g_d, float("nan"))
    M.mosaic_bsa_bwd_three_branch(p, local_h, local_w, q_d, k_d, v_d, g_d, do_d, idx, ws_f,
                                  dq, dk, dv, dg, ws_b)
    torch.cuda.synchronize()
    return (out.float().cpu().numpy(), idx.cpu().numpy(), dq.float().cpu().numpy(),
            dk.float().cpu().numpy(), dv.float().cpu().numpy(), dg.cpu().numpy())
