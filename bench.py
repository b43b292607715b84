#!/usr/bin/env python3
"""Benchmark of the block-sparse attention hot path on one MI355X.

One "step" is one pass of the whole hot path -- block selection (pooling,
block scores, top-n) followed by the block-sparse attention forward -- over
one batch of seeded synthetic grid fields that already reside in HBM.

Default workload: the 1.5 degree global grid (120 x 240 = 28,800 tokens) with a
24-member ensemble batch, 16 heads, head dim 64, 8 x 8 tiles and the 16 best
blocks per query block, bf16 I/O with fp32 accumulation.

Prints ONE JSON line: tokens/s of the whole step as `value`, effective
TFLOP/s of the dense block products, the roofline of the dominant kernel (the
attention forward, MFMA-bound) from HIP-event timings taken inside the timed
region, and the CPU oracle timed on a bounded sample on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0

# HBM bytes per forward launch come from the rocprofv3 counter runs summarised
# under profiles/ (FETCH_SIZE, then WRITE_SIZE, each scaled by the same counter
# on a plain copy kernel of known size).  A summary carries a line
#   bench-traffic: config=<id> bytes=<float> sources-sha256=<hex>
# where the hash covers the sources of the forward kernel it was measured on;
# the figure is reported only while those sources are unchanged.
FWD_KERNEL_SOURCES = ("bsa_fwd_mfma.hip", "bsa_mfma_common.h", "bsa_device.h")


def fwd_sources_sha256() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in FWD_KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_16429_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_fwd_traffic(config_id: int):
    """(bytes per launch, where it was read) or (None, why not)."""
    import glob
    import re
    sha = fwd_sources_sha256()
    stale = None
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for m in re.finditer(r"bench-traffic:\s*config=(\d+)\s+bytes=([0-9.eE+]+)\s+"
                             r"sources-sha256=([0-9a-f]+)", open(path).read()):
            if int(m.group(1)) != config_id:
                continue
            if m.group(3) == sha:
                return float(m.group(2)), os.path.relpath(path, ROOT)
            stale = os.path.relpath(path, ROOT)
    return None, (f"{stale} was measured on other kernel sources" if stale
                  else "not measured for this workload")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="configuration id (1-5: the benchmark configurations; 6, 7: the paper's stage-1 shape, block-contiguous and tiled; 8, 9: configurations 3 and 6 with 4 query heads per key/value head; 10-12: the paper's stage-1, stage-2 and bottleneck attention layers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--three-branch", type=int, nargs=2, metavar=("LOCAL_H", "LOCAL_W"),
                    help="also time the three-branch forward (coarse + selection + local "
                         "branches, gated sum) with large local blocks of LOCAL_H x LOCAL_W tiles")
    ap.add_argument("--hip-graph", action="store_true",
                    help="also capture one step in a HIP graph and time its replays (the small "
                         "configurations are launch-bound)")
    ap.add_argument("--with-bwd", action="store_true",
                    help="also run the backward (selection held fixed) after the timed steps "
                         "and report its time; it is not part of a step")
    return ap.parse_args()


def cpu_baseline(problem, cfg):
    """The oracle, as it stands, on the host cores: the first batch entries
    (all heads) of the same workload through select + forward."""
    import dataclasses
    from oracle import bsa_oracle
    nb = min(cfg.batch, 8)
    sub = dataclasses.replace(cfg, batch=nb)
    s = bsa_oracle.shape_of(sub)
    q, k, v = problem.q[:nb], problem.k[:nb], problem.v[:nb]
    t0 = time.perf_counter()
    idx = bsa_oracle.select_gqa(s, q, k)
    t1 = time.perf_counter()
    bsa_oracle.fwd_gqa(s, q, k, v, idx)
    t2 = time.perf_counter()
    return {
        "value": nb * cfg.n_tokens / (t2 - t0), "unit": "tokens/s",
        "cores": bsa_oracle.threads(), "kind": "oracle",
        "sample": (f"batch entries 0..{nb - 1} of the workload, all {cfg.heads} heads "
                   f"({nb * cfg.n_tokens} tokens): select {t1 - t0:.2f} s + forward "
                   f"{t2 - t1:.2f} s, double-precision attention"),
        "seconds": t2 - t0,
        "extrapolated_full_workload_seconds": (t2 - t0) * cfg.batch / nb,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path "
              "(batch and heads shard without any exchange); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    from inputs.fields import get_config, make_problem

    cfg = get_config(args.config)
    problem = make_problem(args.config)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    is_bf16 = cfg.dtype == "bf16"

    def up(x):
        t = torch.from_numpy(x).to(dev)
        return t.to(torch.bfloat16) if is_bf16 else t

    q, k, v = up(problem.q), up(problem.k), up(problem.v)
    prm = M.Params(cfg.batch, cfg.heads, cfg.grid_h, cfg.grid_w, cfg.block_h, cfg.block_w,
                   cfg.head_dim, cfg.n_select, binding.BF16 if is_bf16 else binding.F32, 0.0,
                   cfg.kv_heads)
    idx = torch.empty((cfg.batch, cfg.heads, cfg.n_blocks, cfg.n_select), dtype=torch.int32,
                      device=dev)
    out = torch.empty_like(q)
    lse = torch.empty((cfg.batch, cfg.heads, cfg.n_tokens), dtype=torch.float32, device=dev)
    ws = torch.empty(max(M.mosaic_bsa_workspace_bytes(prm, binding.OP_SELECT), 256),
                     dtype=torch.uint8, device=dev)

    def step(events=None):
        if events is not None:
            events[0].record()
        M.mosaic_bsa_select(prm, q, k, idx, ws)
        if events is not None:
            events[1].record()
        M.mosaic_bsa_fwd(prm, q, k, v, idx, out, lse)
        if events is not None:
            events[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sel_all = sorted(e[0].elapsed_time(e[1]) for e in evs)
    fwd_all = sorted(e[1].elapsed_time(e[2]) for e in evs)
    sel_ms = sum(sel_all) / args.steps
    fwd_ms = sum(fwd_all) / args.steps

    # One cold step: a 1 GiB fill pushes the inputs out of L2 and the memory-side
    # cache first (outside the timed region above).
    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    flush.fill_(1)
    cold = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    step(cold)
    torch.cuda.synchronize()
    del flush

    # The matrix pipe's sustained rate on this machine: a register-resident bf16 MFMA
    # loop (2 wavefronts per SIMD, mixed-sign operands), nothing else running.
    probe_wgs, probe_iters = 2048, 4000
    sink = torch.empty(probe_wgs * 256, dtype=torch.float32, device=dev)
    M.mosaic_bsa_probe_mfma(sink, probe_wgs, 200)
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    M.mosaic_bsa_probe_mfma(sink, probe_wgs, probe_iters)
    p1.record()
    torch.cuda.synchronize()
    probe_tflops = probe_wgs * 4 * 16 * probe_iters * 32768 / (p0.elapsed_time(p1) * 1e-3) / 1e12
    del sink

    # Sustained dense bf16 matrix rate of this machine (library GEMM on random
    # operands), for context: clocks under matrix load are below nominal.
    gemm_tflops = None
    if is_bf16:
        ga = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
        gb = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
        for _ in range(3):
            torch.matmul(ga, gb)
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(10):
            torch.matmul(ga, gb)
        g1.record()
        torch.cuda.synchronize()
        gemm_tflops = 10 * 2 * 8192 ** 3 / (g0.elapsed_time(g1) * 1e-3) / 1e12
        del ga, gb
    tokens = cfg.batch * cfg.n_tokens
    flops = cfg.fwd_flops()
    eff_tflops = flops / (fwd_ms * 1e-3) / 1e12
    esz = 2 if is_bf16 else 4
    kv_heads = cfg.kv_heads or cfg.heads
    compulsory = 2 * cfg.batch * (cfg.heads + kv_heads) * cfg.n_tokens * cfg.head_dim * esz
    traffic, traffic_from = measured_fwd_traffic(args.config)
    # workgroups per query block in the forward (each gathers the block's tiles once):
    # head dim 64 groups 4, 2 or 1 sub-blocks of 64 queries, head dim 128 the whole block
    subs = max(1, cfg.block_tokens // 64)
    gathers_per_block = (subs // (4 if subs % 4 == 0 else 2 if subs % 2 == 0 else 1)
                         if cfg.head_dim == 64 else 1)

    result = {
        "metric": "block-sparse attn tokens/s @1.5deg grid (select + forward); "
                  "effective TFLOP/s and % MFMA peak alongside",
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {
            "workload": (f"config {cfg.config_id}: {cfg.grid_h}x{cfg.grid_w} lat-lon grid "
                         f"({cfg.n_tokens} tokens), batch {cfg.batch}, {cfg.heads} heads, "
                         f"head_dim {cfg.head_dim}, tiles {cfg.block_h}x{cfg.block_w}, "
                         f"local + top-{cfg.n_select} blocks"
                         + (f", {cfg.kv_heads} key/value heads" if cfg.kv_heads else "")),
            "tokens_per_step": tokens,
        },
        "select_ms": sel_ms, "fwd_ms": fwd_ms,
        "fwd_ms_median": fwd_all[len(fwd_all) // 2], "fwd_ms_min": fwd_all[0],
        "select_ms_median": sel_all[len(sel_all) // 2], "select_ms_min": sel_all[0],
        "cold_select_ms": cold[0].elapsed_time(cold[1]),
        "cold_fwd_ms": cold[1].elapsed_time(cold[2]),
        "dense_equivalent_tflops": (4 * cfg.batch * cfg.heads * cfg.n_tokens ** 2 * cfg.head_dim
                                    / (fwd_ms * 1e-3) / 1e12),
        "mfma_loop_bf16_tflops": probe_tflops,
        "pct_of_mfma_loop": 100.0 * eff_tflops / probe_tflops,
        "library_gemm_bf16_tflops": gemm_tflops,
        "pct_of_library_gemm": (100.0 * eff_tflops / gemm_tflops) if gemm_tflops else None,
        "hbm_frac_fwd": (traffic / (fwd_ms * 1e-3) / (HBM_PEAK_GBS * 1e9)) if traffic else None,
        "effective_tflops": eff_tflops,
        "pct_mfma_peak": 100.0 * eff_tflops / MFMA_BF16_PEAK_TFLOPS,
        "fwd_only_tokens_per_s": tokens / (fwd_ms * 1e-3),
        "compulsory_hbm_gbs": compulsory / (fwd_ms * 1e-3) / 1e9,
        # K/V bytes that the forward gathers into LDS (every attended tile once per
        # query block) over the forward time, against what the CUs' vector-memory
        # path moves at most: 64 B per clock and CU, 256 CUs, 2.4 GHz nominal.  At
        # 64-token query blocks this path, not the matrix pipe, bounds the kernel.
        "gather_path": {
            "achieved_tbs": (cfg.batch * cfg.heads * cfg.n_tokens * (cfg.n_select + 1)
                             * 2 * cfg.head_dim * esz * gathers_per_block
                             / (fwd_ms * 1e-3) / 1e12),
            "peak_tbs": 256 * 64 * 2.4e9 / 1e12,
            "flop_per_gathered_byte": cfg.block_tokens * 2 / esz / gathers_per_block,
        },
        "roofline": {
            "kernel": "attention forward",
            "bound": "mfma", "achieved": eff_tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": eff_tflops / MFMA_BF16_PEAK_TFLOPS,
            "traffic": traffic, "traffic_source": traffic_from,
        },
    }
    if args.hip_graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        result["hip_graph_ms_per_step"] = (time.perf_counter() - tg0) * 1e3 / args.steps
    if args.with_bwd:
        if problem.dout is not None:
            dout = up(problem.dout)
        else:       # workloads without an upstream gradient in their recipe: seeded white noise
            gen = torch.Generator(device=dev).manual_seed(16429003)
            dout = torch.randn(q.shape, generator=gen, device=dev, dtype=torch.float32).to(q.dtype)
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws_b = torch.empty(max(M.mosaic_bsa_workspace_bytes(prm, binding.OP_BWD), 256),
                           dtype=torch.uint8, device=dev)
        reps = max(2, args.steps // 4)
        M.mosaic_bsa_bwd(prm, q, k, v, out, lse, dout, idx, dq, dk, dv, ws_b)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.mosaic_bsa_bwd(prm, q, k, v, out, lse, dout, idx, dq, dk, dv, ws_b)
        e1.record()
        torch.cuda.synchronize()
        bwd_ms = e0.elapsed_time(e1) / reps
        result["bwd_ms"] = bwd_ms
        # five block products per pair against the forward's two
        result["bwd_effective_tflops"] = 2.5 * flops / (bwd_ms * 1e-3) / 1e12
    if args.three_branch:
        lh, lw = args.three_branch
        nbytes = M.mosaic_bsa_three_branch_workspace_bytes(prm, lh, lw)
        if nbytes == 0:
            sys.exit(f"--three-branch {lh} {lw}: the local group must divide the grid of tiles")
        ws_t = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        gen = torch.Generator(device=dev).manual_seed(16429004)
        gates = torch.rand((cfg.batch, cfg.heads, cfg.n_tokens, 3), generator=gen, device=dev,
                           dtype=torch.float32)
        out3 = torch.empty_like(q)
        reps = max(2, args.steps // 2)
        M.mosaic_bsa_fwd_three_branch(prm, lh, lw, q, k, v, gates, out3, idx, ws_t)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.mosaic_bsa_fwd_three_branch(prm, lh, lw, q, k, v, gates, out3, idx, ws_t)
        e1.record()
        torch.cuda.synchronize()
        tb_ms = e0.elapsed_time(e1) / reps
        # block products of the two attention branches: n selected blocks, and the
        # lh*lw tiles of the large local block
        tb_flops = flops // (cfg.n_select + 1) * (cfg.n_select + lh * lw)
        result["three_branch"] = {
            "local_group": [lh, lw], "ms": tb_ms,
            "tokens_per_s": tokens / (tb_ms * 1e-3),
            "effective_tflops": tb_flops / (tb_ms * 1e-3) / 1e12,
        }
        if args.with_bwd:
            nb = M.mosaic_bsa_three_branch_bwd_workspace_bytes(prm, lh, lw)
            ws_tb = torch.empty(nb, dtype=torch.uint8, device=dev)
            gen = torch.Generator(device=dev).manual_seed(16429005)
            dout3 = torch.randn(q.shape, generator=gen, device=dev,
                                dtype=torch.float32).to(q.dtype)
            dq3, dk3, dv3 = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
            dg3 = torch.empty_like(gates)

            def bwd3():
                M.mosaic_bsa_bwd_three_branch(prm, lh, lw, q, k, v, gates, dout3, idx, ws_t,
                                              dq3, dk3, dv3, dg3, ws_tb)
            bwd3()
            torch.cuda.synchronize()
            reps = max(2, args.steps // 4)
            e0.record()
            for _ in range(reps):
                bwd3()
            e1.record()
            torch.cuda.synchronize()
            result["three_branch"]["bwd_ms"] = e0.elapsed_time(e1) / reps
            del ws_tb, dout3, dq3, dk3, dv3, dg3
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(problem, cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
