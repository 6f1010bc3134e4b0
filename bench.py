#!/usr/bin/env python3
"""Benchmark of the Jigsaw linear-layer forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--ways 4]

A *step* is one ``jg_linear_forward``: every virtual rank's two block products, the
hand-off of partial products (and, 4-way, weight blocks) and the combine, with all
shards already resident in HBM.  ``value`` = items/s = (M*K elements of X) / step time.
Prints ONE JSON line.
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

FP32_MFMA_PEAK_TFLOPS = 157.3   # MI355X dense FP32 matrix peak
BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense BF16 matrix peak
HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--ways", type=int, default=4, choices=[1, 2, 4])
    ap.add_argument("--op", choices=["forward", "backward", "xw", "xtw", "mlp", "mixing", "mixing_backward", "token_mixing",
                                   "token_mixing_backward", "encoder"],
                    default="forward",
                    help="forward: Y = X W^T (the headline); backward: dX = dY W and dW = dY^T X; xw: the third permutation Y = X W (weights stored along the contracted index) at --config's size; "
                         "xtw: the transposed layer Y = X^T W at the token-mixing size; mlp: one mixing MLP "
                         "(GELU between two layers, residual) at the channel-mixing size; mixing: the same behind a layer norm "
                         "(the channel-mixing half of a mixing block); token_mixing: the token-mixing half (norm, transposed "
                         "layer with GELU, the layer back with the skip connection); encoder: patch rearrangement of a "
                         "field + linear layer at the 1B model's encoder size (these ignore --config)")
    ap.add_argument("--dtype", choices=["f32", "bf16", "bf16x3"], default="f32",
                    help="forward only: f32 (the headline), or a reduced-precision mode: operands rounded to bfloat16 "
                         "when they are sharded (bf16), or split in two bfloat16 parts and multiplied in three "
                         "passes (bf16x3)")
    ap.add_argument("--combine", choices=["fused", "separate"], default="fused")
    ap.add_argument("--weights", choices=["copy", "direct"], default="copy")
    ap.add_argument("--accumulate", choices=["levels", "single"], default="levels",
                    help="reduced precision: second summation level between launches (default), or one launch per product")
    ap.add_argument("--tail", choices=["split", "whole"], default="split",
                    help="last partial round of a GEMM launch: cut into runs when that pays (default), or whole tiles")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="target CPU time of the oracle baseline sample (0 disables it)")
    ap.add_argument("--extras", action="store_true", help="(accepted for older command lines: the extras are on by default)")
    ap.add_argument("--only-headline", action="store_true",
                    help="the headline configuration only: skip the streaming kernels, the other values of `ways`, one "
                         "rank's share, the separate combine, the reduced-precision modes and the other configs")
    return ap.parse_args()


def tail_of(args):
    from paper_2507_05753_amd import binding as jg
    return jg.JG_TAIL_SPLIT if args.tail == "split" else jg.JG_TAIL_WHOLE


def acc_of(args):
    from paper_2507_05753_amd import binding as jg
    return jg.JG_ACC_LEVELS if args.accumulate == "levels" else jg.JG_ACC_SINGLE


def dtype_of(args, jg):
    return {"f32": jg.JG_F32, "bf16": jg.JG_BF16, "bf16x3": jg.JG_BF16X3}[args.dtype]


def gemm_roofline(args, r):
    """The roofline object of the MLP / mixing lines: the GEMM kernel of the chosen precision against its peak."""
    terms = 3 if args.dtype == "bf16x3" else 1
    reduced = args.dtype != "f32"
    peak = BF16_MFMA_PEAK_TFLOPS if reduced else FP32_MFMA_PEAK_TFLOPS
    achieved = r["gemm_tflops"] * terms if r["gemm_tflops"] else None      # matrix-core work: three products per block
    kernel = {"f32": "jg::gemm_f32_stream<false, false, false>", "bf16": "jg::gemm_bf16_nt",
              "bf16x3": "jg::gemm_bf16x3_nt"}[args.dtype]
    out = {"bound": "mfma", "kernel": kernel, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
           "frac": achieved / peak if achieved else None, "avg_launch_ms": r["gemm_avg_launch_ms"],
           "launches": r["gemm_launches_timed"], "traffic": None}
    if reduced:
        out["matrix_passes"] = terms
    return out


def precision_words(args):
    return {"f32": "fp32", "bf16": "mixed precision: bfloat16 products, fp32 sums and activations",
            "bf16x3": "mixed precision: split bfloat16 operands (three products), fp32 sums and activations"}[args.dtype]


def make_inputs(cfg, dev):
    """Global X [M,K] and W [N,K] on the device (seeded, synthetic)."""
    import torch
    from paper_2507_05753_amd import inputs
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    if cfg["x_mode"] == "Z":   # Zipf ranks are drawn on the host in float64
        X = torch.from_numpy(inputs.matrix(seed, M, K, "Z")).to(dev)
    else:
        X = inputs.matrix_torch(seed, M, K, "R", 0, device=dev)
    W = inputs.matrix_torch(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP, device=dev)
    return X, W


def time_forward(L, jg, steps, warmup, norm=None, untimed_events=False):
    """(seconds per step by wall clock, GEMM ms total, GEMM launches, weight-copy and combine ms per step);
    `norm`: a dict that receives the layer-norm kernel's total ms and launch count.
    untimed_events: for steps of a few dozen microseconds, where the two event records around every launch are a
    visible share of the wall clock: the step time is taken from a loop of its own without them."""
    import torch
    for _ in range(warmup):
        L.forward()
    torch.cuda.synchronize()
    plain = None
    if untimed_events:
        t0 = time.perf_counter()
        for _ in range(steps):
            L.forward()
        torch.cuda.synchronize()
        plain = (time.perf_counter() - t0) / steps
    for k in (jg.JG_KERNEL_GEMM, jg.JG_KERNEL_WEIGHT_COPY, jg.JG_KERNEL_COMBINE, jg.JG_KERNEL_JOIN, jg.JG_KERNEL_NORM,
              jg.JG_KERNEL_SHARD):
        jg.jg_profile_read(L.ctx, k)
    jg.jg_profile(L.ctx, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        L.forward()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    jg.jg_profile(L.ctx, False)
    gemm_ms, gemm_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_GEMM)
    wc_ms, _ = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_WEIGHT_COPY)
    cb_ms, _ = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_COMBINE)
    join_ms, _ = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_JOIN)   # tail join of split launches, counted with the hand-off copy
    cvt_ms, _ = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_SHARD)   # a mixed-precision chain rounds its activations per layer
    if norm is not None:
        norm["ms"], norm["launches"] = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_NORM)
        norm["cvt_ms_per_step"] = cvt_ms / steps
    return (t1 - t0) / steps if plain is None else plain, gemm_ms, gemm_n, (wc_ms + join_ms + cvt_ms) / steps, cb_ms / steps


def measure(cfg, ways, args, X, W, streaming=False, steps=None, warmup=None, combine=None, dtype=None, share=False,
            accumulate=None):
    """One configuration of the forward layer.  steps / warmup / combine / dtype default to the command line's."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = cfg["M"], cfg["K"], cfg["N"]
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    combine = args.combine if combine is None else combine
    dtype_name = args.dtype if dtype is None else dtype
    combine = jg.JG_COMBINE_FUSED if combine == "fused" else jg.JG_COMBINE_SEPARATE
    weights = jg.JG_WEIGHTS_COPY if args.weights == "copy" else jg.JG_WEIGHTS_DIRECT
    out = {}
    dtype = {"f32": jg.JG_F32, "bf16": jg.JG_BF16, "bf16x3": jg.JG_BF16X3}[dtype_name]
    acc = {"levels": jg.JG_ACC_LEVELS, "single": jg.JG_ACC_SINGLE}[args.accumulate if accumulate is None else accumulate]
    with JigsawLinear(M, K, N, ways, combine=combine, weights=weights, tail=tail_of(args), dtype=dtype,
                      accumulate=acc) as L:
        L.shard(X, W)
        sec, gemm_ms, gemm_n, wcopy_ms, comb_ms = time_forward(L, jg, steps, warmup, untimed_events=M * K * N < 10 ** 10)
        other_ms = wcopy_ms + comb_ms
        flops = L.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.query(jg.JG_Q_GEMM_LAUNCHES)
        algo_bytes = L.query(jg.JG_Q_HBM_BYTES_ALGO)
        avg_launch_ms = gemm_ms / max(gemm_n, 1)
        out = dict(
            ms_per_step=sec * 1e3, items_per_s=M * K / sec, tflops=flops / sec / 1e12,
            gemm_avg_launch_ms=avg_launch_ms, gemm_launches_timed=gemm_n,
            gemm_launches_per_step=launches,
            gemm_tflops=(flops / launches) / (avg_launch_ms * 1e-3) / 1e12 if gemm_n else None,
            other_kernels_ms_per_step=other_ms,
            hbm_algo_gbps=algo_bytes / sec / 1e9, hbm_algo_frac=algo_bytes / sec / 1e9 / HBM_PEAK_GBPS,
            workspace_bytes=L.ws_bytes)
        if comb_ms > 0:   # separate combine: two reads and one write per output element
            out["combine_gbps"] = 12.0 * M * N / (comb_ms * 1e-3) / 1e9
        if streaming:
            # the HBM-bound steps around the forward: shard (X), gather (Y); bytes = read + write
            stream = {}
            jg.jg_profile(L.ctx, True)
            reps = 5
            for _ in range(reps):
                L.shard(X=X)
            Yg = L.gather()
            for _ in range(reps - 1):
                L.gather(Yg)
            jg.jg_profile(L.ctx, False)
            sh_ms, sh_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_SHARD)
            ga_ms, ga_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_GATHER)
            shard_bytes = {"f32": 8.0, "bf16": 6.0, "bf16x3": 8.0}[dtype_name]   # read FP32, write the shard format
            stream["shard_x_gbps"] = shard_bytes * M * K / (sh_ms / sh_n * 1e-3) / 1e9
            stream["gather_y_gbps"] = 8.0 * M * N / (ga_ms / ga_n * 1e-3) / 1e9
            stream["shard_x_frac"] = stream["shard_x_gbps"] / HBM_PEAK_GBPS
            stream["gather_y_frac"] = stream["gather_y_gbps"] / HBM_PEAK_GBPS
            out["streaming"] = stream
            del Yg
    if share and ways > 1:
        # One rank's share at its real shape: its two block products, alone on the GPU
        # (what one GPU of an n-GPU node would run per layer, exchange excluded).
        Mr, Kr, Nr = (M, K // 2, N // 2) if ways == 2 else (M // 2, K // 2, N // 2)
        with JigsawLinear(Mr, Kr, Nr, 1, dtype=dtype) as R:
            R.shard(X[:Mr, :Kr], W[:Nr, :Kr])
            for _ in range(2 * warmup):
                R.forward()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                R.forward()
                R.forward()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / steps
            out["one_rank_share"] = dict(ms=dt * 1e3, tflops=2 * R.query(jg.JG_Q_FLOPS_TOTAL) / dt / 1e12,
                                         shape=f"2 x ([{Mr} x {Kr}] . [{Nr} x {Kr}]^T)")
    torch.cuda.empty_cache()
    return out


def measure_backward(cfg, ways, args, X, W):
    """One step = one jg_linear_backward (dX and dW of all ranks), shards resident in HBM."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = cfg["M"], cfg["K"], cfg["N"]
    dY = inputs.matrix_torch(cfg["seed"] + 3000, M, N, "R", 0, device=X.device)
    reduced = args.dtype != "f32"
    terms = 3 if args.dtype == "bf16x3" else 1
    with JigsawLinear(M, K, N, ways, tail=tail_of(args), dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        if reduced:
            L.shard_master(X, W)        # the backward of a reduced-precision plan reads FP32 X and W and rounds them
        else:
            L.shard(X, W)
        L.shard_dy(dY)
        del dY
        for _ in range(args.warmup):
            L.backward()
        torch.cuda.synchronize()
        for k in (jg.JG_KERNEL_GEMM_DX, jg.JG_KERNEL_GEMM_DW, jg.JG_KERNEL_SHARD, jg.JG_KERNEL_JOIN):
            jg.jg_profile_read(L.ctx, k)
        jg.jg_profile(L.ctx, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            L.backward()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / args.steps
        jg.jg_profile(L.ctx, False)
        dx_ms, dx_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_GEMM_DX)
        dw_ms, dw_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_GEMM_DW)
        cvt_ms, cvt_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_SHARD)
        join_ms, _ = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_JOIN)
        flops = L.query(jg.JG_Q_BACKWARD_FLOPS_TOTAL)
        half = flops / 2   # dX and dW cost the same
        names = {"f32": ("jg::gemm_f32_stream<false, true, false>", "jg::gemm_f32_stream<true, true, false>"),
                 "bf16": ("jg::gemm_bf16_nt", "jg::gemm_bf16_nt"), "bf16x3": ("jg::gemm_bf16x3_nt", "jg::gemm_bf16x3_nt")}[args.dtype]
        # (tflops: the matrix cores' work - the split mode multiplies three times per product of the layer)
        kernels = {
            "dx": dict(kernel=names[0] + (" (dX)" if reduced else ""), avg_launch_ms=dx_ms / max(dx_n, 1), launches=dx_n,
                       tflops=terms * half * args.steps / (dx_ms * 1e-3) / 1e12),
            "dw": dict(kernel=names[1] + (" (dW)" if reduced else ""), avg_launch_ms=dw_ms / max(dw_n, 1), launches=dw_n,
                       tflops=terms * half * args.steps / (dw_ms * 1e-3) / 1e12),
        }
        if reduced:
            # the rounding passes: dY twice, X and W once each; 4 B read and 2 B (split mode 4 B) written per element
            out_b = 4 if terms == 3 else 2
            cvt_bytes = (4 + out_b) * (2 * M * N + M * K + N * K)
            kernels["cvt"] = dict(kernel="jg::cvt_bf16 / jg::cvt_bf16_transposed", ms_per_step=cvt_ms / args.steps,
                                  launches=cvt_n, gbps=cvt_bytes * args.steps / (cvt_ms * 1e-3) / 1e9 if cvt_ms > 0 else None)
            kernels["join"] = dict(kernel="jg::gemm_bf16_join", ms_per_step=join_ms / args.steps)
        ws = L.bw_ws_bytes
        # the bias gradient (column sums of dY), timed on its own: it is not part of jg_linear_backward
        for _ in range(args.warmup):
            L.bias_backward()
        torch.cuda.synchronize()
        jg.jg_profile_read(L.ctx, jg.JG_KERNEL_REDUCE)
        jg.jg_profile(L.ctx, True)
        for _ in range(args.steps):
            L.bias_backward()
        jg.jg_profile(L.ctx, False)
        db_ms, db_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_REDUCE)
        db_avg = db_ms / max(db_n, 1)
        kernels["db"] = dict(kernel="jg::colsum_f32<true>", avg_launch_ms=db_avg, launches=db_n,
                             gbps=4.0 * M * N / (db_avg * 1e-3) / 1e9 if db_n else None,
                             frac_of_hbm_peak=4.0 * M * N / (db_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS if db_n else None)
    torch.cuda.empty_cache()
    return dict(ms_per_step=sec * 1e3, items_per_s=M * K / sec, tflops=flops / sec / 1e12, kernels=kernels,
                workspace_bytes=ws)


def measure_xw(cfg, ways, args):
    """One step = one forward of the permutation Y = X W (W stored [K, N]; all ranks), shards resident in HBM."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    dev = torch.device("cuda", 0)
    X = inputs.matrix_torch(seed, M, K, cfg["x_mode"], 0, device=dev)
    W = inputs.matrix_torch(seed + inputs.W_STREAM, K, N, "R", inputs.W_SCALE_EXP, device=dev)
    weights = jg.JG_WEIGHTS_COPY if args.weights == "copy" else jg.JG_WEIGHTS_DIRECT
    with JigsawLinear(M, K, N, ways, weights=weights, op=jg.JG_OP_XW, tail=tail_of(args)) as L:
        L.shard(X, W)
        del X, W
        sec, gemm_ms, gemm_n, copy_ms, comb_ms = time_forward(L, jg, args.steps, args.warmup)
        flops = L.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.query(jg.JG_Q_GEMM_LAUNCHES)
        avg = gemm_ms / max(gemm_n, 1)
        out = dict(ms_per_step=sec * 1e3, items_per_s=M * K / sec, tflops=flops / sec / 1e12,
                   gemm_avg_launch_ms=avg, gemm_launches_timed=gemm_n,
                   gemm_tflops=(flops / launches) / (avg * 1e-3) / 1e12 if gemm_n else None,
                   other_kernels_ms_per_step=copy_ms + comb_ms,
                   hbm_algo_gbps=L.query(jg.JG_Q_HBM_BYTES_ALGO) / sec / 1e9, workspace_bytes=L.ws_bytes)
    torch.cuda.empty_cache()
    return out


def cpu_baseline_xw(cfg, seconds):
    """The oracle of Y = X W timed on a bounded sample of rows of X."""
    import numpy as np
    import oracle
    from paper_2507_05753_amd import inputs
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    W = inputs.matrix(seed + inputs.W_STREAM, K, N, "R", inputs.W_SCALE_EXP)

    def run(rows):
        Xs = inputs.matrix(seed, M, K, cfg["x_mode"], row_begin=0, row_end=rows)
        t0 = time.perf_counter()
        Y = oracle.linear_xw(Xs, W, None, nthreads=cores)
        dt = time.perf_counter() - t0
        assert np.isfinite(Y).all()
        return dt

    probe = min(M, 2 * cores)
    rate = probe / max(run(probe), 1e-9)
    rows = int(min(M, max(probe, rate * seconds)))
    rows = min(M, max(cores, rows // cores * cores))
    dt = run(rows)
    return dict(value=rows * K / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"rows 0..{rows - 1} of X ({rows} x {K}) against all of W ({K} x {N}), {dt:.1f} s, fp64 triple loop")


def measure_xtw(cfg, ways, args):
    """One step = one forward of the transposed layer Y = X^T W (all ranks), shards resident in HBM."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawLinear
    K, M, N, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    dev = torch.device("cuda", 0)
    X = inputs.matrix_torch(seed, K, M, "R", 0, device=dev)
    W = inputs.matrix_torch(seed + inputs.W_STREAM, K, N, "R", inputs.W_SCALE_EXP, device=dev)
    combine = jg.JG_COMBINE_FUSED if args.combine == "fused" else jg.JG_COMBINE_SEPARATE
    weights = jg.JG_WEIGHTS_COPY if args.weights == "copy" else jg.JG_WEIGHTS_DIRECT
    with JigsawLinear(M, K, N, ways, combine=combine, weights=weights, op=jg.JG_OP_XTW, tail=tail_of(args),
                      dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        L.shard(X, W)
        del X, W
        sec, gemm_ms, gemm_n, copy_ms, comb_ms = time_forward(L, jg, args.steps, args.warmup)
        flops = L.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.query(jg.JG_Q_GEMM_LAUNCHES)
        avg = gemm_ms / max(gemm_n, 1)
        out = dict(ms_per_step=sec * 1e3, items_per_s=M * K / sec, tflops=flops / sec / 1e12,
                   gemm_avg_launch_ms=avg, gemm_launches_timed=gemm_n,
                   gemm_tflops=(flops / launches) / (avg * 1e-3) / 1e12 if gemm_n else None,
                   other_kernels_ms_per_step=copy_ms + comb_ms,
                   hbm_algo_gbps=L.query(jg.JG_Q_HBM_BYTES_ALGO) / sec / 1e9, workspace_bytes=L.ws_bytes)
    torch.cuda.empty_cache()
    return out


def measure_encoder(cfg, ways, args):
    """One step = jg_shard_patches (field -> X shards) + jg_linear_forward; field and weights resident in HBM."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawLinear
    C, H, W, p, N, seed = cfg["C"], cfg["H"], cfg["W"], cfg["p"], cfg["N"], cfg["seed"]
    M, K = (H // p) * (W // p), C * p * p
    dev = torch.device("cuda", 0)
    field = inputs.matrix_torch(seed, C * H, W, "R", 0, device=dev).reshape(C, H, W)
    Wt = inputs.matrix_torch(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP, device=dev)
    with JigsawLinear(M, K, N, ways, tail=tail_of(args)) as L:
        L.shard(None, Wt)
        del Wt

        class Step:            # what time_forward drives
            ctx = L.ctx

            @staticmethod
            def forward():
                L.shard_patches(field, p)
                L.forward()

        for k in (jg.JG_KERNEL_SHARD,):
            jg.jg_profile_read(L.ctx, k)
        sec, gemm_ms, gemm_n, copy_ms, comb_ms = time_forward(Step, jg, args.steps, args.warmup)
        sh_ms, sh_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_SHARD)
        flops = L.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.query(jg.JG_Q_GEMM_LAUNCHES)
        avg = gemm_ms / max(gemm_n, 1)
        out = dict(ms_per_step=sec * 1e3, items_per_s=M * K / sec, tflops=flops / sec / 1e12,
                   gemm_avg_launch_ms=avg, gemm_launches_timed=gemm_n,
                   gemm_tflops=(flops / launches) / (avg * 1e-3) / 1e12 if gemm_n else None,
                   other_kernels_ms_per_step=copy_ms + comb_ms + sh_ms / args.steps,
                   patch_shard_gbps=8.0 * M * K / (sh_ms / max(sh_n, 1) * 1e-3) / 1e9 if sh_n else None,
                   M=M, K=K)
    torch.cuda.empty_cache()
    return out


def cpu_baseline_encoder(cfg, seconds):
    """Oracle: plain-loop patch rearrangement of a band of the field, then the forward oracle on those rows."""
    import oracle
    from paper_2507_05753_amd import inputs
    C, H, W, p, N, seed = cfg["C"], cfg["H"], cfg["W"], cfg["p"], cfg["N"], cfg["seed"]
    K, wp = C * p * p, W // p
    cores = min(oracle.host_threads(), 16)
    Wt = inputs.matrix(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP)

    def run(bands):            # bands of p field rows = wp patches each
        import numpy as np
        ids = [c * H + y for c in range(C) for y in range(bands * p)]
        band = inputs.matrix_rows(seed, W, ids, "R").reshape(C, bands * p, W)
        t0 = time.perf_counter()
        P = oracle.patchify(band, p)
        oracle.linear_rows(P, Wt, None, 0, P.shape[0], nthreads=cores)
        return time.perf_counter() - t0, P.shape[0]

    dt, rows = run(1)
    bands = int(max(1, min(H // p, seconds / max(dt, 1e-9))))
    dt, rows = run(bands)
    return dict(value=rows * K / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"{bands} band(s) of {p} field rows = {rows} patches x {K} features against all of W "
                       f"({N} x {K}), {dt:.1f} s, plain-loop rearrangement + fp64 triple loop")


def measure_mlp(cfg, ways, args):
    """One step = one jg_mlp_forward: H = gelu(X W1^T + b1), Y = X + H W2^T + b2, shards resident in HBM."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawMLP
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    dev = torch.device("cuda", 0)
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device=dev)
    with JigsawMLP(M, C, Hd, ways, tail=tail_of(args), dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        L.shard(gen(seed, M, C), gen(seed + 1, Hd, C, inputs.W_SCALE_EXP), gen(seed + 2, 1, Hd)[0].contiguous(),
                gen(seed + 3, C, Hd, inputs.W_SCALE_EXP), gen(seed + 4, 1, C)[0].contiguous())
        sec, gemm_ms, gemm_n, copy_ms, comb_ms = time_forward(L, jg, args.steps, args.warmup)
        flops = L.first.query(jg.JG_Q_FLOPS_TOTAL) + L.second.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.first.query(jg.JG_Q_GEMM_LAUNCHES) + L.second.query(jg.JG_Q_GEMM_LAUNCHES)
        avg = gemm_ms / max(gemm_n, 1)
        out = dict(ms_per_step=sec * 1e3, items_per_s=M * C / sec, tflops=flops / sec / 1e12,
                   gemm_avg_launch_ms=avg, gemm_launches_timed=gemm_n,
                   gemm_tflops=(flops / launches) / (avg * 1e-3) / 1e12 if gemm_n else None,
                   other_kernels_ms_per_step=copy_ms + comb_ms, workspace_bytes=L.ws_bytes)
    torch.cuda.empty_cache()
    return out


def measure_mixing(cfg, ways, args):
    """One step = one jg_mixing_forward: Xn = layernorm(X), H = gelu(Xn W1^T + b1), Y = X + H W2^T + b2."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawMixing
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    dev = torch.device("cuda", 0)
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device=dev)
    with JigsawMixing(M, C, Hd, ways, tail=tail_of(args), dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        L.shard(gen(seed, M, C), (gen(seed + 5, 1, C)[0] + 1.5).contiguous(), gen(seed + 6, 1, C)[0].contiguous(),
                gen(seed + 1, Hd, C, inputs.W_SCALE_EXP), gen(seed + 2, 1, Hd)[0].contiguous(),
                gen(seed + 3, C, Hd, inputs.W_SCALE_EXP), gen(seed + 4, 1, C)[0].contiguous())
        norm = {}
        sec, gemm_ms, gemm_n, copy_ms, comb_ms = time_forward(L, jg, args.steps, args.warmup, norm)
        flops = L.first.query(jg.JG_Q_FLOPS_TOTAL) + L.second.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.first.query(jg.JG_Q_GEMM_LAUNCHES) + L.second.query(jg.JG_Q_GEMM_LAUNCHES)
        avg = gemm_ms / max(gemm_n, 1)
        norm_avg = norm["ms"] / max(norm["launches"], 1)
        out = dict(ms_per_step=sec * 1e3, items_per_s=M * C / sec, tflops=flops / sec / 1e12,
                   gemm_avg_launch_ms=avg, gemm_launches_timed=gemm_n,
                   gemm_tflops=(flops / launches) / (avg * 1e-3) / 1e12 if gemm_n else None,
                   other_kernels_ms_per_step=copy_ms + comb_ms, workspace_bytes=L.ws_bytes,
                   norm_avg_launch_ms=norm_avg, norm_launches_timed=norm["launches"],
                   norm_gbps=norm_bytes_per_element(args) * M * C / (norm_avg * 1e-3) / 1e9 if norm["launches"] else None)
    torch.cuda.empty_cache()
    return out


def measure_token_mixing(cfg, ways, args):
    """One step = one jg_token_mixing_forward: Xn = layernorm(X), H = gelu(Xn^T W1 + b1), Y = X + W2 H^T + b2 1^T."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    T, C, D, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    dev = torch.device("cuda", 0)
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device=dev)
    with JigsawTokenMixing(T, C, D, ways, tail=tail_of(args), dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        L.shard(gen(seed, T, C), (gen(seed + 5, 1, C)[0] + 1.5).contiguous(), gen(seed + 6, 1, C)[0].contiguous(),
                gen(seed + 1, T, D, inputs.W_SCALE_EXP), gen(seed + 2, 1, D)[0].contiguous(),
                gen(seed + 3, T, D, inputs.W_SCALE_EXP), gen(seed + 4, 1, T)[0].contiguous())
        norm = {}
        sec, gemm_ms, gemm_n, copy_ms, comb_ms = time_forward(L, jg, args.steps, args.warmup, norm)
        flops = L.first.query(jg.JG_Q_FLOPS_TOTAL) + L.second.query(jg.JG_Q_FLOPS_TOTAL)
        launches = L.first.query(jg.JG_Q_GEMM_LAUNCHES) + L.second.query(jg.JG_Q_GEMM_LAUNCHES)
        avg = gemm_ms / max(gemm_n, 1)
        norm_avg = norm["ms"] / max(norm["launches"], 1)
        out = dict(ms_per_step=sec * 1e3, items_per_s=T * C / sec, tflops=flops / sec / 1e12,
                   gemm_avg_launch_ms=avg, gemm_launches_timed=gemm_n,
                   gemm_tflops=(flops / launches) / (avg * 1e-3) / 1e12 if gemm_n else None,
                   other_kernels_ms_per_step=copy_ms + comb_ms, workspace_bytes=L.ws_bytes,
                   norm_avg_launch_ms=norm_avg, norm_launches_timed=norm["launches"],
                   norm_gbps=12.0 * T * C / (norm_avg * 1e-3) / 1e9 if norm["launches"] else None)
    torch.cuda.empty_cache()
    return out


def cpu_baseline_token_mixing(cfg, seconds, terms=0):
    """The token-mixing oracle timed on a bounded sample of channels (columns of X; the norm sees only those)."""
    import oracle
    from paper_2507_05753_amd import inputs
    import numpy as np
    T, C, D, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    W1 = inputs.matrix(seed + 1, T, D, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, D, "R")[0]
    W2 = inputs.matrix(seed + 3, T, D, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, T, "R")[0]
    X = inputs.matrix(seed, T, C, "R")

    def run(ch):
        Xs = np.ascontiguousarray(X[:, :ch])
        gamma = (inputs.matrix(seed + 5, 1, C, "R")[0][:ch] + 1.5).astype("float32")
        beta = inputs.matrix(seed + 6, 1, C, "R")[0][:ch]
        t0 = time.perf_counter()
        if terms:
            oracle.token_mixing_block_reduced(1, Xs, gamma, beta, W1, b1, W2, b2, terms)
        else:
            oracle.token_mixing_block(1, Xs, gamma, beta, W1, b1, W2, b2)
        return time.perf_counter() - t0

    probe = min(C, 4)
    rate = probe / max(run(probe), 1e-9)
    ch = int(min(C, max(probe, rate * seconds)))
    dt = run(ch)
    return dict(value=ch * T / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"channels 0..{ch - 1} of X ({T} x {ch}) through the norm and both layers ({D} hidden), {dt:.1f} s, "
                       f"fp64 loops")


def norm_bytes_per_element(args):
    """The layer norm reads and writes FP32; in a mixed-precision block it also writes the first layer's rounded input."""
    return {"f32": 8.0, "bf16": 10.0, "bf16x3": 12.0}[args.dtype]


def reduced_terms(args):
    return {"f32": 0, "bf16": 1, "bf16x3": 3}[args.dtype]


def time_block_backward(L, dY, n_items, args, jg):
    """Times L.backward(dY) of a block holder whose forward has run; per-kernel-class HIP-event times per step."""
    import torch
    names = {"dx": jg.JG_KERNEL_GEMM_DX, "dw": jg.JG_KERNEL_GEMM_DW, "a": jg.JG_KERNEL_GEMM, "norm": jg.JG_KERNEL_NORM,
             "db": jg.JG_KERNEL_REDUCE, "elementwise": jg.JG_KERNEL_COMBINE, "join": jg.JG_KERNEL_JOIN,
             "weight_copy": jg.JG_KERNEL_WEIGHT_COPY}
    for _ in range(args.warmup):
        L.backward(dY)
    torch.cuda.synchronize()
    for k in names.values():
        jg.jg_profile_read(L.ctx, k)
    jg.jg_profile_read(L.ctx, jg.JG_KERNEL_SHARD)
    jg.jg_profile(L.ctx, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        L.backward(dY)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    jg.jg_profile(L.ctx, False)
    shard_ms, shard_n = jg.jg_profile_read(L.ctx, jg.JG_KERNEL_SHARD)
    kernels = {}
    if L.dtype == jg.JG_F32:       # dY is sharded by the wrapper on every call: not part of the step
        sec -= shard_ms * 1e-3 / args.steps
    else:                          # mixed precision: the rounding passes are part of the step, and the same class;
        # the wrapper's copy of dY onto shards is in that class too and stays in: the step is overstated by it
        kernels["rounding_and_dy_shard"] = dict(ms_per_step=shard_ms / args.steps, launches_per_step=shard_n / args.steps)
    for name, k in names.items():
        ms, n = jg.jg_profile_read(L.ctx, k)
        kernels[name] = dict(ms_per_step=ms / args.steps, launches_per_step=n / args.steps)
    f, s2 = L.first, L.second
    flops = (f.query(jg.JG_Q_BACKWARD_FLOPS_TOTAL) + s2.query(jg.JG_Q_BACKWARD_FLOPS_TOTAL) +
             f.query(jg.JG_Q_FLOPS_TOTAL))
    gemm_ms = sum(kernels[k]["ms_per_step"] for k in ("dx", "dw", "a"))
    return dict(ms_per_step=sec * 1e3, items_per_s=n_items / sec, tflops=flops / sec / 1e12, kernels=kernels,
                gemm_tflops=flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else None, gemm_ms_per_step=gemm_ms,
                workspace_bytes=L.bw_ws_bytes)


def measure_mixing_backward(cfg, ways, args):
    """One step = one jg_mixing_backward after a forward pass: the gradients of the channel-mixing block."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawMixing
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    dev = torch.device("cuda", 0)
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device=dev)
    with JigsawMixing(M, C, Hd, ways, tail=tail_of(args), dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        L.keep_masters = True
        L.shard(gen(seed, M, C), (gen(seed + 5, 1, C)[0] + 1.5).contiguous(), gen(seed + 6, 1, C)[0].contiguous(),
                gen(seed + 1, Hd, C, inputs.W_SCALE_EXP), gen(seed + 2, 1, Hd)[0].contiguous(),
                gen(seed + 3, C, Hd, inputs.W_SCALE_EXP), gen(seed + 4, 1, C)[0].contiguous())
        L.forward()
        out = time_block_backward(L, gen(seed + 7, M, C), M * C, args, jg)
    torch.cuda.empty_cache()
    return out


def measure_token_mixing_backward(cfg, ways, args):
    """One step = one jg_token_mixing_backward after a forward pass: the gradients of the token-mixing block."""
    import torch
    from paper_2507_05753_amd import binding as jg
    from paper_2507_05753_amd import inputs
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    T, C, D, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    dev = torch.device("cuda", 0)
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device=dev)
    with JigsawTokenMixing(T, C, D, ways, tail=tail_of(args), dtype=dtype_of(args, jg), accumulate=acc_of(args)) as L:
        L.keep_masters = True
        L.shard(gen(seed, T, C), (gen(seed + 5, 1, C)[0] + 1.5).contiguous(), gen(seed + 6, 1, C)[0].contiguous(),
                gen(seed + 1, T, D, inputs.W_SCALE_EXP), gen(seed + 2, 1, D)[0].contiguous(),
                gen(seed + 3, T, D, inputs.W_SCALE_EXP), gen(seed + 4, 1, T)[0].contiguous())
        L.forward()
        out = time_block_backward(L, gen(seed + 7, T, C), T * C, args, jg)
    torch.cuda.empty_cache()
    return out


def cpu_baseline_token_mixing_backward(cfg, seconds, terms=0):
    """The oracle's backward of the token-mixing block timed on a bounded sample of channels (columns of X and dY;
    the norm sees only those)."""
    import oracle
    from paper_2507_05753_amd import inputs
    import numpy as np
    T, C, D, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    W1 = inputs.matrix(seed + 1, T, D, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, D, "R")[0]
    W2 = inputs.matrix(seed + 3, T, D, "R", inputs.W_SCALE_EXP)
    X = inputs.matrix(seed, T, C, "R")
    dY = inputs.matrix(seed + 7, T, C, "R")
    gamma = (inputs.matrix(seed + 5, 1, C, "R")[0] + 1.5).astype("float32")
    beta = inputs.matrix(seed + 6, 1, C, "R")[0]

    def run(ch):
        Xs, Gs = np.ascontiguousarray(X[:, :ch]), np.ascontiguousarray(dY[:, :ch])
        t0 = time.perf_counter()
        if terms:
            oracle.token_mixing_block_backward_reduced(1, Xs, gamma[:ch], beta[:ch], W1, b1, W2, Gs, terms)
        else:
            oracle.token_mixing_block_backward(1, Xs, gamma[:ch], beta[:ch], W1, b1, W2, Gs)
        return time.perf_counter() - t0

    # a probe's time holds a fixed part (the weights converted to double): scaling it up underestimates the sample,
    # so the run stays within the budget plus that fixed part
    probe = min(C, 16)
    ch = int(min(C, max(probe, probe * seconds / max(run(probe), 1e-9))))
    dt = run(ch)
    return dict(value=ch * T / dt, unit="items/s", cores=oracle.host_threads(), kind="oracle",
                sample=f"channels 0..{ch - 1} of X and dY ({T} x {ch}) through the block's backward ({D} hidden; the "
                       f"weight gradients are those channels' share), {dt:.1f} s, fp64")


def cpu_baseline_mixing_backward(cfg, seconds, terms=0):
    """The oracle's backward of the mixing block timed on a bounded sample of tokens (rows of X and dY)."""
    import oracle
    from paper_2507_05753_amd import inputs
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    W1 = inputs.matrix(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    W2 = inputs.matrix(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP)
    gamma = inputs.matrix(seed + 5, 1, C, "R")[0] + 1.5
    beta = inputs.matrix(seed + 6, 1, C, "R")[0]

    def run(rows):
        X = inputs.matrix(seed, M, C, "R", row_begin=0, row_end=rows)
        dY = inputs.matrix(seed + 7, M, C, "R", row_begin=0, row_end=rows)
        t0 = time.perf_counter()
        if terms:
            oracle.mixing_block_backward_reduced(1, X, gamma, beta, W1, b1, W2, dY, terms)
        else:
            oracle.mixing_block_backward(1, X, gamma, beta, W1, b1, W2, dY)
        return time.perf_counter() - t0

    # a probe's time holds a fixed part (the weights converted to double): scaling it up underestimates the sample,
    # so the run stays within the budget plus that fixed part
    probe = min(M, 128)
    rows = int(min(M, max(probe, probe * seconds / max(run(probe), 1e-9))))
    dt = run(rows)
    return dict(value=rows * C / dt, unit="items/s", cores=oracle.host_threads(), kind="oracle",
                sample=f"tokens 0..{rows - 1} of X and dY ({rows} x {C}) through the block's backward ({Hd} hidden; "
                       f"the weight gradients are those rows' share), {dt:.1f} s, fp64")


def cpu_baseline_mixing(cfg, seconds, terms=0):
    """The mixing-block oracle (layer norm + MLP + skip) timed on a bounded sample of tokens (rows of X)."""
    import oracle
    from paper_2507_05753_amd import inputs
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    W1 = inputs.matrix(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    W2 = inputs.matrix(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]
    gamma = inputs.matrix(seed + 5, 1, C, "R")[0] + 1.5
    beta = inputs.matrix(seed + 6, 1, C, "R")[0]

    def run(rows):
        X = inputs.matrix(seed, M, C, "R", row_begin=0, row_end=rows)
        t0 = time.perf_counter()
        if terms:
            oracle.mixing_block_reduced(1, X, gamma, beta, W1, b1, W2, b2, terms)
        else:
            Xn = oracle.layernorm(X, gamma, beta, 1, nthreads=cores)
            oracle.mlp(Xn.astype("float32"), W1, b1, W2, b2, residual=False, nthreads=cores)["Y"] + X
        return time.perf_counter() - t0

    probe = min(M, 2 * cores)
    rate = probe / max(run(probe), 1e-9)
    rows = int(min(M, max(probe, rate * seconds)))
    rows = min(M, max(cores, rows // cores * cores))
    dt = run(rows)
    return dict(value=rows * C / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"tokens 0..{rows - 1} of X ({rows} x {C}) through the norm and both layers ({Hd} hidden), "
                       f"{dt:.1f} s, " + ("fp64 loops" if not terms else f"bfloat16 rounding / split + fp64 loops, {terms} per layer"))


def cpu_baseline_mlp(cfg, seconds, terms=0):
    """The MLP oracle timed on a bounded sample of tokens (rows of X)."""
    import oracle
    from paper_2507_05753_amd import inputs
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    W1 = inputs.matrix(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    W2 = inputs.matrix(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]

    def run(rows):
        X = inputs.matrix(seed, M, C, "R", row_begin=0, row_end=rows)
        t0 = time.perf_counter()
        if terms:
            oracle.mlp_reduced(X, W1, b1, W2, b2, terms, nthreads=cores)
        else:
            oracle.mlp(X, W1, b1, W2, b2, nthreads=cores)
        return time.perf_counter() - t0

    probe = min(M, 2 * cores)
    rate = probe / max(run(probe), 1e-9)
    rows = int(min(M, max(probe, rate * seconds)))
    rows = min(M, max(cores, rows // cores * cores))
    dt = run(rows)
    return dict(value=rows * C / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"tokens 0..{rows - 1} of X ({rows} x {C}) through both layers ({Hd} hidden), {dt:.1f} s, "
                       + ("fp64 loops" if not terms else f"bfloat16 rounding / split + fp64 loops, {terms} per layer"))


def cpu_baseline_xtw(cfg, seconds, terms=0):
    """The transposed-layer oracle timed on a bounded sample of channels (columns of X = rows of Y)."""
    import numpy as np
    import oracle
    from paper_2507_05753_amd import inputs
    K, M, N, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    X = inputs.matrix(seed, K, M, "R")
    W = inputs.matrix(seed + inputs.W_STREAM, K, N, "R", inputs.W_SCALE_EXP)

    def run(ch):
        Xs = np.ascontiguousarray(X[:, :ch])
        t0 = time.perf_counter()
        if terms:
            oracle.linear_xtw_reduced(Xs, W, None, terms, nthreads=cores)
        else:
            oracle.linear_xtw(Xs, W, None, nthreads=cores)
        return time.perf_counter() - t0

    probe = min(M, cores)
    rate = probe / max(run(probe), 1e-9)            # channels per second
    ch = int(min(M, max(probe, rate * seconds)))
    ch = min(M, max(cores, ch // cores * cores))
    dt = run(ch)
    return dict(value=ch * K / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"channels 0..{ch - 1} of X ({K} x {ch}) against all of W ({K} x {N}), {dt:.1f} s, "
                       + ("fp64 loops" if not terms else f"bfloat16 rounding / split + fp64 loops, {terms} product(s)"))


def cpu_baseline_backward(cfg, seconds, terms=0):
    """The backward oracle timed on a bounded row sample (dX rows and the matching share of dW)."""
    import oracle
    from paper_2507_05753_amd import inputs
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    W = inputs.matrix(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP)

    def run(rows):
        X = inputs.matrix(seed, M, K, cfg["x_mode"], row_begin=0, row_end=rows)
        dY = inputs.matrix(seed + 3000, M, N, "R", row_begin=0, row_end=rows)
        t0 = time.perf_counter()
        if terms:
            oracle.backward_reduced(X, W, dY, terms, nthreads=cores)
        else:
            oracle.backward(X, W, dY, nthreads=cores)
        return time.perf_counter() - t0

    probe = min(M, 4 * cores)
    rate = probe / max(run(probe), 1e-9)
    rows = int(min(M, max(probe, rate * seconds)))
    dt = run(rows)
    return dict(value=rows * K / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"dX and dW from rows 0..{rows - 1} of X and dY ({rows} x {K}, {rows} x {N}) and all of W, "
                       f"{dt:.1f} s, " + ("fp64 loops" if not terms else f"bfloat16 rounding / split + fp64 loops, {terms} product(s)"))


def cpu_baseline(cfg, seconds, reduced_terms=0):
    """The oracle as it stands, timed on a bounded sample of rows of the same workload (reduced_terms = 1 or 3:
    the reduced-precision layer, operands rounded or split first)."""
    import numpy as np
    import oracle
    from paper_2507_05753_amd import inputs
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    cores = min(oracle.host_threads(), 16)
    W = inputs.matrix(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP)
    probe = min(M, 2 * cores)
    Xp = inputs.matrix(seed, M, K, cfg["x_mode"], row_begin=0, row_end=probe)
    t0 = time.perf_counter()
    oracle.linear_rows(Xp, W, None, 0, probe, nthreads=cores)
    rate = probe / max(time.perf_counter() - t0, 1e-9)          # rows per second
    rows = int(min(M, max(probe, rate * seconds)))
    rows = max(cores, rows // cores * cores)
    rows = min(rows, M)
    if reduced_terms == 3:
        rows = max(cores, rows // 3 // cores * cores)
    Xs = inputs.matrix(seed, M, K, cfg["x_mode"], row_begin=0, row_end=rows)
    t0 = time.perf_counter()
    if reduced_terms:
        Y = oracle.linear_reduced(Xs, W, None, reduced_terms, nthreads=cores)
    else:
        Y = oracle.linear_rows(Xs, W, None, 0, rows, nthreads=cores)
    dt = time.perf_counter() - t0
    assert np.isfinite(Y).all()
    how = {0: "fp64 triple loop", 1: "bfloat16 rounding + fp64 triple loop",
           3: "bfloat16 split + three fp64 triple loops"}[reduced_terms]
    return dict(value=rows * K / dt, unit="items/s", cores=cores, kind="oracle",
                sample=f"rows 0..{rows - 1} of X ({rows} x {K}) against all of W ({N} x {K}), {dt:.1f} s, {how}")


# HBM-side bytes per GEMM launch, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by
# what the same counters read for the plain copy kernel of known size; the runs, the raw readings and
# the factors are in profiles/gemm_f32_stream_forward_config3_ways4_hbm_counters.md.  Counters cannot be read
# from inside this script, so the figure is quoted, keyed by workload, and is null for the others.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {
    ("config3", 4): 3.76e9,   # reads 3.35 GB (FETCH_SIZE / 0.5118) + writes 0.405 GB (WRITE_SIZE / 1.0001)
    # jg::gemm_bf16_nt, whole tiles (profiles/gemm_bf16_nt_forward_config3_kernel_trace.md): reads 1.51 GB, writes 0.46 GB
    ("config3", 1, "bf16"): 1.98e9,
}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all n ranks of the layer are virtual ranks on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    from paper_2507_05753_amd import inputs
    if args.dtype != "f32" and args.op not in ("forward", "backward", "xtw", "mlp", "mixing", "mixing_backward",
                                               "token_mixing", "token_mixing_backward"):
        print("bench.py: --dtype bf16 / bf16x3 does not go with --op encoder or --op xw",
              file=sys.stderr)
        sys.exit(2)

    if args.op == "xw":
        cfg = inputs.CONFIGS[args.config]
        r = measure_xw(cfg, args.ways, args)
        M, K, N = cfg["M"], cfg["K"], cfg["N"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"config {args.config}: Y = X W, M={M} K={K} N={N}, W stored [K, N], "
                                   f"{args.ways}-way Jigsaw, fp32",
                       "n_items": M * K, "ways": args.ways, "M": M, "K": K, "N": N, "seed": cfg["seed"],
                       "x_values": cfg["x_mode"], "op": "xw", "weights": args.weights, "tail": args.tail, "mode": "f32"},
            "tflops": r["tflops"], "hbm_algo_gbps": r["hbm_algo_gbps"],
            "roofline": gemm_roofline(args, r),
            "other_kernels_ms_per_step": r["other_kernels_ms_per_step"],
        }
        line["roofline"]["kernel"] = "jg::gemm_f32_stream<false, true, false>"
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_xw(cfg, args.cpu_seconds)
        print(json.dumps(line), flush=True)
        return

    if args.op == "xtw":
        xc = inputs.XTW_CONFIGS["token_mixing_1b"]
        r = measure_xtw(xc, args.ways, args)
        K, M, N = xc["K"], xc["M"], xc["N"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"token mixing of the 1B model: Y = X^T W, X {K} x {M} [tokens, channels], "
                                   f"W {K} x {N}, {args.ways}-way Jigsaw, {precision_words(args)}",
                       "n_items": M * K, "ways": args.ways, "M": M, "K": K, "N": N, "seed": xc["seed"],
                       "x_values": "R", "op": "xtw", "combine": args.combine, "weights": args.weights, "tail": args.tail,
                       "mode": args.dtype},
            "tflops": r["tflops"], "hbm_algo_gbps": r["hbm_algo_gbps"],
            "roofline": gemm_roofline(args, r),
            "other_kernels_ms_per_step": r["other_kernels_ms_per_step"],
        }
        if args.dtype == "f32":
            line["roofline"]["kernel"] = "jg::gemm_f32_stream<true, true, false>"
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_xtw(xc, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    if args.op == "token_mixing":
        xc = inputs.XTW_CONFIGS["token_mixing_1b"]
        r = measure_token_mixing(xc, args.ways, args)
        T, C, D = xc["K"], xc["M"], xc["N"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"token-mixing half of a mixing block of the 1B model: Xn = layernorm(X), "
                                   f"H = gelu(Xn^T W1 + b1), Y = X + W2 H^T + b2, X {T} x {C} [tokens, channels], "
                                   f"hidden {D}, {args.ways}-way Jigsaw, {precision_words(args)}",
                       "n_items": T * C, "ways": args.ways, "T": T, "C": C, "D": D, "seed": xc["seed"],
                       "x_values": "R", "op": "token_mixing", "tail": args.tail, "mode": args.dtype},
            "tflops": r["tflops"],
            "roofline": gemm_roofline(args, r),
            "layernorm": {"bound": "hbm", "kernel": "jg::layernorm_rows_f32", "achieved": r["norm_gbps"],
                          "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                          "frac": r["norm_gbps"] / HBM_PEAK_GBPS if r["norm_gbps"] else None,
                          "avg_launch_ms": r["norm_avg_launch_ms"], "launches": r["norm_launches_timed"],
                          "bytes_per_element": 12},
            "other_kernels_ms_per_step": r["other_kernels_ms_per_step"],
        }
        if args.dtype == "f32":
            line["roofline"]["kernel"] = "jg::gemm_f32_stream (<true, true> and <false, false>)"
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_token_mixing(xc, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    if args.op == "encoder":
        ec = inputs.ENCODER_CONFIGS["encoder_1b"]
        r = measure_encoder(ec, args.ways, args)
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"patch encoder of the 1B model: field {ec['C']} x {ec['H']} x {ec['W']}, "
                                   f"{ec['p']} x {ec['p']} patches -> {r['M']} x {r['K']} . W^T ({ec['N']} x {r['K']}), "
                                   f"{args.ways}-way Jigsaw, fp32",
                       "n_items": r["M"] * r["K"], "ways": args.ways, "M": r["M"], "K": r["K"], "N": ec["N"],
                       "seed": ec["seed"], "x_values": "R", "op": "encoder", "tail": args.tail},
            "tflops": r["tflops"],
            "roofline": {"bound": "mfma", "kernel": "jg::gemm_f32_stream<false, false, false>",
                         "achieved": r["gemm_tflops"], "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": r["gemm_tflops"] / FP32_MFMA_PEAK_TFLOPS if r["gemm_tflops"] else None,
                         "avg_launch_ms": r["gemm_avg_launch_ms"], "launches": r["gemm_launches_timed"],
                         "traffic": None},
            "other_kernels_ms_per_step": r["other_kernels_ms_per_step"],
            "streaming": {"patch_shard_gbps": r["patch_shard_gbps"],
                          "patch_shard_frac": r["patch_shard_gbps"] / HBM_PEAK_GBPS if r["patch_shard_gbps"] else None},
        }
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_encoder(ec, args.cpu_seconds)
        print(json.dumps(line), flush=True)
        return

    if args.op == "mixing":
        mc = inputs.MLP_CONFIGS["channel_mixing_1b"]
        r = measure_mixing(mc, args.ways, args)
        M, C, Hd = mc["M"], mc["C"], mc["Hd"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"channel-mixing half of a mixing block of the 1B model: Xn = layernorm(X), "
                                   f"H = gelu(Xn W1^T + b1), Y = X + H W2^T + b2, X {M} x {C}, hidden {Hd}, "
                                   f"{args.ways}-way Jigsaw, {precision_words(args)}",
                       "n_items": M * C, "ways": args.ways, "M": M, "C": C, "Hd": Hd, "seed": mc["seed"],
                       "x_values": "R", "op": "mixing", "tail": args.tail, "mode": args.dtype},
            "tflops": r["tflops"],
            "roofline": gemm_roofline(args, r),
            "layernorm": {"bound": "hbm", "kernel": "jg::layernorm_rows_f32", "achieved": r["norm_gbps"],
                          "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                          "frac": r["norm_gbps"] / HBM_PEAK_GBPS if r["norm_gbps"] else None,
                          "avg_launch_ms": r["norm_avg_launch_ms"], "launches": r["norm_launches_timed"],
                          "bytes_per_element": norm_bytes_per_element(args)},
            "other_kernels_ms_per_step": r["other_kernels_ms_per_step"],
        }
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_mixing(mc, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    if args.op == "mixing_backward":
        mc = inputs.MLP_CONFIGS["channel_mixing_1b"]
        r = measure_mixing_backward(mc, args.ways, args)
        M, C, Hd = mc["M"], mc["C"], mc["Hd"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"backward of the channel-mixing half of a mixing block of the 1B model: gradients "
                                   f"of Y = X + gelu(layernorm(X) W1^T + b1) W2^T + b2 for X, gamma, beta, W1, b1, W2, "
                                   f"b2; X {M} x {C}, hidden {Hd}, {args.ways}-way Jigsaw, {precision_words(args)}",
                       "n_items": M * C, "ways": args.ways, "M": M, "C": C, "Hd": Hd, "seed": mc["seed"],
                       "x_values": "R", "op": "mixing_backward", "tail": args.tail},
            "tflops": r["tflops"],
            "roofline": {"bound": "mfma",
                         "kernel": {"f32": "jg::gemm_f32_stream", "bf16": "jg::gemm_bf16_nt", "bf16x3": "jg::gemm_bf16x3_nt"}[args.dtype]
                                   + " (dX, dW and recomputed A launches together)",
                         "achieved": r["gemm_tflops"] * (3 if args.dtype == "bf16x3" else 1) if r["gemm_tflops"] else None,
                         "peak": FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": (r["gemm_tflops"] * (3 if args.dtype == "bf16x3" else 1) /
                                  (FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS))
                                 if r["gemm_tflops"] else None,
                         "ms_per_step": r["gemm_ms_per_step"], "traffic": None},
            "kernels": r["kernels"],
        }
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_mixing_backward(mc, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    if args.op == "token_mixing_backward":
        xc = inputs.XTW_CONFIGS["token_mixing_1b"]
        r = measure_token_mixing_backward(xc, args.ways, args)
        T, C, D = xc["K"], xc["M"], xc["N"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"backward of the token-mixing half of a mixing block of the 1B model: gradients of "
                                   f"Y = X + W2 gelu(layernorm(X)^T W1 + b1)^T + b2 for X, gamma, beta, W1, b1, W2, b2; "
                                   f"X {T} x {C} [tokens, channels], hidden {D}, {args.ways}-way Jigsaw, {precision_words(args)}",
                       "n_items": T * C, "ways": args.ways, "T": T, "C": C, "D": D, "seed": xc["seed"],
                       "x_values": "R", "op": "token_mixing_backward", "tail": args.tail},
            "tflops": r["tflops"],
            "roofline": {"bound": "mfma",
                         "kernel": {"f32": "jg::gemm_f32_stream", "bf16": "jg::gemm_bf16_nt", "bf16x3": "jg::gemm_bf16x3_nt"}[args.dtype]
                                   + " (dX, dW and recomputed A launches together)",
                         "achieved": r["gemm_tflops"] * (3 if args.dtype == "bf16x3" else 1) if r["gemm_tflops"] else None,
                         "peak": FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": (r["gemm_tflops"] * (3 if args.dtype == "bf16x3" else 1) /
                                  (FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS))
                                 if r["gemm_tflops"] else None,
                         "ms_per_step": r["gemm_ms_per_step"], "traffic": None},
            "kernels": r["kernels"],
        }
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_token_mixing_backward(xc, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    if args.op == "mlp":
        mc = inputs.MLP_CONFIGS["channel_mixing_1b"]
        r = measure_mlp(mc, args.ways, args)
        M, C, Hd = mc["M"], mc["C"], mc["Hd"]
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": r["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"channel-mixing MLP of the 1B model: H = gelu(X W1^T + b1), Y = X + H W2^T + b2, "
                                   f"X {M} x {C}, hidden {Hd}, {args.ways}-way Jigsaw, {precision_words(args)}",
                       "n_items": M * C, "ways": args.ways, "M": M, "C": C, "Hd": Hd, "seed": mc["seed"],
                       "x_values": "R", "op": "mlp", "tail": args.tail, "mode": args.dtype},
            "tflops": r["tflops"],
            "roofline": gemm_roofline(args, r),
            "other_kernels_ms_per_step": r["other_kernels_ms_per_step"],
        }
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_mlp(mc, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    cfg = inputs.CONFIGS[args.config]
    M, K, N = cfg["M"], cfg["K"], cfg["N"]
    dev = torch.device("cuda", 0)
    X, W = make_inputs(cfg, dev)

    if args.op == "backward":
        bw = measure_backward(cfg, args.ways, args, X, W)
        del X, W
        torch.cuda.empty_cache()
        dom = max((bw["kernels"][k] for k in ("dx", "dw")), key=lambda k: k["avg_launch_ms"] * k["launches"])
        peak = FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS
        line = {
            "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
            "value": bw["items_per_s"], "unit": "items/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": bw["ms_per_step"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"config {args.config}: dX = dY W and dW = dY^T X, M={M} K={K} N={N}, "
                                   f"{args.ways}-way Jigsaw backward, {precision_words(args)}",
                       "n_items": M * K, "ways": args.ways, "M": M, "K": K, "N": N, "seed": cfg["seed"],
                       "x_values": cfg["x_mode"], "op": "backward", "mode": args.dtype},
            "tflops": bw["tflops"],
            "roofline": {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["tflops"],
                         "peak": peak, "unit": "TFLOP/s",
                         "frac": dom["tflops"] / peak, "avg_launch_ms": dom["avg_launch_ms"],
                         "launches": dom["launches"], "traffic": None},
            "kernels": bw["kernels"],
        }
        if args.cpu_seconds > 0:
            line["cpu_baseline"] = cpu_baseline_backward(cfg, args.cpu_seconds, reduced_terms(args))
        print(json.dumps(line), flush=True)
        return

    extras = not args.only_headline
    head = measure(cfg, args.ways, args, X, W, streaming=extras, share=extras)
    by_ways, modes, configs = {}, {}, {}
    few = max(3, min(args.steps, 10))
    pick = lambda r: {k: r[k] for k in ("ms_per_step", "items_per_s", "tflops", "gemm_tflops")}
    if extras:
        mine = pick(head)
        mine["steps"] = args.steps
        by_ways[str(args.ways)] = mine
        for w in (1, 2, 4):
            if w != args.ways:
                by_ways[str(w)] = dict(pick(measure(cfg, w, args, X, W, steps=few, warmup=2)), steps=few)
        if args.combine == "fused" and args.ways > 1:
            # the separate combine kernel (measurement variant): 12 bytes per output element
            r = measure(cfg, args.ways, args, X, W, steps=few, warmup=2, combine="separate")
            if "combine_gbps" in r:
                head["combine_gbps"] = r["combine_gbps"]
        if args.dtype == "f32":
            # the reduced-precision modes of the same layer, for scale (each against the bfloat16 matrix peak)
            # (levels: the default, a second summation level between launches; single: one launch per product)
            for mode in ("bf16", "bf16x3"):
                for acc in ("levels", "single"):
                    r = measure(cfg, args.ways, args, X, W, steps=few, warmup=2, dtype=mode, accumulate=acc)
                    t = 3 if mode == "bf16x3" else 1
                    modes[f"{mode}_{acc}"] = dict(
                        pick(r), steps=few, gemm_launches_per_step=r["gemm_launches_per_step"],
                        matrix_tflops=r["gemm_tflops"] * t if r["gemm_tflops"] else None,
                        frac_of_bf16_peak=r["gemm_tflops"] * t / BF16_MFMA_PEAK_TFLOPS if r["gemm_tflops"] else None)
    del X, W
    torch.cuda.empty_cache()
    if extras:
        # the other configurations of the workload table, same launch options, a few steps each
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                continue
            cc = inputs.CONFIGS[c]
            Xc, Wc = make_inputs(cc, dev)
            n = {1: 200, 2: 200, 5: 3}.get(c, few)
            r = measure(cc, args.ways, args, Xc, Wc, steps=n, warmup=2 if c >= 3 else 20)
            configs[str(c)] = dict(pick(r), steps=n, M=cc["M"], K=cc["K"], N=cc["N"], x_values=cc["x_mode"],
                                   frac_of_peak=r["gemm_tflops"] * (3 if args.dtype == "bf16x3" else 1) /
                                   (FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS)
                                   if r["gemm_tflops"] else None)
            del Xc, Wc
            torch.cuda.empty_cache()

    reduced = args.dtype != "f32"
    terms = 3 if args.dtype == "bf16x3" else 1
    workload = (f"config {args.config}: Y = X W^T, M={M} K={K} N={N}, {args.ways}-way Jigsaw, "
                + {"f32": "fp32", "bf16": "operands rounded to bfloat16, fp32 sums",
                   "bf16x3": "operands split into two bfloat16 parts, three products, fp32 sums"}[args.dtype])
    # the matrix cores' work: the split mode multiplies three times per product of the layer
    achieved = head["gemm_tflops"] * terms if head["gemm_tflops"] else None
    peak = BF16_MFMA_PEAK_TFLOPS if reduced else FP32_MFMA_PEAK_TFLOPS
    line = {
        "metric": "hot-path items/s at n=1e8 + achieved HBM GB/s (% of MI355X peak)",
        "value": head["items_per_s"],
        "unit": "items/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if reduced else "f32",
        "data": "synthetic",
        "config": {"workload": workload, "n_items": M * K, "ways": args.ways, "M": M, "K": K, "N": N,
                   "seed": cfg["seed"], "x_values": cfg["x_mode"], "combine": args.combine,
                   "weights": args.weights, "tail": args.tail, "mode": args.dtype,
                   **({"accumulate": args.accumulate} if args.dtype != "f32" else {})},
        "tflops": head["tflops"],
        "hbm_algo_gbps": head["hbm_algo_gbps"],
        "hbm_algo_frac_of_8TBps": head["hbm_algo_frac"],
        "roofline": {
            "bound": "mfma", "kernel": ("jg::gemm_bf16x3_nt" if terms == 3 else "jg::gemm_bf16_nt") if reduced else "jg::gemm_f32_stream<false, false, false>",
            "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
            "frac": achieved / peak if achieved else None,
            "avg_launch_ms": head["gemm_avg_launch_ms"], "launches": head["gemm_launches_timed"],
            "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(
                (f"config{args.config}", args.ways, args.dtype) if reduced else (f"config{args.config}", args.ways)),
            "traffic_unit": "bytes per launch",
            "traffic_source": "quoted from profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, scaled by "
                              "a copy kernel of known size): counters cannot be read from inside the run",
        },
        "other_kernels_ms_per_step": head["other_kernels_ms_per_step"],
    }
    if "streaming" in head:
        line["streaming"] = head["streaming"]
    if "one_rank_share" in head:
        line["one_rank_share"] = head["one_rank_share"]
    if "combine_gbps" in head:
        line.setdefault("streaming", {})["combine_gbps"] = head["combine_gbps"]
        line["streaming"]["combine_frac"] = head["combine_gbps"] / HBM_PEAK_GBPS
    if by_ways:
        line["by_ways"] = by_ways
    if modes:
        line["reduced_precision"] = modes
    if configs:
        line["configs"] = configs
    if reduced:
        line["roofline"]["matrix_passes"] = terms
    if args.cpu_seconds > 0:
        line["cpu_baseline"] = cpu_baseline(cfg, args.cpu_seconds, terms if reduced else 0)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
