#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic, paper-shaped input:

  stream section (configuration 5)   fused quantize + 64-bin histogram of a 2^28-element
                                     heavy-tailed fp32 gradient tensor, one pass per format
                                     variant (binary16, bfloat16, 1/6/9, each d and n): 6 passes,
                                     8 B of algorithmic HBM traffic per element and pass
  GEMM section (configuration 3)     the ResNet-style 3x3 conv as im2col GEMM in 1/6/9/d:
                                     fused quantize + histogram of X_col, W and dY, then the
                                     forward (NT), dgrad (NN) and wgrad (TN) products
                                     (M=12544, N=256, K=2304 and permutations, 14.8 GFLOP each)

`value` is the quantize+histogram HBM rate of the stream section (GB/s, algorithmic bytes over
the section's event-timed duration); the GEMM section's useful TFLOP/s and its MFMA fraction are
reported beside it under "gemm".  Inputs are resident in HBM before the timed region starts.
The CPU oracle is timed on a bounded sample of the same tensor as a baseline.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (profiles/), scaled by the same counters on a plain copy kernel; None until measured.
MEASURED_TRAFFIC_BYTES = None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--n", type=int, default=1 << 28, help="elements of the stream tensor")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2103_15940_amd as fmt     # raises if libfmt.so is missing: there is no fallback
    import workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # ------------------------------------------------------------------ inputs (resident before timing)
    t0 = time.time()
    n = int(args.n)
    x_host = workloads.config5(n=n)
    x = torch.from_numpy(x_host).to(dev)
    y = torch.empty_like(x)
    cfg3 = workloads.config3()
    xcol = torch.from_numpy(workloads.im2col_3x3(cfg3["X"])).to(dev)      # im2col is done by the harness
    w = torch.from_numpy(cfg3["W"]).to(dev)
    dy = torch.from_numpy(cfg3["dY"]).to(dev)
    xcol_q, w_q, dy_q = torch.empty_like(xcol), torch.empty_like(w), torch.empty_like(dy)
    M, K = xcol.shape
    N = w.shape[0]
    out_fwd = torch.empty((M, N), dtype=torch.float32, device=dev)
    out_dgrad = torch.empty((M, K), dtype=torch.float32, device=dev)
    out_wgrad = torch.empty((N, K), dtype=torch.float32, device=dev)
    hists = [fmt.new_hist(dev) for _ in range(9)]
    variants = list(workloads.FORMATS.values())
    f169 = workloads.FORMATS["1/6/9/d"]
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(record=None):
        if record is not None:
            a, b, c, d = ev(), ev(), ev(), ev()
            a.record()
        for i, f in enumerate(variants):
            fmt.fmt_quantize(x, f, out=y, hist=hists[i])
        if record is not None:
            b.record()
        fmt.fmt_quantize(xcol, f169, out=xcol_q, hist=hists[6])
        fmt.fmt_quantize(w, f169, out=w_q, hist=hists[7])
        fmt.fmt_quantize(dy, f169, out=dy_q, hist=hists[8])
        if record is not None:
            c.record()
        fmt.fmt_gemm(xcol_q, w_q, f169, transB=True, out=out_fwd)          # Y    = X_col W^T
        fmt.fmt_gemm(dy_q, w_q, f169, out=out_dgrad)                        # dX   = dY W
        fmt.fmt_gemm(dy_q, xcol_q, f169, transA=True, out=out_wgrad)        # dW   = dY^T X_col
        if record is not None:
            d.record()
            record.append((a, b, c, d))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    records = []
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step(records)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3
    ms_per_step = wall_ms / args.steps

    stream_ms = sum(a.elapsed_time(b) for a, b, c, d in records) / args.steps
    cfg3_stream_ms = sum(b.elapsed_time(c) for a, b, c, d in records) / args.steps
    gemm_ms = sum(c.elapsed_time(d) for a, b, c, d in records) / args.steps

    stream_bytes = 8.0 * n * len(variants)
    stream_gbs = stream_bytes / (stream_ms * 1e-3) / 1e9
    per_launch_ms = stream_ms / len(variants)
    gemm_flops = 3 * 2.0 * M * N * K
    gemm_tflops = gemm_flops / (gemm_ms * 1e-3) / 1e12

    result = {
        "metric": "quantize+histogram HBM GB/s; 1/6/9-operand GEMM TFLOP/s (% of peak)",
        "value": round(stream_gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 bit patterns of fp32 (quantize/histogram); bf16 pieces with f32 accumulate (GEMM)",
        "data": "synthetic",
        "config": {
            "workload": "config 5 stream: fused quantize+64-bin histogram of a 2^%d-element heavy-tailed fp32 "
                        "tensor, six format variants, one pass each; config 3 GEMMs: 3x3 conv 256->256 at 14x14, "
                        "batch 64 as im2col (M=12544, N=256, K=2304), fwd+dgrad+wgrad in 1/6/9/d with fused "
                        "quantize+histogram of X_col, W, dY" % (n.bit_length() - 1),
            "stream_elements": n,
            "stream_passes": len(variants),
            "gemm_shape": [M, N, K],
        },
        "sections_ms": {"stream": round(stream_ms, 4), "config3_quantize": round(cfg3_stream_ms, 4),
                        "config3_gemms": round(gemm_ms, 4)},
        "gemm": {
            "value": round(gemm_tflops, 2), "unit": "TFLOP/s (useful, 2MNK per product)",
            "issued_tflops": round(4 * gemm_tflops, 2),
            "mfma_frac": round(4 * gemm_tflops / BF16_MFMA_PEAK_TFLOPS, 4),
            "note": "1/6/9 operands are split exactly into two bf16 pieces: 4 MFMA products per multiply",
        },
        "roofline": {
            "kernel": "stream_kernel (fused quantize + histogram)",
            "bound": "hbm",
            "achieved": round(8.0 * n / (per_launch_ms * 1e-3) / 1e9, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(8.0 * n / (per_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES,
            "launch_ms": round(per_launch_ms, 4),
            "algorithmic_bytes_per_launch": 8 * n,
        },
        "input_generation_s": round(gen_s, 1),
    }

    if not args.no_cpu_baseline:
        import oracle
        sample = min(n, 1 << 26)
        xs = x_host[:sample]
        t1 = time.perf_counter()
        for (e, m, d) in (workloads.FORMATS["1/6/9/d"], workloads.FORMATS["1/5/10/d"], workloads.FORMATS["1/8/7/n"]):
            oracle.quantize(xs, e, m, d)
            oracle.histogram(xs, e, m)
        cpu_s = time.perf_counter() - t1
        result["cpu_baseline"] = {
            "value": round(3 * 8.0 * sample / cpu_s / 1e9, 4),
            "unit": "GB/s",
            "cores": 1,
            "kind": "oracle",
            "sample": "quantize + histogram of the first 2^%d elements of the same tensor in 1/6/9/d, 1/5/10/d, "
                      "1/8/7/n (3 passes, %.1f s)" % (sample.bit_length() - 1, cpu_s),
        }

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
