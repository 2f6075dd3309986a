#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic, paper-shaped input:

  stream section (configuration 5)   fused quantize + 64-bin histogram of a 2^28-element
                                     heavy-tailed fp32 gradient tensor, one pass per format
                                     variant (binary16, bfloat16, 1/6/9, each d and n): 6 passes,
                                     8 B of algorithmic HBM traffic per element and pass
  GEMM section (configuration 4)     BERT-Large-shaped encoder-layer GEMMs at 4096 tokens in
                                     1/6/9/d: for each of the four linear layers (QKV, attention
                                     output, FFN1, FFN2) the rounding pass over X, W and dY -- fused
                                     quantize + histogram, and the rounded tensor stored as a prepared
                                     operand in the two orientations its two products need -- then
                                     forward, dgrad and wgrad on the prepared operands: 12 products,
                                     309 GFLOP
  conv section (configuration 3)     the ResNet-style 3x3 conv as im2col GEMM in 1/6/9/d: the same
                                     rounding pass over X_col, W and dY, then the forward, dgrad and
                                     wgrad products (M=12544, N=256, K=2304 and permutations,
                                     14.8 GFLOP each)

The rounding passes inside the configuration 4 and configuration 3 sections are independent of each other
and are handed to the library in ONE fmt_quantize_prepare_pair_batch call per section (every tensor read once for
its rounded copy, its statistics and both prepared orientations); the products of a section are handed over in
one fmt_gemm_prepared_batch call (--no-batch: one fmt_quantize and one fmt_prepare_pair call per tensor and one
fmt_gemm_prepared call per product, round-robin on three side streams, --gemm-streams).  The stream section runs
on one stream.

`value` is the quantize+histogram HBM rate of the stream section (GB/s, algorithmic bytes over
the section's event-timed duration); the GEMM section's useful TFLOP/s and its MFMA fraction are
reported beside it under "gemm" (configuration 4) and "gemm_config3".  Inputs are resident in HBM before the timed region starts.
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
# (profiles/stream_kernel_config5_hbm_traffic.md), scaled by the same counters on a plain 1 GiB copy.
# Vector-ALU issue rate of the chip (one instruction per lane and clock: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz)
# and the vector instructions one FMAC-8 step takes on the single-precision path (rounded count from the ISA).
VALU_LANE_INSTR_PER_S = 256 * 64 * 2.4e9
FMAC8_INSTR_PER_MAC = 12.0
MEASURED_TRAFFIC_BYTES = 2157514900   # profiles/stream_kernel_config5_hbm_traffic.md


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--n", type=int, default=1 << 28, help="elements of the stream tensor")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-copy", action="store_true",
                    help="also run three plain device-to-device copies of the stream tensor (with --gemm: of a 1 GiB tensor) before the warm-up: "
                         "a kernel of known traffic (4 B read + 4 B written per element) that calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters in rocprofv3 --pmc runs")
    ap.add_argument("--no-batch", action="store_true",
                    help="configuration 4 and 3 sections: one fmt_quantize and one fmt_prepare_pair call per tensor and one "
                         "fmt_gemm_prepared call per product on the side streams instead of the batch calls")
    ap.add_argument("--gemm-streams", type=int, default=3,
                    help="side streams the independent calls of the configuration 4 and 3 sections are spread over")
    ap.add_argument("--gemm", default=None, metavar="M,N,K[,transA,transB[,e,m,d]]",
                    help="profiling aid: run only fmt_gemm on one N(0,1) problem of this shape (default NN, 1/6/9/d), "
                         "--steps times after --warmup untimed calls, print its time and exit")
    ap.add_argument("--prepared", action="store_true",
                    help="with --gemm: prepare the operands once (untimed) and time fmt_gemm_prepared")
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

    if args.gemm:
        v = [int(t) for t in args.gemm.split(",")]
        v += [0, 0][len(v) - 3:] if len(v) < 5 else []
        v += [6, 9, 1] if len(v) < 8 else []
        Mg, Ng, Kg, tA, tB, e_, m_, d_ = v[:8]
        torch.manual_seed(0)
        A = torch.randn((Kg, Mg) if tA else (Mg, Kg), device=dev)
        B = torch.randn((Ng, Kg) if tB else (Kg, Ng), device=dev)
        C = torch.empty((Mg, Ng), device=dev)
        if args.prepared:
            Ap = fmt.fmt_prepare(A, (e_, m_, bool(d_)), trans=bool(tA))
            Bp = fmt.fmt_prepare(B, (e_, m_, bool(d_)), trans=not tB)
            call = lambda: fmt.fmt_gemm_prepared(Ap, Bp, out=C)
        else:
            call = lambda: fmt.fmt_gemm(A, B, (e_, m_, bool(d_)), transA=bool(tA), transB=bool(tB), out=C)
        if args.profile_copy:                     # 1 GiB read + 1 GiB written: calibrates FETCH_SIZE / WRITE_SIZE
            src = torch.zeros(1 << 28, device=dev)
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
        for _ in range(args.warmup):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            call()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        print(json.dumps({"gemm": [Mg, Ng, Kg, tA, tB], "format": [e_, m_, d_], "ms": round(ms, 4),
                          "useful_tflops": round(2.0 * Mg * Ng * Kg / (ms * 1e-3) / 1e12, 2)}))
        return 0

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
    cfg4 = workloads.config4()
    layers = []
    for L in cfg4["layers"]:
        X4, W4, dY4 = (torch.from_numpy(L[k]).to(dev) for k in ("X", "W", "dY"))
        layers.append({"X": X4, "W": W4, "dY": dY4, "Xq": torch.empty_like(X4), "Wq": torch.empty_like(W4),
                       "dYq": torch.empty_like(dY4),
                       "Y": torch.empty((X4.shape[0], W4.shape[0]), dtype=torch.float32, device=dev),
                       "dX": torch.empty_like(X4), "dW": torch.empty_like(W4),
                       "h": [fmt.new_hist(dev) for _ in range(3)]})
    f169 = workloads.FORMATS["1/6/9/d"]

    def operand_bufs(t):
        """Device buffers for the two prepared operands of a 2-D tensor: as stored, and transposed."""
        r, c = t.shape
        return (torch.empty(fmt.fmt_operand_bytes(r, c, f169), dtype=torch.uint8, device=dev),
                torch.empty(fmt.fmt_operand_bytes(c, r, f169), dtype=torch.uint8, device=dev))
    for L in layers:
        L["buf"] = {k: operand_bufs(L[k]) for k in ("X", "W", "dY")}
        L["op"] = {}
    c3 = {"t": {"X": xcol, "W": w, "dY": dy}, "op": {}}
    c3["buf"] = {k: operand_bufs(v) for k, v in c3["t"].items()}
    cfg4_flops = sum(3 * 2.0 * L["X"].shape[0] * L["W"].shape[0] * L["W"].shape[1] for L in layers)
    hists = [fmt.new_hist(dev) for _ in range(9)]
    variants = list(workloads.FORMATS.values())
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    ev = lambda: torch.cuda.Event(enable_timing=True)
    side = [torch.cuda.Stream() for _ in range(max(args.gemm_streams, 1))]

    def cfg4_batched():
        # Y = X W^T, dX = dY W, dW = dY^T X of the four layers handed over together (Sec. IV-A)
        A4, B4, C4 = [], [], []
        for L in layers:
            o = L["op"]
            A4 += [o["X"][0], o["dY"][0], o["dY"][1]]
            B4 += [o["W"][0], o["W"][1], o["X"][1]]
            C4 += [L["Y"], L["dX"], L["dW"]]
        fmt.fmt_gemm_prepared_batch(A4, B4, out=C4)

    def step(record=None):
        marks = []

        def mark():
            if record is not None:
                e = ev()
                e.record()
                marks.append(e)

        mark()
        for i, f in enumerate(variants):                                     # configuration 5
            fmt.fmt_quantize(x, f, out=y, hist=hists[i])
        mark()

        # Independent calls of one section go round-robin onto side streams (each stream has its own
        # library scratch): the HBM-bound operand preparation of one product overlaps the MFMA-bound
        # kernel of another, and the small kernels between the large ones (statistics, sums of partial
        # records) stop being gaps.  The section ends when every side stream has been joined.
        def fan_out(calls):
            fork = ev()
            fork.record()
            for j, call in enumerate(calls):
                st_ = side[j % len(side)]
                if j < len(side):
                    st_.wait_event(fork)
                call(st_)
            for st_ in side[:min(len(side), len(calls))]:
                join = ev()
                join.record(st_)
                torch.cuda.current_stream().wait_event(join)

        # The rounding pass of Sec. IV-A over one tensor: statistics and the rounded fp32 copy in one fused
        # pass, and the rounded tensor as a prepared operand in both orientations (each feeds one product; one call).
        def round_tensor(st_, src, dst, hist, bufs, ops, key):
            fmt.fmt_quantize(src, f169, out=dst, hist=hist, stream=st_)
            ops[key] = fmt.fmt_prepare_pair(src, f169, out=bufs[0], out_t=bufs[1], stream=st_)

        # The same for all the section's tensors in ONE call: every tensor is read once for its rounded copy, its
        # statistics and both prepared orientations (shared launches).
        def round_all(entries):
            pairs = fmt.fmt_quantize_prepare_pair_batch([e[0] for e in entries], f169, [e[1] for e in entries],
                                                        [e[2] for e in entries], outs=[e[3][0] for e in entries],
                                                        outs_t=[e[3][1] for e in entries])
            for e, pair in zip(entries, pairs):
                e[4][e[5]] = pair

        q4, p4 = [], []
        for L in layers:                                                     # configuration 4, rounding passes
            for src, dst, hi in (("X", "Xq", 0), ("W", "Wq", 1), ("dY", "dYq", 2)):
                if args.no_batch:
                    q4.append(lambda st_, L=L, src=src, dst=dst, hi=hi:
                              round_tensor(st_, L[src], L[dst], L["h"][hi], L["buf"][src], L["op"], src))
                else:
                    p4.append((L[src], L[dst], L["h"][hi], L["buf"][src], L["op"], src))
        if args.no_batch:
            fan_out(q4)
        else:
            round_all(p4)
        mark()
        if args.no_batch:                                                    # configuration 4, products
            g4 = []
            for L in layers:
                o = L["op"]
                g4.append(lambda st_, L=L, o=o: fmt.fmt_gemm_prepared(o["X"][0], o["W"][0], out=L["Y"], stream=st_))     # Y  = X W^T
                g4.append(lambda st_, L=L, o=o: fmt.fmt_gemm_prepared(o["dY"][0], o["W"][1], out=L["dX"], stream=st_))   # dX = dY W
                g4.append(lambda st_, L=L, o=o: fmt.fmt_gemm_prepared(o["dY"][1], o["X"][1], out=L["dW"], stream=st_))   # dW = dY^T X
            fan_out(g4)
        else:
            cfg4_batched()                                                   # the same twelve products, one call
        mark()
        if args.no_batch:                                                    # configuration 3
            fan_out([lambda st_: round_tensor(st_, xcol, xcol_q, hists[6], c3["buf"]["X"], c3["op"], "X"),
                     lambda st_: round_tensor(st_, w, w_q, hists[7], c3["buf"]["W"], c3["op"], "W"),
                     lambda st_: round_tensor(st_, dy, dy_q, hists[8], c3["buf"]["dY"], c3["op"], "dY")])
        else:
            round_all([(xcol, xcol_q, hists[6], c3["buf"]["X"], c3["op"], "X"), (w, w_q, hists[7], c3["buf"]["W"], c3["op"], "W"),
                       (dy, dy_q, hists[8], c3["buf"]["dY"], c3["op"], "dY")])
        mark()
        o3 = c3["op"]
        if args.no_batch:
            fan_out([lambda st_: fmt.fmt_gemm_prepared(o3["X"][0], o3["W"][0], out=out_fwd, stream=st_),      # Y  = X_col W^T
                     lambda st_: fmt.fmt_gemm_prepared(o3["dY"][0], o3["W"][1], out=out_dgrad, stream=st_),   # dX = dY W
                     lambda st_: fmt.fmt_gemm_prepared(o3["dY"][1], o3["X"][1], out=out_wgrad, stream=st_)])  # dW = dY^T X_col
        else:
            fmt.fmt_gemm_prepared_batch([o3["X"][0], o3["dY"][0], o3["dY"][1]], [o3["W"][0], o3["W"][1], o3["X"][1]],
                                        out=[out_fwd, out_dgrad, out_wgrad])
        mark()
        if record is not None:
            record.append(marks)

    if args.profile_copy:
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
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

    def section(i):
        return sum(m[i].elapsed_time(m[i + 1]) for m in records) / args.steps

    stream_ms, cfg4_q_ms, cfg4_gemm_ms, cfg3_q_ms, cfg3_gemm_ms = (section(i) for i in range(5))

    stream_bytes = 8.0 * n * len(variants)
    stream_gbs = stream_bytes / (stream_ms * 1e-3) / 1e9
    per_launch_ms = stream_ms / len(variants)
    cfg4_tflops = cfg4_flops / (cfg4_gemm_ms * 1e-3) / 1e12
    cfg3_tflops = 3 * 2.0 * M * N * K / (cfg3_gemm_ms * 1e-3) / 1e12

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
        "dtype": "u32 bit patterns of fp32 (quantize/histogram); scaled fp16 or bf16 pieces with f32 accumulate (GEMM)",
        "data": "synthetic",
        "config": {
            "workload": "config 5 stream: fused quantize+64-bin histogram of a 2^%d-element heavy-tailed fp32 "
                        "tensor, six format variants, one pass each; config 4 GEMMs: BERT-Large-shaped encoder "
                        "layer at 4096 tokens, fwd+dgrad+wgrad of QKV/attn-out/FFN1/FFN2 in 1/6/9/d with fused "
                        "quantize+histogram of X, W, dY; config 3 GEMMs: 3x3 conv 256->256 at 14x14, batch 64 as "
                        "im2col (M=12544, N=256, K=2304), fwd+dgrad+wgrad in 1/6/9/d" % (n.bit_length() - 1),
            "stream_elements": n,
            "stream_passes": len(variants),
            "config4_gemm_gflop": round(cfg4_flops / 1e9, 1),
            "config3_gemm_shape": [M, N, K],
            "side_streams": len(side),
            "products": "one fmt_prepare_pair call per tensor and single fmt_gemm_prepared calls on the side streams" if args.no_batch else "one fmt_quantize_prepare_pair_batch call and one fmt_gemm_prepared_batch call per section",
        },
        "sections_ms": {"config5_stream": round(stream_ms, 4), "config4_quantize": round(cfg4_q_ms, 4),
                        "config4_gemms": round(cfg4_gemm_ms, 4), "config3_quantize": round(cfg3_q_ms, 4),
                        "config3_gemms": round(cfg3_gemm_ms, 4)},
        "gemm": {
            "workload": "config 4, 12 products on prepared operands, 1/6/9/d, " +
                        ("12 fmt_gemm_prepared calls on %d side streams" % len(side) if args.no_batch
                         else "one fmt_gemm_prepared_batch call"),
            "value": round(cfg4_tflops, 2), "unit": "TFLOP/s (useful, 2MNK per product, whole calls)",
            "mfma_frac": round(cfg4_tflops / BF16_MFMA_PEAK_TFLOPS, 4),
            "with_rounding_passes_tflops": round(cfg4_flops / ((cfg4_gemm_ms + cfg4_q_ms) * 1e-3) / 1e12, 2),
            "note": "1/6/9 operands are exponent planes: one scaled fp16 piece per value (per-row power-of-two "
                    "scale), the few values outside a row's plane in a second or third plane whose products the same "
                    "kernel adds: 1 MFMA product per multiply, so mfma_frac = useful / 2500 TFLOP/s dense fp16 peak. "
                    "The rounding passes that make the operands (once per tensor and orientation, shared by the "
                    "products that use it) are timed in sections_ms.config4_quantize; with_rounding_passes_tflops "
                    "charges them to the products.  fmt_gemm on fp32 operands (rounds per call) and the two-bf16-piece "
                    "scheme (4 MFMA products per multiply) are measured beside it",
        },
        "gemm_config3": {
            "workload": "config 3, 3 products on prepared operands, 1/6/9/d, " +
                        ("3 fmt_gemm_prepared calls on side streams" if args.no_batch else "one fmt_gemm_prepared_batch call"),
            "value": round(cfg3_tflops, 2), "unit": "TFLOP/s (useful)",
            "with_rounding_passes_tflops": round(3 * 2.0 * M * N * K / ((cfg3_gemm_ms + cfg3_q_ms) * 1e-3) / 1e12, 2),
        },
        "roofline": {
            "kernel": "stream_kernel (fused quantize + histogram)",
            "bound": "hbm",
            "achieved": round(8.0 * n / (per_launch_ms * 1e-3) / 1e9, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(8.0 * n / (per_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES if n == (1 << 28) else None,
            "launch_ms": round(per_launch_ms, 4),
            "algorithmic_bytes_per_launch": 8 * n,
        },
        "input_generation_s": round(gen_s, 1),
    }

    # configuration 3 in all six variants (outside the step; informational): useful TFLOP/s of fwd+dgrad+wgrad
    per_format = {}
    for name, f in workloads.FORMATS.items():
        def conv3():
            fmt.fmt_gemm(xcol, w, f, transB=True, out=out_fwd)
            fmt.fmt_gemm(dy, w, f, out=out_dgrad)
            fmt.fmt_gemm(dy, xcol, f, transA=True, out=out_wgrad)
        conv3()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(max(args.steps // 2, 1)):
            conv3()
        b.record()
        torch.cuda.synchronize()
        per_format[name] = round(3 * 2.0 * M * N * K / (a.elapsed_time(b) / max(args.steps // 2, 1) * 1e-3) / 1e12, 1)
    result["gemm_config3"]["useful_tflops_by_format"] = per_format

    # configuration 4 with the two-piece scheme forced, and one large product in both schemes (informational)
    def cfg4_products():
        for L in layers:
            fmt.fmt_gemm(L["Xq"], L["Wq"], f169, transB=True, out=L["Y"])
            fmt.fmt_gemm(L["dYq"], L["Wq"], f169, out=L["dX"])
            fmt.fmt_gemm(L["dYq"], L["Xq"], f169, transA=True, out=L["dW"])

    def timed0(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    saved = os.environ.get("FMT_GEMM_WINDOW")
    os.environ["FMT_GEMM_WINDOW"] = "0"
    two_ms = timed0(cfg4_products, max(args.steps // 2, 1))
    Abig = torch.randn((8192, 8192), device=dev)
    Bbig = torch.randn((8192, 8192), device=dev) * 0.02
    Cbig = torch.empty((8192, 8192), device=dev)
    big_two_ms = timed0(lambda: fmt.fmt_gemm(Abig, Bbig, f169, out=Cbig), 3)
    if saved is None:
        del os.environ["FMT_GEMM_WINDOW"]
    else:
        os.environ["FMT_GEMM_WINDOW"] = saved
    one_ms = timed0(cfg4_products, max(args.steps // 2, 1))
    big_one_ms = timed0(lambda: fmt.fmt_gemm(Abig, Bbig, f169, out=Cbig), 3)
    del Abig, Bbig, Cbig
    big_flops = 2.0 * 8192 ** 3
    result["gemm"]["fmt_gemm_fp32_operands_tflops"] = round(cfg4_flops / (one_ms * 1e-3) / 1e12, 2)

    def cfg4_prepared():
        for L in layers:
            o = L["op"]
            fmt.fmt_gemm_prepared(o["X"][0], o["W"][0], out=L["Y"])
            fmt.fmt_gemm_prepared(o["dY"][0], o["W"][1], out=L["dX"])
            fmt.fmt_gemm_prepared(o["dY"][1], o["X"][1], out=L["dW"])
    result["gemm"]["single_calls_one_stream_tflops"] = round(cfg4_flops / (timed0(cfg4_prepared, max(args.steps // 2, 1)) * 1e-3) / 1e12, 2)
    result["gemm"]["batch_call_tflops"] = round(cfg4_flops / (timed0(cfg4_batched, max(args.steps // 2, 1)) * 1e-3) / 1e12, 2)

    # Roofline of the product kernel: the largest product of config 4 (FFN1 forward, 4096 x 4096 x 1024,
    # one launch per call), timed with events on the stream it is launched on.
    Lf = layers[2]
    Mr, Nr, Kr = Lf["X"].shape[0], Lf["W"].shape[0], Lf["W"].shape[1]
    reps_r = max(args.steps, 10)
    roof_ms = timed0(lambda: fmt.fmt_gemm_prepared(Lf["op"]["X"][0], Lf["op"]["W"][0], out=Lf["Y"]), reps_r)
    roof_tflops = 2.0 * Mr * Nr * Kr / (roof_ms * 1e-3) / 1e12
    result["roofline_gemm"] = {
        "kernel": "product_kernel<PS=0 (fp16 planes), 256x256 tile> on config 4 FFN1 forward %dx%dx%d" % (Mr, Nr, Kr),
        "bound": "mfma", "achieved": round(roof_tflops, 1), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": round(roof_tflops / BF16_MFMA_PEAK_TFLOPS, 4), "traffic": None,
        "launch_ms": round(roof_ms, 4), "algorithmic_flops_per_launch": 2.0 * Mr * Nr * Kr,
        "note": "fp16 MFMA dense peak; one MFMA product per multiply, so issued = useful flops"}
    batch_ms = timed0(cfg4_batched, reps_r)
    result["roofline_gemm"]["shared_launch"] = {
        "kernel": "product_group_kernel<PS=0, 256x256 tile> + planes_tail_group_kernel: config 4's twelve products in one "
                  "fmt_gemm_prepared_batch call",
        "achieved": round(cfg4_flops / (batch_ms * 1e-3) / 1e12, 1), "unit": "TFLOP/s",
        "frac": round(cfg4_flops / (batch_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4), "launch_ms": round(batch_ms, 4),
        "algorithmic_flops_per_launch": cfg4_flops}
    result["gemm"]["two_piece"] = {
        "value": round(cfg4_flops / (two_ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s (useful), one stream",
        "issued_tflops": round(4 * cfg4_flops / (two_ms * 1e-3) / 1e12, 2),
        "mfma_frac": round(4 * cfg4_flops / (two_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4)}
    result["gemm_8192"] = {
        "workload": "fmt_gemm 8192 x 8192 x 8192, 1/6/9/d, N(0,1) x N(0,0.02^2)",
        "value": round(big_flops / (big_one_ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s (useful)",
        "mfma_frac": round(big_flops / (big_one_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4),
        "two_piece": {"value": round(big_flops / (big_two_ms * 1e-3) / 1e12, 2),
                      "mfma_frac": round(4 * big_flops / (big_two_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4)}}

    # the layers built on top of the three base calls (outside the step; informational)
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    reps = max(args.steps // 2, 1)
    # configuration 3 through the convolution entry points (patches gathered by the operand loader)
    X4d = torch.from_numpy(cfg3["X"]).to(dev)
    nb, cin, hh, ww = X4d.shape
    W4d = w.reshape(N, cin, 3, 3).contiguous()
    dY4d = dy.reshape(nb, hh, ww, N).permute(0, 3, 1, 2).contiguous()           # the same values as NCHW
    Yc, dXc, dWc = torch.empty_like(dY4d), torch.empty_like(X4d), torch.empty_like(W4d)

    def conv_all():
        fmt.fmt_conv2d_fwd(X4d, W4d, f169, out=Yc)
        fmt.fmt_conv2d_dgrad(dY4d, W4d, X4d.shape, f169, out=dXc)
        fmt.fmt_conv2d_wgrad(dY4d, X4d, W4d.shape, f169, out=dWc)
    conv_ms = timed(conv_all, reps)
    result["conv_config3"] = {"workload": "config 3 via fmt_conv2d_fwd/_dgrad/_wgrad, 1/6/9/d, rounding of the tensors included: forward and dgrad gather the patches inside the product kernel (scratch of the tensor's size), wgrad through a gathered 16-bit operand; two bf16 pieces (4 MFMA products per multiply)",
                              "ms": round(conv_ms, 4), "value": round(3 * 2.0 * M * N * K / (conv_ms * 1e-3) / 1e12, 2),
                              "unit": "TFLOP/s (useful)"}
    by_format = {}
    for name, fv in workloads.FORMATS.items():          # binary16 and bfloat16 take one 16-bit piece (1 MFMA product per multiply)
        def conv_f(fv=fv):
            fmt.fmt_conv2d_fwd(X4d, W4d, fv, out=Yc)
            fmt.fmt_conv2d_dgrad(dY4d, W4d, X4d.shape, fv, out=dXc)
            fmt.fmt_conv2d_wgrad(dY4d, X4d, W4d.shape, fv, out=dWc)
        by_format[name] = round(3 * 2.0 * M * N * K / (timed(conv_f, max(reps // 2, 1)) * 1e-3) / 1e12, 1)
    result["conv_config3"]["useful_tflops_by_format"] = by_format
    # the operands of config 4's twelve tensors, both orientations each, by themselves: one fmt_prepare_pair_batch call
    # (two launches) against one fmt_prepare_pair call per tensor; 8 algorithmic bytes per element (4 read, 2 + 2 written)
    p4_keys = [(L, k) for L in layers for k in ("X", "W", "dY")]
    p4_src = [L[k] for L, k in p4_keys]
    p4_out, p4_out_t = [L["buf"][k][0] for L, k in p4_keys], [L["buf"][k][1] for L, k in p4_keys]
    prep_ms = timed(lambda: fmt.fmt_prepare_pair_batch(p4_src, f169, outs=p4_out, outs_t=p4_out_t), reps)

    def prepare_one_by_one():
        for t, o, ot in zip(p4_src, p4_out, p4_out_t):
            fmt.fmt_prepare_pair(t, f169, out=o, out_t=ot)
    prep1_ms = timed(prepare_one_by_one, reps)
    p4_bytes = 8.0 * sum(t.numel() for t in p4_src)
    result["prepare_config4"] = {"workload": "fmt_prepare_pair_batch: both prepared orientations of config 4's 12 tensors "
                                             "(X, W, dY of the four layers), 1/6/9/d, one call",
                                 "ms": round(prep_ms, 4), "value": round(p4_bytes / (prep_ms * 1e-3) / 1e9, 1),
                                 "unit": "GB/s (algorithmic: 4 B read + 2 + 2 B written per element; statistics launch included)",
                                 "hbm_frac": round(p4_bytes / (prep_ms * 1e-3) / 1e9 / 8000.0, 3),
                                 "single_calls_one_stream_ms": round(prep1_ms, 4)}
    # the whole rounding pass over the same tensors (rounded fp32 copy + statistics + both orientations) in one call:
    # 12 algorithmic bytes per element (4 read, 4 + 2 + 2 written)
    p4_q = [L[k] for L in layers for k in ("Xq", "Wq", "dYq")]
    p4_h = [L["h"][i] for L in layers for i in range(3)]
    round_ms = timed(lambda: fmt.fmt_quantize_prepare_pair_batch(p4_src, f169, p4_q, p4_h, outs=p4_out, outs_t=p4_out_t), reps)
    result["round_config4"] = {"workload": "fmt_quantize_prepare_pair_batch: rounded fp32 copy, statistics and both prepared "
                                           "orientations of config 4's 12 tensors, 1/6/9/d, one call",
                               "ms": round(round_ms, 4), "value": round(1.5 * p4_bytes / (round_ms * 1e-3) / 1e9, 1),
                               "unit": "GB/s (algorithmic: 4 B read + 4 + 2 + 2 B written per element; statistics launches included)",
                               "hbm_frac": round(1.5 * p4_bytes / (round_ms * 1e-3) / 1e9 / 8000.0, 3)}
    # quantized Linear forward of the four encoder layers: product, bias, both output roundings, statistics of t
    biases = [torch.zeros(L["W"].shape[0], dtype=torch.float32, device=dev) for L in layers]

    def linear_all():
        for L, b in zip(layers, biases):
            fmt.fmt_linear(L["X"], L["W"], b, f169, out=L["Y"], hist=L["h"][0])
    lin_ms = timed(linear_all, reps)
    result["linear_config4"] = {"workload": "fmt_linear forward of the 4 encoder layers (bias, output roundings, "
                                            "statistics of the output), 1/6/9/d",
                                "ms": round(lin_ms, 4), "value": round(cfg4_flops / 3 / (lin_ms * 1e-3) / 1e12, 2),
                                "unit": "TFLOP/s (useful)"}

    # the same four layers on the operands the step prepared (X and W as stored): no rounding pass in the call
    def linear_prepared_all():
        for L, b in zip(layers, biases):
            fmt.fmt_linear_prepared(L["op"]["X"][0], L["op"]["W"][0], b, out=L["Y"], hist=L["h"][0])
    linp_ms = timed(linear_prepared_all, reps)
    result["linear_config4"]["prepared"] = {"workload": "fmt_linear_prepared on the prepared operands of the step",
                                            "ms": round(linp_ms, 4),
                                            "value": round(cfg4_flops / 3 / (linp_ms * 1e-3) / 1e12, 2)}
    # the same layers and the config 5 stream with 16-bit code output (2 instead of 4 bytes written per element)
    Y16 = [torch.empty(L["Y"].shape, dtype=torch.int16, device=dev) for L in layers]

    def linear16_all():
        for L, b, o in zip(layers, biases, Y16):
            fmt.fmt_linear_pack16(L["X"], L["W"], b, f169, out=o, hist=L["h"][0])
    lin16_ms = timed(linear16_all, reps)
    codes = torch.empty(x.shape, dtype=torch.int16, device=dev)
    pack_ms = timed(lambda: fmt.fmt_pack16(x, f169, out=codes, hist=hists[0]), reps)
    unpack_ms = timed(lambda: fmt.fmt_unpack16(codes, f169, out=y), reps)
    result["pack16"] = {"workload": "16-bit code storage, 1/6/9/d: fmt_pack16 (+ statistics) and fmt_unpack16 on the "
                                    "config 5 tensor (6 B per element each), fmt_linear_pack16 on the 4 encoder layers",
                        "pack_gbps": round(6.0 * n / (pack_ms * 1e-3) / 1e9, 1),
                        "unpack_gbps": round(6.0 * n / (unpack_ms * 1e-3) / 1e9, 1),
                        "linear_ms": round(lin16_ms, 4),
                        "linear_tflops": round(cfg4_flops / 3 / (lin16_ms * 1e-3) / 1e12, 2)}
    del codes, Y16
    # the other passes over the config 5 tensor, and the device's own copy, beside `value` (informational)
    hist_ms = timed(lambda: fmt.fmt_histogram(x, f169, hist=hists[0]), reps)
    quant_ms = timed(lambda: fmt.fmt_quantize(x, f169, out=y), reps)
    copy_ms = timed(lambda: y.copy_(x), reps)
    result["stream_context"] = {
        "workload": "config 5 tensor, 1/6/9/d: fmt_histogram alone (4 B per element), fmt_quantize without "
                    "statistics (8 B per element), and the runtime's device-to-device copy of the same tensor "
                    "(8 B per element)",
        "histogram_only_gbps": round(4.0 * n / (hist_ms * 1e-3) / 1e9, 1),
        "quantize_only_gbps": round(8.0 * n / (quant_ms * 1e-3) / 1e9, 1),
        "device_copy_gbps": round(8.0 * n / (copy_ms * 1e-3) / 1e9, 1)}
    # configurations 1 and 2: cache-resident tensors and small products -- latency-bound, reported as times
    c1 = workloads.config1()
    x1 = torch.from_numpy(c1["x"]).to(dev)
    y1 = torch.empty_like(x1)
    A1, B1 = torch.from_numpy(c1["A"]).to(dev), torch.from_numpy(c1["B"]).to(dev)
    C1 = torch.empty((256, 256), dtype=torch.float32, device=dev)
    c2 = workloads.config2()
    X2 = torch.from_numpy(c2["X"]).to(dev)
    W2 = [torch.from_numpy(wl).to(dev) for wl in c2["W"]]
    acts = [X2] + [torch.rand((X2.shape[0], wl.shape[0]), device=dev) for wl in W2[:-1]]
    grads = [torch.randn((X2.shape[0], wl.shape[0]), device=dev) * 1e-3 for wl in W2]
    outs2 = [(torch.empty((a.shape[0], wl.shape[0]), device=dev), torch.empty_like(a), torch.empty_like(wl))
             for a, wl in zip(acts, W2)]

    def mlp_products():
        for a, wl, gl, (yo, dxo, dwo) in zip(acts, W2, grads, outs2):
            fmt.fmt_gemm(a, wl, f169, transB=True, out=yo)          # forward  (batch x in)(out x in)^T
            fmt.fmt_gemm(gl, wl, f169, out=dxo)                      # dgrad    (batch x out)(out x in)
            fmt.fmt_gemm(gl, a, f169, transA=True, out=dwo)          # wgrad    (batch x out)^T(batch x in)
    # the same nine products replayed from a HIP graph (the calls neither allocate nor synchronise once a
    # first call on the stream has grown the library's scratch, so they can be captured)
    gstream = torch.cuda.Stream()
    gstream.wait_stream(torch.cuda.current_stream())
    mlp_graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(gstream):
        mlp_products()
        gstream.synchronize()
        with torch.cuda.graph(mlp_graph, stream=gstream):
            mlp_products()
    torch.cuda.current_stream().wait_stream(gstream)
    torch.cuda.synchronize()
    result["small_configs"] = {
        "workload": "config 1 (2^20 elements, 256^3 product) and config 2 (MLP 784-1024-1024-10, batch 256: 9 products), "
                    "1/6/9/d; latency-bound, times per call",
        "config1_quantize_hist_us": round(timed(lambda: fmt.fmt_quantize(x1, f169, out=y1, hist=hists[0]), 50) * 1e3, 2),
        "config1_gemm_us": round(timed(lambda: fmt.fmt_gemm(A1, B1, f169, out=C1), 50) * 1e3, 2),
        "config2_products_us": round(timed(mlp_products, 20) * 1e3, 2),
        "config2_products_graph_replay_us": round(timed(mlp_graph.replay, 20) * 1e3, 2),
    }
    # FMAC-8 accumulation (Algorithm 1): a sequential chain of roundings per output, vector ALUs only
    A8 = torch.randn((2048, 1024), device=dev)
    B8 = torch.randn((1024, 2048), device=dev) * 0.05
    C8 = torch.empty((2048, 2048), device=dev)
    f8_ms = timed(lambda: fmt.fmt_gemm_fmac8(A8, B8, f169, out=C8), reps)
    result["fmac8"] = {"workload": "fmt_gemm_fmac8 2048x2048x1024, 1/6/9/d", "ms": round(f8_ms, 4),
                       "value": round(2048.0 * 2048 * 1024 / (f8_ms * 1e-3) / 1e12, 3), "unit": "T fused-MAC/s",
                       "roofline": {"bound": "alu", "unit": "T fused-MAC/s",
                                    "peak": round(VALU_LANE_INSTR_PER_S / FMAC8_INSTR_PER_MAC / 1e12, 3),
                                    "achieved": round(2048.0 * 2048 * 1024 / (f8_ms * 1e-3) / 1e12, 3),
                                    "frac": round(2048.0 * 2048 * 1024 / (f8_ms * 1e-3)
                                                  / (VALU_LANE_INSTR_PER_S / FMAC8_INSTR_PER_MAC), 4),
                                    "note": "vector issue rate 256 CUs x 64 lanes x 2.4 GHz = 39.3 T "
                                            "lane-instructions/s over the 12 instructions of the fused step "
                                            "of the single-precision path (16 are executed per step with the "
                                            "midpoint handling, operand rounding and master additions: "
                                            "profiles/fmac8_kernel_counters.md)"}}
    # loss-scale controller on the nine statistics records of configuration 4's gradient tensors
    recs = torch.stack([L["h"][2] for L in layers])
    st = fmt.fmt_dls_init(1024.0)
    result["dls_step_us"] = round(timed(lambda: fmt.fmt_dls_step(recs, st), 20) * 1e3, 2)

    if not args.no_cpu_baseline:
        import oracle
        sample = min(n, 1 << 26)
        xs = x_host[:sample]
        t1 = time.perf_counter()
        for (e, m, d) in variants:                        # the six passes of the timed stream section
            oracle.quantize(xs, e, m, d)
            oracle.histogram(xs, e, m)
        cpu_s = time.perf_counter() - t1
        result["cpu_baseline"] = {
            "value": round(len(variants) * 8.0 * sample / cpu_s / 1e9, 4),
            "unit": "GB/s",
            "cores": 1,
            "kind": "oracle",
            "sample": "quantize + histogram of the first 2^%d elements of the same tensor in the six format "
                      "variants (%d passes, %.1f s)" % (sample.bit_length() - 1, len(variants), cpu_s),
        }
        # the same oracle passes spread over all host cores (independent chunks of the sample, one thread each;
        # the oracle's loops are serial C and release the interpreter lock inside ctypes)
        import concurrent.futures
        cores = max(1, min(len(os.sched_getaffinity(0)), 16))
        chunks = np.array_split(xs, cores)

        def one_chunk(c):
            for (e, m, d) in variants:
                oracle.quantize(c, e, m, d)
                oracle.histogram(c, e, m)
        t1 = time.perf_counter()
        with concurrent.futures.ThreadPoolExecutor(cores) as ex:
            list(ex.map(one_chunk, chunks))
        par_s = time.perf_counter() - t1
        result["cpu_baseline"]["all_cores"] = {"value": round(len(variants) * 8.0 * sample / par_s / 1e9, 4),
                                               "unit": "GB/s", "cores": cores}
        # the GEMM oracle (fp64 triple loop, OpenMP over rows) on a bounded sample of config 4: the attention-output
        # layer's forward product (4096 x 1024 x 1024: a few tenths of a second on 16 cores)
        La = cfg4["layers"][1]
        Xs = np.ascontiguousarray(La["X"])
        t1 = time.perf_counter()
        oracle.gemm(Xs, La["W"], f169[0], f169[1], f169[2], transB=True)
        g_s = time.perf_counter() - t1
        result["cpu_baseline"]["gemm"] = {
            "value": round(2.0 * Xs.shape[0] * La["W"].shape[0] * La["W"].shape[1] / g_s / 1e12, 5), "unit": "TFLOP/s",
            "cores": int(os.environ.get("OMP_NUM_THREADS", cores)), "kind": "oracle",
            "sample": "oracle.gemm of config 4's attention-output forward product "
                      "(%d x 1024 x 1024, %.2f s)" % (Xs.shape[0], g_s)}

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
