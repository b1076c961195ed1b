#!/usr/bin/env python3
"""Benchmark of the NVFP4 quantized linear layer on one MI355X.

One "step" = forward + backward + update (Eqs. 4-6 of the paper) of the three linear layers of
a Llama2-7B SwiGLU MLP at 4096 tokens: every tensor-maximum pass, every row/column quantizer
(RtN forward, Philox SR backward) and all nine block-scaled GEMMs, through the C ABI.  Inputs are
synthetic (seeded Gaussians, gradient tensor with sparse outliers) and resident in HBM before
the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_F16_TFLOPS = 2500.0   # dense fp16/bf16 MFMA: the instruction the exact NVFP4 GEMM issues
PEAK_FP4_TFLOPS = 10100.0  # dense FP4 MFMA: the denominator the headline metric names


def event_time_ms(fn, iters, torch, warmup=2):
    """Average milliseconds per call of fn(i), measured with events on the stream fn launches on."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(iters):
        fn(i)
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--streams", type=int, default=1,
                    help="1: every call on one stream (the timed default); 2: gate and up side by side on two "
                         "streams as the MLP's dependency graph allows (timed next to it either way)")
    ap.add_argument("--probe", action="store_true",
                    help="run each kernel of interest a few times and exit (for rocprofv3 --pmc passes)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc runs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2505_19115_amd import binding as nv
    from paper_2505_19115_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    dev = "cuda"

    if args.probe:
        # a plain copy of known size (128 MiB in, 128 MiB out) calibrates the byte counters;
        # then the dominant GEMM and every quantizer kernel on the benchmark's tensors
        src = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        Xp, Wp = synth.normal(4096, 4096, 1.0, 100).to(dev), synth.normal(11008, 4096, 0.02, 200).to(dev)
        # operands in the slab layout, as the fused calls of the step hand them to the GEMM
        qa, qb = nv.quantize_dual(Xp, slab_rows=True)[0], nv.quantize_dual(Wp, slab_rows=True)[0]
        Yp = torch.empty((4096, 11008), dtype=torch.bfloat16, device=dev)
        for _ in range(10):
            nv.gemm(qa, qb, out=Yp, slabs=(True, True), shape=(4096, 11008, 4096))
        qam, qbm = nv.quantize_dual(Xp, fmt=nv.MXFP4, slab_rows=True)[0], nv.quantize_dual(Wp, fmt=nv.MXFP4, slab_rows=True)[0]
        for _ in range(10):
            nv.gemm(qam, qbm, nv.MXFP4, out=Yp, slabs=(True, True), shape=(4096, 11008, 4096))
        # the other two GEMM shapes of the step: dX of gate/up (4096 x 4096 x 11008) and dW of gate/up (11008 x 4096 x 4096)
        dYp = synth.gradient_like(4096, 11008, 300).to(dev)
        for fmt in (nv.NVFP4, nv.MXFP4):
            qd = nv.quantize_dual(dYp, nv.SR, 1, nv.SR, 2, fmt, slab_rows=True, slab_cols=True)
            qw = nv.quantize_dual(Wp, fmt=fmt, slab_cols=True)
            qx = nv.quantize_dual(Xp, nv.RTN, 0, nv.SR, 3, fmt, slab_cols=True)
            dXp = torch.empty((4096, 4096), dtype=torch.bfloat16, device=dev)
            dWp = torch.empty((11008, 4096), dtype=torch.bfloat16, device=dev)
            for _ in range(5):
                nv.gemm(qd[0], qw[1], fmt, out=dXp, slabs=(True, True), shape=(4096, 4096, 11008))
            for _ in range(5):
                nv.gemm(qd[1], qx[1], fmt, out=dWp, slabs=(True, True), shape=(11008, 4096, 4096))
            del qd, qw, qx
        xq = synth.student_t_outliers(8192, 8192, seed=100).to(dev)
        g = nv.tensor_scale(xq)
        for axis in (1, 0):
            for rnd in (nv.RTN, nv.SR):
                for _ in range(2):
                    nv.quantize(xq, axis, rnd, 1, tensor_scale=g)
        for rnd in (nv.RTN, nv.SR):
            for _ in range(2):
                nv.quantize_dual(xq, rnd, 1, rnd, 2, tensor_scale=g, slab_rows=True, slab_cols=True)
        # the dual passes of the step at their own shapes: X (RtN rows, SR columns), W (RtN, RtN), dY (SR, SR)
        for t, rr, rc in ((Xp, nv.RTN, nv.SR), (Wp, nv.RTN, nv.RTN), (dYp, nv.SR, nv.SR)):
            gt = nv.tensor_scale(t)
            for _ in range(2):
                nv.quantize_dual(t, rr, 1, rc, 2, tensor_scale=gt, slab_rows=True, slab_cols=True)
        torch.cuda.synchronize()
        print("probe done")
        return 0

    # ---- workload: the 7B SwiGLU MLP's three linears, tokens = 4096 (batch 2 x seq 2048)
    M = 4096
    layers = [("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
    data = []
    for idx, (name, N, K) in enumerate(layers):
        X = synth.normal(M, K, 1.0, 100 + idx).to(dev)
        W = synth.normal(N, K, 0.02, 200 + idx).to(dev)
        dY = synth.gradient_like(M, N, 300 + idx).to(dev)
        f = nv.NVFP4.c()
        wf = torch.empty(nv.lib.nvfp4_linear_fwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device=dev)
        wb = torch.empty(nv.lib.nvfp4_linear_bwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device=dev)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        dW = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
        saved = torch.empty(nv.linear_saved_bytes(M, N, K), dtype=torch.uint8, device=dev)
        data.append((name, N, K, X, W, dY, wf, wb, Y, dX, dW, saved))
    flop_per_step = sum(3 * 2 * M * N * K for _, N, K in layers)

    def fwd(layer, s, fmt, base):
        name, N, K, X, W, dY, wf, wb, Y, dX, dW, saved = layer
        # the forward call's passes over X and W also leave Q_SR(X^T), Q_RtN(W^T) and the per-tensor
        # scales for the backward call, which then reads only dY (once)
        nv.linear_fwd(X, W, fmt, workspace=wf, out=Y, saved=saved, bwd_seed=base + 3 * s)

    def bwd(layer, s, fmt, base):
        name, N, K, X, W, dY, wf, wb, Y, dX, dW, saved = layer
        nv.linear_bwd(dY, None, None, base + 3 * s, fmt, workspace=wb, out=(dX, dW), saved=saved, K=K)

    def step_serial(s, fmt=nv.NVFP4, base=1000):
        for layer in data:
            fwd(layer, s, fmt, base)
            bwd(layer, s, fmt, base)

    # The MLP's own dependency graph: gate and up read the same input and do not depend on each
    # other, down consumes both; backward runs the graph in reverse.  gate runs on the timing
    # stream, up on a second stream of default priority, forked and joined with events.
    side = torch.cuda.Stream()
    ev = [torch.cuda.Event() for _ in range(4)]

    def step_graph(s, fmt=nv.NVFP4, base=1000):
        gate, up, down = data
        main = torch.cuda.current_stream()
        ev[0].record(main)
        side.wait_event(ev[0])
        fwd(gate, s, fmt, base)
        with torch.cuda.stream(side):
            fwd(up, s, fmt, base)
            ev[1].record(side)
        main.wait_event(ev[1])
        fwd(down, s, fmt, base)
        bwd(down, s, fmt, base)
        ev[2].record(main)
        side.wait_event(ev[2])
        bwd(gate, s, fmt, base)
        with torch.cuda.stream(side):
            bwd(up, s, fmt, base)
            ev[3].record(side)
        main.wait_event(ev[3])

    step = step_graph if args.streams >= 2 else step_serial
    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(args.warmup + s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    tflops = flop_per_step / (elapsed / args.steps) / 1e12
    # the other schedule, for comparison
    other = step_serial if args.streams >= 2 else step_graph
    other_ms = event_time_ms(other, max(args.steps // 2, 3), torch)
    schedules = {"timed": "mlp_graph_2_streams" if args.streams >= 2 else "one_stream",
                 "one_stream_ms" if args.streams >= 2 else "mlp_graph_2_streams_ms": round(other_ms, 3)}

    # ---- the same step composed from the single entry points (tensor-maximum pass + dual quantizer through
    # nvfp4_quantize_dual with slab outputs, GEMMs through nvfp4_gemm_slab): exactly the kernels of the fused
    # calls, in their order, with an event pair around every GEMM, so that the three GEMM shapes are timed
    # INSIDE the step (the clock a GEMM sees depends on what ran just before it) and the parts can be added up
    def composed(fmt):
        parts = []
        for name, N, K, X, W, dY, wf, wb, Y, dX, dW, saved in data:
            takes = lambda m, n, k: bool(nv.lib.nvfp4_gemm_takes_slabs(m, n, k, C.byref(fmt.c())))
            s_fwd, s_dx, s_dw = takes(M, N, K), takes(M, K, N), takes(N, K, M)
            qx = nv.quantize_dual(X, nv.RTN, 0, nv.SR, 1002, fmt, slab_rows=s_fwd, slab_cols=s_dw)
            qw = nv.quantize_dual(W, nv.RTN, 0, nv.RTN, 0, fmt, slab_rows=s_fwd, slab_cols=s_dx)
            qd = nv.quantize_dual(dY, nv.SR, 1000, nv.SR, 1001, fmt, slab_rows=s_dx, slab_cols=s_dw)
            ts = [torch.cat([a[2], b[2]]) for a, b in ((qx[0], qw[0]), (qd[0], qw[1]), (qd[1], qx[1]))]
            flat = lambda q: (q[0][0], q[0][1], q[1][0], q[1][1], torch.empty(1, dtype=torch.float32, device=dev))
            parts.append(dict(N=N, K=K, X=X, W=W, dY=dY, Y=Y, dX=dX, dW=dW, qx=qx, qw=qw, qd=qd, ts=ts,
                              ox=flat(qx), ow=flat(qw), od=flat(qd), s=(s_fwd, s_dx, s_dw)))
        return parts

    def step_composed(parts, fmt, events=None):
        def gemm(mnk, *a, **k):
            if events is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            nv.gemm(*a, shape=mnk, **k)
            if events is not None:
                e1.record()
                events.append((mnk, e0, e1))
        for p in parts:
            N, K, (s_fwd, s_dx, s_dw) = p["N"], p["K"], p["s"]
            nv.quantize_dual(p["X"], nv.RTN, 0, nv.SR, 1002, fmt, out=p["ox"], slab_rows=s_fwd, slab_cols=s_dw)
            nv.quantize_dual(p["W"], nv.RTN, 0, nv.RTN, 0, fmt, out=p["ow"], slab_rows=s_fwd, slab_cols=s_dx)
            gemm((M, N, K), p["qx"][0], p["qw"][0], fmt, out=p["Y"], slabs=(s_fwd, s_fwd), tensor_scales=p["ts"][0])
            nv.quantize_dual(p["dY"], nv.SR, 1000, nv.SR, 1001, fmt, out=p["od"], slab_rows=s_dx, slab_cols=s_dw)
            gemm((M, K, N), p["qd"][0], p["qw"][1], fmt, out=p["dX"], slabs=(s_dx, s_dx), tensor_scales=p["ts"][1])
            gemm((N, K, M), p["qd"][1], p["qx"][1], fmt, out=p["dW"], slabs=(s_dw, s_dw), tensor_scales=p["ts"][2])

    def in_step_gemm_times(fmt, peak):
        parts = composed(fmt)
        n_it = max(args.steps // 2, 3)
        plain_ms = event_time_ms(lambda i: step_composed(parts, fmt), n_it, torch)
        events = []
        for i in range(2):
            step_composed(parts, fmt)
        torch.cuda.synchronize()
        for i in range(n_it):
            step_composed(parts, fmt, events)
        torch.cuda.synchronize()
        per = {}
        for shape, e0, e1 in events:
            per.setdefault(shape, []).append(e0.elapsed_time(e1))
        out, total = {}, 0.0
        for shape, v in per.items():
            ms = sum(v) / len(v)
            calls = len(v) // n_it
            total += ms * calls
            fl = 2.0 * shape[0] * shape[1] * shape[2]
            out["x".join(map(str, shape))] = {"calls_per_step": calls, "avg_ms": round(ms, 4), "min_ms": round(min(v), 4),
                                              "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1), "frac_of_peak": round(fl / (ms * 1e-3) / 1e12 / peak, 4)}
        out["gemm_ms_per_step"] = round(total, 3)
        out["composed_step_ms"] = round(plain_ms, 3)
        out["other_kernels_ms_per_step"] = round(plain_ms - total, 3)
        out["how"] = ("the step composed from nvfp4_quantize_dual (maximum pass + dual quantizer, slab outputs) and nvfp4_gemm_slab: the same "
                      "kernels in the same order as the fused calls; event pair around each GEMM; M x N x K of the GEMM (contraction last)")
        return out

    in_step = in_step_gemm_times(nv.NVFP4, PEAK_F16_TFLOPS)
    in_step_mx = in_step_gemm_times(nv.MXFP4, PEAK_FP4_TFLOPS)

    # the same step in MXFP4 (block 32, E8M0; the GEMMs then run on the FP4 matrix instruction)
    def step_mx(s):
        step(s, nv.MXFP4, 2000)

    mx_step_ms = event_time_ms(step_mx, max(args.steps // 2, 3), torch)
    mx_step = {"ms_per_step": round(mx_step_ms, 3), "TFLOP/s": round(flop_per_step / (mx_step_ms * 1e-3) / 1e12, 1),
               "frac_of_fp4_peak": round(flop_per_step / (mx_step_ms * 1e-3) / 1e12 / PEAK_FP4_TFLOPS, 4)}

    # ---- the step of a later micro-batch of the same optimizer step: W's operands (Eqs. 4-5) were quantized once
    # by nvfp4_quantize_weight and are reused, so no pass over W is made (reported beside the headline, which
    # quantizes W in every step)
    def weights_reused(fmt, base):
        wqs = [nv.quantize_weight(layer[4], M, fmt) for layer in data]
        t_q = event_time_ms(lambda i: [nv.quantize_weight(layer[4], M, fmt, out=wq) for layer, wq in zip(data, wqs)], 5, torch)

        def step_wq(s):
            for (name, N, K, X, W, dY, wf, wb, Y, dX, dW, saved), wq in zip(data, wqs):
                nv.linear_fwd(X, None, fmt, workspace=wf, out=Y, saved=saved, bwd_seed=base + 3 * s, w_operands=wq, N=N)
                nv.linear_bwd(dY, None, None, base + 3 * s, fmt, workspace=wb, out=(dX, dW), saved=saved, K=K, w_operands=wq)

        ms = event_time_ms(step_wq, max(args.steps // 2, 3), torch)
        return {"ms_per_step": round(ms, 3), "TFLOP/s": round(flop_per_step / (ms * 1e-3) / 1e12, 1),
                "frac_of_fp4_peak": round(flop_per_step / (ms * 1e-3) / 1e12 / PEAK_FP4_TFLOPS, 4),
                "quantize_weights_once_ms": round(t_q, 3)}

    reuse = {"nvfp4": weights_reused(nv.NVFP4, 3000), "mxfp4": weights_reused(nv.MXFP4, 4000),
             "what": "nvfp4_linear_fwd_wq / nvfp4_linear_bwd_wq on operands of W written once by nvfp4_quantize_weight (3 tensor-maximum "
                     "passes and 3 dual passes over W, timed separately): per step 9 GEMMs + 6 dual passes + 6 maximum passes"}

    # ---- dominant kernel: the block-scaled GEMM at the gate/up shape (same launch as in step)
    name, N, K, X, W, dY, wf, wb, Y, dX, dW, _ = data[0]
    # operands in the slab layout, which is how the fused calls of the step hand them to this kernel; the same
    # launch on row-major operands (what nvfp4_gemm takes) is timed beside it
    # (the two are timed in alternating batches: the clock under a run of GEMMs depends on what ran just before)
    qa, qb = nv.quantize_dual(X, slab_rows=True)[0], nv.quantize_dual(W, slab_rows=True)[0]
    pa, pb = nv.quantize(X, 1), nv.quantize(W, 1)
    batches = [], []
    for _ in range(3):
        batches[0].append(event_time_ms(lambda i: nv.gemm(qa, qb, out=Y, slabs=(True, True), shape=(M, N, K)), max(args.steps, 5), torch))
        batches[1].append(event_time_ms(lambda i: nv.gemm(pa, pb, out=Y), max(args.steps, 5), torch))
    gemm_ms, gemm_plain_ms = sum(batches[0]) / 3, sum(batches[1]) / 3
    gemm_tflops = 2.0 * M * N * K / (gemm_ms * 1e-3) / 1e12
    del pa, pb
    traffic = mx_traffic = None
    if os.path.exists(args.traffic_json):
        try:
            tj = json.load(open(args.traffic_json))
            traffic, mx_traffic = tj.get("gemm_step_avg_bytes_per_launch"), tj.get("mxfp4_gemm_step_avg_bytes_per_launch")
        except Exception:
            traffic = mx_traffic = None
    # sustained rate of the two matrix instructions from a register-only loop (power-managed clock;
    # depends on operand bit activity): the practical ceiling next to the published peak
    sustained = {
        "f16_random_operands": round(nv.probe_mfma_rate(nv.MFMA_F16, True), 1),
        "f16_zero_operands": round(nv.probe_mfma_rate(nv.MFMA_F16, False), 1),
        "fp4_random_operands": round(nv.probe_mfma_rate(nv.MFMA_FP4, True), 1),
        "fp4_zero_operands": round(nv.probe_mfma_rate(nv.MFMA_FP4, False), 1),
        "unit": "TFLOP/s", "how": "nvfp4_probe_mfma_rate: registers only, one workgroup per CU",
    }
    # The dominant kernel's launches as the step makes them: 9 per step in three shapes, timed with event pairs inside
    # the step (in_step_gemms); achieved = the step's GEMM FLOPs / their summed durations, i.e. the average launch.
    step_gemm_ms = in_step["gemm_ms_per_step"]
    step_gemm_tflops = flop_per_step / (step_gemm_ms * 1e-3) / 1e12
    roofline = {"kernel": "gemm_nt_f16_kernel: the 9 GEMM launches of the step (4 x 4096x11008x4096, 3 x 4096x4096x11008, 2 x 11008x4096x4096)",
                "bound": "mfma", "achieved": round(step_gemm_tflops, 2), "peak": PEAK_F16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(step_gemm_tflops / PEAK_F16_TFLOPS, 4),
                "frac_of_fp4_peak": round(step_gemm_tflops / PEAK_FP4_TFLOPS, 4),
                "frac_of_sustained_f16": round(step_gemm_tflops / max(sustained["f16_random_operands"], 1e-9), 4),
                "avg_launch_ms": round(step_gemm_ms / 9, 4), "traffic": traffic,
                "how": "event pairs around each GEMM inside the composed step (see in_step_gemms); 369.4 GFLOP per launch",
                "isolated_gate_launches": {"avg_launch_ms": round(gemm_ms, 4), "TFLOP/s": round(gemm_tflops, 2),
                                           "avg_launch_ms_row_major_operands": round(gemm_plain_ms, 4),
                                           "note": "the gate-shape launch repeated back to back, outside the step: a run of GEMMs alone heats the chip and runs slower than the same launch between the step's memory-bound kernels"}}

    # ---- MXFP4 (block 32, E8M0): the same GEMM on the FP4 matrix instruction, and the format sweep
    # of the paper's Table 1 / Fig. 1 axes on the down-projection shape (forward linear, bf16 in/out)
    qam, qbm = nv.quantize_dual(X, fmt=nv.MXFP4, slab_rows=True)[0], nv.quantize_dual(W, fmt=nv.MXFP4, slab_rows=True)[0]
    mx_ms = event_time_ms(lambda i: nv.gemm(qam, qbm, nv.MXFP4, out=Y, slabs=(True, True), shape=(M, N, K)), max(args.steps, 5), torch)
    mx_tflops = 2.0 * M * N * K / (mx_ms * 1e-3) / 1e12
    mx_step_gemm_ms = in_step_mx["gemm_ms_per_step"]
    mx_step_tflops = flop_per_step / (mx_step_gemm_ms * 1e-3) / 1e12
    mxfp4 = {"kernel": "gemm_nt_mxfp4_dma_kernel: the 9 GEMM launches of the MXFP4 step (same three shapes)", "bound": "mfma",
             "achieved": round(mx_step_tflops, 2), "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s",
             "frac": round(mx_step_tflops / PEAK_FP4_TFLOPS, 4),
             "frac_of_sustained_fp4": round(mx_step_tflops / max(sustained["fp4_random_operands"], 1e-9), 4),
             "avg_launch_ms": round(mx_step_gemm_ms / 9, 4), "traffic": mx_traffic,
             "isolated_gate_launches": {"avg_launch_ms": round(mx_ms, 4), "TFLOP/s": round(mx_tflops, 2)}}
    del qam, qbm
    # Format / block-size sweep (Table 1, Figs. 1-2 axes) on the down projection at 8192 tokens: forward
    # (RtN) + backward (SR) of the linear layer per format, and the relative quantization MSE of the
    # activation (RtN) and of the upstream gradient (SR) from the on-GPU noise statistics.
    sM, sN, sK = 8192, 4096, 11008
    sX, sW = synth.normal(sM, sK, 1.0, 500).to(dev), synth.normal(sN, sK, 0.02, 501).to(dev)
    sdY = synth.gradient_like(sM, sN, 502).to(dev)
    sY = torch.empty((sM, sN), dtype=torch.bfloat16, device=dev)
    sdX, sdW = torch.empty((sM, sK), dtype=torch.bfloat16, device=dev), torch.empty((sN, sK), dtype=torch.bfloat16, device=dev)
    sweep = {}
    for label, fmt in (("nvfp4_b16_e4m3", nv.NVFP4), ("mxfp4_b32_e8m0", nv.MXFP4),
                       ("b32_e4m3", nv.Format(32, nv.SCALE_E4M3, 1)), ("b64_e4m3", nv.Format(64, nv.SCALE_E4M3, 1)),
                       ("b128_e4m3", nv.Format(128, nv.SCALE_E4M3, 1))):
        f = fmt.c()
        wf = torch.empty(nv.lib.nvfp4_linear_fwd_workspace_bytes(sM, sN, sK, C.byref(f)), dtype=torch.uint8, device=dev)
        wb = torch.empty(nv.lib.nvfp4_linear_bwd_workspace_bytes(sM, sN, sK, C.byref(f)), dtype=torch.uint8, device=dev)
        ssaved = torch.empty(nv.linear_saved_bytes(sM, sN, sK, fmt), dtype=torch.uint8, device=dev)

        def fwd_bwd(i):
            nv.linear_fwd(sX, sW, fmt, workspace=wf, out=sY, saved=ssaved, bwd_seed=7000 + 3 * i)
            nv.linear_bwd(sdY, None, None, 7000 + 3 * i, fmt, workspace=wb, out=(sdX, sdW), saved=ssaved, K=sK)

        ms = event_time_ms(fwd_bwd, 4, torch)
        ms_fp4 = None
        if fmt.block >= 64:
            # the other exact route for these formats (unit-scale FP4 MFMA per block + binary32 rescale), for comparison
            before = nv.cross_check_switches(nv.SWITCH_FP4_WIDE_BLOCKS)
            ms_fp4 = event_time_ms(fwd_bwd, 4, torch)
            nv.cross_check_switches(before)
        nx = nv.quant_noise(sX, nv.quantize(sX, 1, nv.RTN, 0, fmt), 1, fmt).cpu().numpy()
        ng = nv.quant_noise(sdY, nv.quantize(sdY, 1, nv.SR, 9, fmt), 1, fmt).cpu().numpy()
        sweep[label] = {"fwd_bwd_ms": round(ms, 4), "TFLOP/s": round(3 * 2.0 * sM * sN * sK / (ms * 1e-3) / 1e12, 1),
                        "rel_mse_activation_rtn": float(f"{nx[1] / nx[0]:.4e}"),
                        "rel_mse_gradient_sr": float(f"{ng[1] / ng[0]:.4e}"),
                        "gradient_to_noise_ratio": round(float((ng[0] / ng[1]) ** 0.5), 3)}
        if ms_fp4 is not None:
            sweep[label]["gemm_route"] = "operands expanded to fp16 (as NVFP4)"
            sweep[label]["fwd_bwd_ms_fp4_mfma_rescale_route"] = round(ms_fp4, 4)
        del wf, wb
    sweep["workload"] = (f"linear fwd (RtN) + bwd (SR), down projection at 8192 tokens: M={sM} N={sN} K={sK}, bf16 in/out; "
                         "rel_mse = sum (Q(x)-x)^2 / sum x^2; ratio = ||dY|| / (sigma_q sqrt(d)), threshold sqrt(3)")
    del sX, sW, sdY, sY, sdX, sdW

    # ---- the five forward linears of the 7B block at 4096 tokens (RtN, bf16 in and out), and the single small
    # fp32 forward linear: secondary rows, same entry point (nvfp4_linear_fwd), nothing saved for a backward pass
    fwd_layers = []
    for idx, (lname, N, K) in enumerate(synth.LLAMA2_7B_LINEARS):
        Xl, Wl = synth.normal(M, K, 1.0, 600 + idx).to(dev), synth.normal(N, K, 0.02, 700 + idx).to(dev)
        f = nv.NVFP4.c()
        wsl = torch.empty(nv.lib.nvfp4_linear_fwd_workspace_bytes(M, N, K, C.byref(f)), dtype=torch.uint8, device=dev)
        fwd_layers.append((lname, N, K, Xl, Wl, wsl, torch.empty((M, N), dtype=torch.bfloat16, device=dev)))
    fwd_flop = sum(2.0 * M * N * K for _, N, K, *_ in fwd_layers)
    forward_linears = {}
    for label, fmt in (("nvfp4", nv.NVFP4), ("mxfp4", nv.MXFP4)):
        def fwd_all(i):
            for lname, N, K, Xl, Wl, wsl, Yl in fwd_layers:
                nv.linear_fwd(Xl, Wl, fmt, workspace=wsl, out=Yl)
        ms = event_time_ms(fwd_all, max(args.steps, 5), torch)
        tf = fwd_flop / (ms * 1e-3) / 1e12
        forward_linears[label] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_of_fp4_peak": round(tf / PEAK_FP4_TFLOPS, 4),
                                  "frac_of_f16_peak": round(tf / PEAK_F16_TFLOPS, 4)}
    forward_linears["workload"] = (f"QKV 4096->12288, out-proj 4096->4096, gate and up 4096->11008, down 11008->4096 at {M} tokens: "
                                   f"{fwd_flop / 1e9:.1f} GFLOP; per linear two tensor-maximum passes, two row quantizers (RtN), one GEMM")
    del fwd_layers
    X1, W1 = synth.normal(256, 256, 1.0, 1, torch.float32).to(dev), synth.normal(256, 256, 1.0, 2, torch.float32).to(dev)
    f = nv.NVFP4.c()
    ws1 = torch.empty(nv.lib.nvfp4_linear_fwd_workspace_bytes(256, 256, 256, C.byref(f)), dtype=torch.uint8, device=dev)
    Y1 = torch.empty((256, 256), dtype=torch.float32, device=dev)
    ms1 = event_time_ms(lambda i: nv.linear_fwd(X1, W1, workspace=ws1, out=Y1), 200, torch, warmup=10)
    small_forward = {"workload": "single NVFP4 linear forward, X and W fp32 [256 x 256], fp32 out: 5 kernel launches", "us_per_call": round(ms1 * 1e3, 2),
                     "GFLOP/s": round(2.0 * 256 ** 3 / (ms1 * 1e-3) / 1e9, 1)}

    # ---- SwiGLU backward + the quantizers of dG and dU at the 7B shape [4096 x 11008]: fused (maxima pass + one
    # dual pass per result, nothing stored) against the same step unfused (elementwise kernel storing dG, dU in
    # bf16, then a maximum pass and a dual pass over each)
    Fw = 11008
    dHs, Gs, Us = synth.gradient_like(M, Fw, 800).to(dev), synth.normal(M, Fw, 2.0, 801).to(dev), synth.normal(M, Fw, 1.0, 802).to(dev)
    fo = (nv.empty_dual_operands(M, Fw, nv.NVFP4, True, True), nv.empty_dual_operands(M, Fw, nv.NVFP4, True, True))
    t_fused = event_time_ms(lambda i: nv.swiglu_bwd_quantize(dHs, Gs, Us, 10 + i, 20 + i, out=fo), 10, torch)
    tG, tU = torch.empty_like(dHs), torch.empty_like(dHs)
    t_stored = event_time_ms(lambda i: nv.swiglu_bwd_quantize(dHs, Gs, Us, 10 + i, 20 + i, out=fo, store=(tG, tU)), 10, torch)
    flat = lambda o: (o.codes_rows, o.scales_rows, o.codes_cols, o.scales_cols, o.g)

    def unfused(i):
        nv.swiglu_bwd(dHs, Gs, Us, out=(tG, tU))
        nv.quantize_dual(tG, nv.SR, 10 + i, nv.SR, 11 + i, out=flat(fo[0]), slab_rows=True, slab_cols=True)
        nv.quantize_dual(tU, nv.SR, 20 + i, nv.SR, 21 + i, out=flat(fo[1]), slab_rows=True, slab_cols=True)

    t_unfused = event_time_ms(unfused, 10, torch)
    swiglu = {"fused_results_stored_ms": round(t_stored, 4), "fused_nothing_stored_ms": round(t_fused, 4), "unfused_ms": round(t_unfused, 4),
              "workload": f"dH, G, U bf16 [{M} x {Fw}] -> Q_SR(dG), Q_SR(dU), both orientations, slab layout (NVFP4)",
              "fused_results_stored": "nvfp4_swiglu_bwd_quantize with dG_store/dU_store: 1 pass evaluates, stores and leaves the maxima + 2 dual passes over the stored results",
              "fused_nothing_stored": "nvfp4_swiglu_bwd_quantize: 1 maxima pass + 2 dual passes that evaluate the result again while loading",
              "unfused": "nvfp4_swiglu_bwd (stores dG, dU) + 2 x nvfp4_quantize_dual (maximum pass + dual pass each)"}
    del dHs, Gs, Us, tG, tU, fo

    # ---- quantizer sweep tensor (second half of the metric): bf16 [8192, 8192].
    # Four different tensors are cycled (512 MiB in total) so that the 256 MB last-level cache
    # cannot serve the reads of the next call: the rate is an HBM rate.
    NQ = 4
    xqs = [synth.student_t_outliers(8192, 8192, seed=100 + i).to(dev) for i in range(NQ)]
    gs = [nv.tensor_scale(x) for x in xqs]
    nel = xqs[0].numel()
    quant = {}
    for label, axis, rnd in (("rows_rtn", 1, nv.RTN), ("rows_sr", 1, nv.SR), ("cols_rtn", 0, nv.RTN), ("cols_sr", 0, nv.SR)):
        outs = [nv.quantize(xqs[i], axis, rnd, 1, tensor_scale=gs[i]) for i in range(NQ)]
        ms = event_time_ms(lambda i: nv.quantize(xqs[i % NQ], axis, rnd, 1, tensor_scale=gs[i % NQ], out=outs[i % NQ]),
                           12, torch, warmup=NQ)
        gbs = nel * 2.5625 / (ms * 1e-3) / 1e9
        quant[label] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
    # both orientations in one pass (what the fused forward / backward calls run): 2 + 2 x 0.5625 B/elt
    # (row-major outputs, and the slab layout the fused calls use between quantizer and GEMM)
    for label, rr, rc, slab in (("dual_rtn_rtn", nv.RTN, nv.RTN, False), ("dual_rtn_sr", nv.RTN, nv.SR, False),
                                ("dual_sr_sr", nv.SR, nv.SR, False), ("dual_rtn_rtn_slabs", nv.RTN, nv.RTN, True),
                                ("dual_rtn_sr_slabs", nv.RTN, nv.SR, True), ("dual_sr_sr_slabs", nv.SR, nv.SR, True)):
        douts = [nv.quantize_dual(xqs[i], rr, 1, rc, 2, tensor_scale=gs[i], slab_rows=slab, slab_cols=slab) for i in range(NQ)]
        douts = [(a[0], a[1], b[0], b[1], a[2]) for a, b in douts]
        ms = event_time_ms(lambda i: nv.quantize_dual(xqs[i % NQ], rr, 1, rc, 2, tensor_scale=gs[i % NQ], out=douts[i % NQ],
                                                      slab_rows=slab, slab_cols=slab), 12, torch, warmup=NQ)
        gbs = nel * 3.125 / (ms * 1e-3) / 1e9
        quant[label] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
    del douts
    outs = [nv.quantize(xqs[i], 1, nv.RTN, 0) for i in range(NQ)]
    ms = event_time_ms(lambda i: nv.quantize(xqs[i % NQ], 1, nv.RTN, 0, out=outs[i % NQ]), 12, torch, warmup=NQ)
    gbs = nel * 4.5625 / (ms * 1e-3) / 1e9
    quant["rows_rtn_with_amax_pass"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
    for label, axis in (("noise_stats_rows", 1), ("noise_stats_cols", 0)):
        qs = [nv.quantize(xqs[i], axis, nv.SR, 1, tensor_scale=gs[i]) for i in range(NQ)]
        acc = torch.empty(2, dtype=torch.float64, device=dev)
        nws = torch.empty(nv.lib.nvfp4_quant_noise_workspace_bytes(8192, 8192, axis), dtype=torch.uint8, device=dev)
        ms = event_time_ms(lambda i: nv.quant_noise(xqs[i % NQ], qs[i % NQ], axis, out=acc, workspace=nws), 12, torch, warmup=NQ)
        gbs = nel * 2.5625 / (ms * 1e-3) / 1e9
        quant[label] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
        del qs
    quant["bytes_per_element"] = {"preset_scale": 2.5625, "with_amax_pass": 4.5625, "dual": 3.125, "noise_stats": 2.5625}
    del xqs, outs

    # ---- the oracle on the host cores, bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        Ms, Ns, Ks = 4096, 11008, 4096  # the gate layer of the timed step, whole: about 20 s of host work
        Xs, Ws, dYs = synth.normal(Ms, Ks, 1.0, 1), synth.normal(Ns, Ks, 0.02, 2), synth.gradient_like(Ms, Ns, 3)
        t0 = time.perf_counter()
        oracle.linear_fwd(Xs, Ws)
        oracle.linear_bwd(dYs, Xs, Ws, 5)
        dt = time.perf_counter() - t0
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cores = min(cores, os.cpu_count() or cores)
        cpu = {"value": round(3 * 2 * Ms * Ns * Ks / dt / 1e12, 6), "unit": "TFLOP/s", "cores": cores,
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": f"one linear fwd+bwd (Eqs. 4-6), M={Ms} N={Ns} K={Ks}, NVFP4: 6 quantize calls + 3 fp64 GEMMs"}

    line = {
        "metric": "NVFP4 linear fwd+bwd TFLOP/s (% FP4 MFMA peak); quantize GB/s (% HBM peak)",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "e2m1 codes x e4m3 scales, expanded exactly to f16 for MFMA, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "Llama2-7B SwiGLU MLP linears fwd+bwd (gate, up, down), tokens=4096: "
                               "9 GEMMs + 9 dual-orientation quantize passes (X, W in the forward call, which saves Q_SR(X^T), Q_RtN(W^T) and the scales for the backward call; dY in the backward call) + 9 tensor-maximum passes per step, bf16 in and out; packed operands pass from the quantizers to the GEMMs in the library's slab layout",
                   "M": M, "layers": [[n, N, K] for n, N, K in layers], "format": "NVFP4 (block 16, E4M3, tensor scale)",
                   "rounding": "fwd RtN; bwd/update SR (Philox4x32-10)",
                   "not_included": "the elementwise SwiGLU between the linears (three independent linear layers with synthetic inputs each)",
                   "schedule": ("all forward calls, then all backward calls, in the MLP's dependency order; gate and up side by side "
                                "on two HIP streams (fork/join with events), down after both" if args.streams >= 2 else
                                "fwd then bwd per layer, every call on one stream")},
        "schedules": schedules,
        "frac_of_fp4_peak": round(tflops / PEAK_FP4_TFLOPS, 4),
        "roofline": roofline, "in_step_gemms": in_step, "mfma_sustained": sustained, "mxfp4_gemm": mxfp4, "mxfp4_step": mx_step,
        "mxfp4_in_step_gemms": in_step_mx, "weights_reused_step": reuse, "forward_linears_7b": forward_linears, "small_forward": small_forward, "swiglu_bwd_quantize": swiglu, "format_sweep": sweep,
        "quantize": quant, "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
