#!/usr/bin/env python3
"""Benchmark of the dynamically scaled float8 linear layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
fp8_linear_fwd (quantize X, W; Y = X W^T) followed by fp8_linear_bwd
(re-quantize dY, W, X along the contraction axes; dX = dY W, dW = dY^T X), all
inputs resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is the step's throughput in TFLOP/s (6 M N K
flop per step, quantization time included).  `roofline` describes the dominant
kernel (the forward scaled GEMM) from HIP-event timing of that kernel alone;
`kernels` lists every kernel of the path with its own roofline figure;
`cpu_baseline` is the CPU oracle timed on a bounded sample of the workload.
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

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
FP8_PEAK_TFLOPS = 5000.0    # MI355X dense FP8 MFMA
BF16_PEAK_TFLOPS = 2500.0


def _event_time_ms(fn, iters: int, warmup: int, torch) -> float:
    """Average duration of fn() in ms from HIP events on the current stream
    (the stream the library launches on)."""
    for _ in range(warmup):
        fn()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def _graph_time_ms(fn, iters: int, torch) -> float:
    """The same step replayed from a HIP graph: the launches are submitted by the
    runtime in one go, so the host's per-call cost (which dominates small shapes)
    is out of the measurement.  Captured after an eager warm-up on a side stream."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    for _ in range(2):
        g.replay()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        g.replay()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def _profiled_traffic(workload: str):
    """HBM bytes per launch of the forward GEMM as measured with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size); kept as a
    figure in profiles/ because counters cannot be read from inside this script."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith("gemm_fwd_traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def _sweep(torch, fp8, dev, iters: int) -> dict:
    """When is the fp8 linear faster than bf16 (Section 2.1 and the appendix on
    microbenchmarks)?  Forward + backward of one linear layer, dynamic
    quantization included, against the same three products in bf16 by the
    vendor BLAS, over a grid of forward shapes.  Linear layer only (no
    normalisation / activation around it)."""
    rows = []
    sizes = (1024, 2048, 4096, 8192, 16384)
    for M in (1024, 2048, 4096, 16384):
        for K in sizes:
            for N in sizes:
                x = torch.randn((M, K), device=dev).to(torch.bfloat16)
                w = (torch.randn((N, K), device=dev) * 0.02).to(torch.bfloat16)
                dy = (torch.randn((M, N), device=dev) * 1e-3).to(torch.bfloat16)
                y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
                dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
                dw = torch.empty((N, K), dtype=torch.bfloat16, device=dev)

                def bf16_step():
                    torch.matmul(x, w.t(), out=y)
                    torch.matmul(dy, w, out=dx)
                    torch.matmul(dy.t(), x, out=dw)
                entry = {"M": M, "K": K, "N": N, "bf16_ms": round(_event_time_ms(bf16_step, iters, 2, torch), 4),
                         "bf16_graph_ms": round(_graph_time_ms(bf16_step, iters, torch), 4)}
                # forward and backward share one workspace (FP8_SAVE_FOR_BWD): the forward also makes the fp8
                # copies of X and W that the backward needs (tensorwise: 3 quantizations per step instead of 5)
                for tag, gran in (("rowwise", fp8.FP8_ROW), ("tensorwise", fp8.FP8_TENSOR)):
                    r = fp8.Recipe(gran=gran, flags=fp8.FP8_SAVE_FOR_BWD)
                    wf = wb = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, True), dtype=torch.uint8, device=dev)

                    def fp8_step():
                        fp8.fp8_linear_fwd(x, w, r, y=y, workspace=wf)
                        fp8.fp8_linear_bwd(dy, (M, K), (N, K), r, dx=dx, dw=dw, workspace=wb)
                    ms = _event_time_ms(fp8_step, iters, 2, torch)
                    entry[f"fp8_{tag}_ms"] = round(ms, 4)
                    entry[f"speedup_{tag}"] = round(entry["bf16_ms"] / ms, 3)
                    entry[f"fp8_{tag}_TFLOP/s"] = round(6.0 * M * N * K / (ms * 1e-3) / 1e12, 1)
                    gms = _graph_time_ms(fp8_step, iters, torch)
                    entry[f"fp8_{tag}_graph_ms"] = round(gms, 4)
                    entry[f"speedup_{tag}_graph"] = round(entry["bf16_graph_ms"] / gms, 3)
                # rowwise with the weight gradient from the unquantized tensors on the bf16 matrix cores
                # (Appendix A, rowwise_gw_hp): where does it beat plain rowwise on this chip?
                r = fp8.Recipe(gran=fp8.FP8_ROW, flags=fp8.FP8_SAVE_FOR_BWD | fp8.FP8_GRAD_WEIGHT_HP)
                wh = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, True), dtype=torch.uint8, device=dev)

                def gw_hp_step():
                    fp8.fp8_linear_fwd(x, w, r, y=y, workspace=wh)
                    fp8.fp8_linear_bwd(dy, x, (N, K), r, dx=dx, dw=dw, workspace=wh)
                ms = _event_time_ms(gw_hp_step, iters, 2, torch)
                entry["fp8_rowwise_gw_hp_ms"] = round(ms, 4)
                entry["speedup_rowwise_gw_hp"] = round(entry["bf16_ms"] / ms, 3)
                entry["gw_hp_vs_rowwise"] = round(entry["fp8_rowwise_ms"] / ms, 3)   # > 1: the bf16 weight gradient is the faster choice
                rows.append(entry)
                del x, w, dy, y, dx, dw
    return {"sweep": "fp8 linear fwd+bwd (quantization included) vs bf16 torch.matmul x3, one MI355X; *_graph_ms: the same step "
                     "replayed from a HIP graph (no per-call host cost)",
            "iters": iters, "rows": rows}


def _block(torch, fp8, dev, iters: int) -> dict:
    """The paper's microbenchmark block (appendix "Float8 Training Microbenchmarks"):
    LayerNorm -> Linear -> Sigmoid, forward and backward, float8 (rowwise) against
    bfloat16.  Three variants of the same computation:
      bf16:       framework LayerNorm, vendor-BLAS matmuls, framework sigmoid;
      fp8:        the same framework ops around fp8_linear_fwd / fp8_linear_bwd;
      fp8_fused:  the forward's casts fused by hand where the paper relies on the compiler:
                  fp8_layernorm_quantize (normalisation + cast of the activations) and the
                  sigmoid inside the GEMM's epilogue; backward as in `fp8`;
      fp8_fused_fwd_bwd: additionally the gradient through the sigmoid formed inside the
                  backward's quantization passes (fp8_linear_bwd_sigmoid).
    The backward of the normalisation is a framework op in all four."""
    E4, ROW = fp8.FP8_E4M3FN, fp8.FP8_ROW
    F = torch.nn.functional
    rows = []
    shapes = [(M, K, N) for M in (4096, 16384) for K in (2048, 4096, 8192) for N in (2048, 4096, 8192)]
    shapes.append((16384, 4096, 14336))
    r = fp8.Recipe(gran=ROW)
    for M, K, N in shapes:
        x = torch.randn((M, K), device=dev).to(torch.bfloat16)
        w = (torch.randn((N, K), device=dev) * 0.02).to(torch.bfloat16)
        g = (torch.rand(K, device=dev) + 0.5).to(torch.bfloat16)
        b = (torch.rand(K, device=dev) - 0.5).to(torch.bfloat16)
        dy = (torch.randn((M, N), device=dev) * 1e-3).to(torch.bfloat16)
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        dh = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
        wf = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, False), dtype=torch.uint8, device=dev)
        wb = torch.empty(fp8.fp8_linear_bwd_sigmoid_workspace_bytes(M, K, N, r), dtype=torch.uint8, device=dev)
        lnq = fp8.fp8_layernorm_quantize(x, g, b, 1e-5, E4)
        wq = fp8.fp8_quantize(w, ROW, E4)

        def ln_sig_bwd(h, mean, rstd, yy, linear_bwd):
            dz = dy * yy * (1 - yy)
            linear_bwd(dz, h)
            torch.ops.aten.native_layer_norm_backward(dh, x, [K], mean, rstd, g, b, [True, True, True])

        def bf16_step():
            h, mean, rstd = torch.native_layer_norm(x, [K], g, b, 1e-5)
            yy = torch.sigmoid(torch.matmul(h, w.t()))

            def lb(dz, hh):
                torch.matmul(dz, w, out=dh)
                torch.matmul(dz.t(), hh, out=dw)
            ln_sig_bwd(h, mean, rstd, yy, lb)

        def fp8_step():
            h, mean, rstd = torch.native_layer_norm(x, [K], g, b, 1e-5)
            fp8.fp8_linear_fwd(h, w, r, y=y, workspace=wf)
            yy = torch.sigmoid(y)
            ln_sig_bwd(h, mean, rstd, yy, lambda dz, hh: fp8.fp8_linear_bwd(dz, hh, w, r, dx=dh, dw=dw, workspace=wb))

        def fused_step():
            h, hq, sh, mean, rstd = fp8.fp8_layernorm_quantize(x, g, b, 1e-5, E4, out=lnq)
            fp8.fp8_quantize(w, ROW, E4, out=wq[0], scale_out=wq[1])
            fp8.fp8_scaled_mm(hq, E4, sh, ROW, wq[0], E4, wq[1], ROW, fp8.FP8_EPILOGUE_SIGMOID, out=y)
            ln_sig_bwd(h, mean.view(M, 1), rstd.view(M, 1), y, lambda dz, hh: fp8.fp8_linear_bwd(dz, hh, w, r, dx=dh, dw=dw, workspace=wb))

        def fused_fwd_bwd_step():
            h, hq, sh, mean, rstd = fp8.fp8_layernorm_quantize(x, g, b, 1e-5, E4, out=lnq)
            fp8.fp8_quantize(w, ROW, E4, out=wq[0], scale_out=wq[1])
            fp8.fp8_scaled_mm(hq, E4, sh, ROW, wq[0], E4, wq[1], ROW, fp8.FP8_EPILOGUE_SIGMOID, out=y)
            fp8.fp8_linear_bwd_sigmoid(dy, y, h, w, r, dx=dh, dw=dw, workspace=wb)
            torch.ops.aten.native_layer_norm_backward(dh, x, [K], mean.view(M, 1), rstd.view(M, 1), g, b, [True, True, True])

        t_bf, t_f8, t_fu, t_fb = (_event_time_ms(f, iters, 2, torch) for f in (bf16_step, fp8_step, fused_step, fused_fwd_bwd_step))
        rows.append({"M": M, "K": K, "N": N, "bf16_ms": round(t_bf, 4), "fp8_ms": round(t_f8, 4), "fp8_fused_fwd_ms": round(t_fu, 4),
                     "fp8_fused_fwd_bwd_ms": round(t_fb, 4), "speedup_fp8": round(t_bf / t_f8, 3),
                     "speedup_fp8_fused_fwd": round(t_bf / t_fu, 3), "speedup_fp8_fused_fwd_bwd": round(t_bf / t_fb, 3)})
        del x, w, dy, y, dh, dw, wf, wb, lnq, wq
        torch.cuda.empty_cache()
    return {"block": "LayerNorm + Linear + Sigmoid forward and backward, float8 rowwise vs bfloat16, one MI355X",
            "iters": iters, "rows": rows}


def _configs(torch, fp8, dev, iters: int) -> dict:
    """Every synthetic workload of the configuration list (the Llama-3 8B / 70B
    linear shapes and the outlier case) on its own seeded data: the fp8 step of
    its recipe (forward only where the configuration has no backward) against
    the same products in bfloat16 by the vendor BLAS."""
    import synthetic_inputs as si

    def dev_bf16(bits):
        return torch.from_numpy(bits.view("int16")).to(dev).view(torch.bfloat16)

    rows = []
    for name, wl in si.WORKLOADS.items():
        M, K, N = wl.M, wl.K, wl.N
        x, w = dev_bf16(wl.x()), dev_bf16(wl.w())
        dy = dev_bf16(wl.dy()) if wl.backward else None
        gran = fp8.FP8_ROW if wl.recipe == si.ROWWISE else fp8.FP8_TENSOR
        fl = (fp8.FP8_POW2_SCALE if wl.pow2 else 0) | (fp8.FP8_SAVE_FOR_BWD if wl.backward else 0)
        r = fp8.Recipe(gran=gran, flags=fl)
        ws = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, r, wl.backward), dtype=torch.uint8, device=dev)
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        dw = torch.empty((N, K), dtype=torch.bfloat16, device=dev)

        def fp8_step():
            fp8.fp8_linear_fwd(x, w, r, y=y, workspace=ws)
            if wl.backward:
                fp8.fp8_linear_bwd(dy, (M, K), (N, K), r, dx=dx, dw=dw, workspace=ws)

        def bf16_step():
            torch.matmul(x, w.t(), out=y)
            if wl.backward:
                torch.matmul(dy, w, out=dx)
                torch.matmul(dy.t(), x, out=dw)
        t8 = _event_time_ms(fp8_step, iters, 3, torch)
        tb = _event_time_ms(bf16_step, iters, 3, torch)
        flop = (6.0 if wl.backward else 2.0) * M * N * K
        rows.append({"workload": name, "M": M, "K": K, "N": N, "recipe": "rowwise" if gran == fp8.FP8_ROW else "tensorwise",
                     "pow2_scales": bool(wl.pow2), "pass": "fwd+bwd" if wl.backward else "fwd",
                     "fp8_ms": round(t8, 4), "fp8_TFLOP/s": round(flop / t8 / 1e9, 1), "bf16_ms": round(tb, 4),
                     "speedup": round(tb / t8, 3)})
        del x, w, dy, y, dx, dw, ws
        torch.cuda.empty_cache()
    return {"configs": "fp8 linear step (dynamic quantization included) vs bf16 torch.matmul on every synthetic workload, one MI355X",
            "iters": iters, "rows": rows}


def _data_probe(torch, fp8, dev, iters: int) -> dict:
    """How much of the forward GEMM's rate depends on the operand DATA: the same
    kernel and launch on the benchmark shape with operands that do not toggle
    (all codes equal) and with realistic ones.  The difference is the board's
    power limit at work (the clock drops under toggling data), not the schedule."""
    import synthetic_inputs as si
    wl = si.WORKLOADS[si.BENCH_WORKLOAD]
    M, K, N = wl.M, wl.K, wl.N
    sa = torch.rand(M, device=dev) + 0.5
    sb = torch.rand(N, device=dev) + 0.5
    out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    x = torch.randn((M, K), device=dev).to(torch.bfloat16)
    w = (torch.randn((N, K), device=dev) * 0.02).to(torch.bfloat16)
    cases = {
        "all_zero_codes": (torch.zeros((M, K), dtype=torch.uint8, device=dev), torch.zeros((N, K), dtype=torch.uint8, device=dev)),
        "constant_codes_1.0": (torch.full((M, K), 0x38, dtype=torch.uint8, device=dev), torch.full((N, K), 0x38, dtype=torch.uint8, device=dev)),
        "uniform_random_codes": (torch.randint(0, 0x70, (M, K), dtype=torch.uint8, device=dev), torch.randint(0, 0x70, (N, K), dtype=torch.uint8, device=dev)),
        "rowwise_quantized_gaussian": (fp8.fp8_quantize(x, fp8.FP8_ROW, fp8.FP8_E4M3FN)[0], fp8.fp8_quantize(w, fp8.FP8_ROW, fp8.FP8_E4M3FN)[0]),
    }
    rows = {}
    for name, (a, b) in cases.items():
        run = lambda: fp8.fp8_scaled_mm(a, 0, sa, fp8.FP8_ROW, b, 0, sb, fp8.FP8_ROW, 0, out=out)
        best = min(_event_time_ms(run, iters, 3, torch) for _ in range(3))
        rows[name] = {"ms": round(best, 4), "TFLOP/s": round(2.0 * M * N * K / (best * 1e-3) / 1e12, 1),
                      "frac_of_fp8_peak": round(2.0 * M * N * K / (best * 1e-3) / 1e12 / FP8_PEAK_TFLOPS, 4)}
        clk = _shader_clock_under_load(run, torch)
        if clk:
            rows[name]["shader_clock_MHz_under_load"] = clk
    return {"data_probe": f"forward GEMM M={M} K={K} N={N}, same kernel, operands of different bit activity; the shader clock is "
                          "what rocm-smi reports while the kernel runs back to back for 1.5 s (nominal 2400 MHz)", "rows": rows}


def _shader_clock_under_load(run, torch, seconds: float = 1.5):
    """Median of the shader clock that `rocm-smi --showclocks` reports while run() is launched back to
    back (None if the tool is not there or prints something else)."""
    import re
    import subprocess
    import threading
    import time
    if any(k.startswith(("ROCP_", "ROCPROF")) for k in os.environ):
        return None                      # under a profiler: its environment would reach the child process too
    samples, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            try:
                out = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=10).stdout
                m = re.search(r'"sclk clock speed:"\s*:\s*"\((\d+)Mhz\)"', out)
                if m:
                    samples.append(int(m.group(1)))
            except (OSError, subprocess.SubprocessError):
                return
            time.sleep(0.1)
    th = threading.Thread(target=poll)
    th.start()
    t0 = time.time()
    while time.time() - t0 < seconds:
        for _ in range(20):
            run()
        torch.cuda.synchronize()
    stop.set()
    th.join()
    samples = sorted(samples[1:])          # the first sample may predate the load
    return samples[len(samples) // 2] if samples else None


def _decode(torch, fp8, dev, iters: int) -> dict:
    """Inference with weights quantized once (Section 3: dynamic activation +
    weight FP8 quantization, per row), few tokens per step: the GEMM streams the
    weight once, so the roofline is HBM (N*K bytes per launch).  Weights rotate
    through > 1.5 GB of copies, as the layers of a model would, so that nothing
    is served from the last-level cache.  bf16 comparator: torch.matmul."""
    rows = []
    shapes = (("llama3_8b_qkv", 6144, 4096), ("llama3_8b_o", 4096, 4096), ("llama3_8b_ffn_up", 14336, 4096),
              ("llama3_8b_ffn_down", 4096, 14336), ("llama3_70b_ffn_up", 28672, 8192), ("llama3_70b_ffn_down", 8192, 28672))
    E4, ROW = fp8.FP8_E4M3FN, fp8.FP8_ROW
    # what one launch costs when it follows another in a graph: a one-thread kernel (fp8_scale of one amax), 64 in a row
    one_amax, one_scale = torch.ones(1, device=dev), torch.empty(1, device=dev)
    floor_us = _graph_time_ms(lambda: [fp8.fp8_scale(one_amax, E4, 0, out=one_scale) for _ in range(64)], 20, torch) / 64 * 1e3
    for name, N, K in shapes:
        ncopy = max(2, -(-1_600_000_000 // (N * K)))
        ws = [(torch.randn((N, K), device=dev) * 0.02).to(torch.bfloat16) for _ in range(ncopy)]
        q = [fp8.fp8_quantize(w, ROW, E4) for w in ws]
        for M in (1, 4, 8, 16, 32):
            x = torch.randn((M, K), device=dev).to(torch.bfloat16)
            y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            wsp = torch.empty(fp8.fp8_linear_prequantized_workspace_bytes(M, K), dtype=torch.uint8, device=dev)
            xq, sx = fp8.fp8_quantize(x, ROW, E4)
            st = {"i": 0}

            def full():
                i = st["i"] = (st["i"] + 1) % len(q)
                fp8.fp8_linear_fwd_prequantized(x, q[i][0], E4, q[i][1], ROW, E4, ROW, 0, y=y, workspace=wsp)

            def gemm():
                i = st["i"] = (st["i"] + 1) % len(q)
                fp8.fp8_scaled_mm(xq, E4, sx, ROW, q[i][0], E4, q[i][1], ROW, 0, out=y)

            def bf16():
                i = st["i"] = (st["i"] + 1) % len(ws)
                torch.matmul(x, ws[i].t(), out=y)
            t_full = _event_time_ms(full, iters, len(q), torch)
            t_gemm = _event_time_ms(gemm, iters, len(q), torch)
            t_bf16 = _event_time_ms(bf16, iters, len(ws), torch)
            # the same calls replayed from a HIP graph that walks all weight copies once (what a serving engine does
            # with its decode step): no per-call host cost, the launches follow each other on the GPU
            reps = max(1, iters // len(q))
            g_full = _graph_time_ms(lambda: [full() for _ in range(len(q))], reps, torch) / len(q)
            g_gemm = _graph_time_ms(lambda: [gemm() for _ in range(len(q))], reps, torch) / len(q)
            g_bf16 = _graph_time_ms(lambda: [bf16() for _ in range(len(ws))], reps, torch) / len(ws)
            gbs = N * K / (t_gemm * 1e-3) / 1e9
            ggbs = N * K / (g_gemm * 1e-3) / 1e9
            rows.append({"layer": name, "M": M, "N": N, "K": K, "fp8_linear_us": round(t_full * 1e3, 2),
                         "fp8_gemm_us": round(t_gemm * 1e3, 2), "weight_stream_GB/s": round(gbs, 1),
                         "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "bf16_matmul_us": round(t_bf16 * 1e3, 2),
                         "speedup_vs_bf16": round(t_bf16 / t_full, 3),
                         "graph_fp8_linear_us": round(g_full * 1e3, 2), "graph_fp8_gemm_us": round(g_gemm * 1e3, 2),
                         "graph_weight_stream_GB/s": round(ggbs, 1), "graph_frac_of_hbm_peak": round(ggbs / HBM_PEAK_GBS, 4),
                         "graph_bf16_matmul_us": round(g_bf16 * 1e3, 2), "graph_speedup_vs_bf16": round(g_bf16 / g_full, 3)})
        del ws, q
        torch.cuda.empty_cache()
    return {"decode": "fp8_linear_fwd_prequantized (rowwise activations and weights) vs torch.matmul bf16, one MI355X; "
                      "both cycle through > 1.6 GB of fp8 weight copies (and their bf16 originals)",
            "roofline": {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "algorithmic_bytes_per_launch": "N*K weight bytes"},
            "graph_one_thread_kernel_us": round(floor_us, 2), "iters": iters, "rows": rows}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-legs", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=2048)
    ap.add_argument("--cpu-full", action="store_true",
                    help="time the CPU oracle on the WHOLE workload instead of a token sample (minutes of CPU time)")
    ap.add_argument("--sweep", action="store_true",
                    help="fp8 vs bf16 linear fwd+bwd over a grid of (M, K, N); prints a JSON table and exits")
    ap.add_argument("--decode", action="store_true",
                    help="inference with pre-quantized weights at decode batch sizes (weight-streaming GEMM); "
                         "prints a JSON table and exits")
    ap.add_argument("--block", action="store_true",
                    help="LayerNorm + Linear + Sigmoid forward and backward, float8 vs bfloat16 over shapes, then exit")
    ap.add_argument("--configs", action="store_true",
                    help="the fp8 step of every synthetic workload (Llama-3 8B / 70B shapes, outlier case) vs bf16, then exit")
    ap.add_argument("--data-probe", action="store_true",
                    help="time the forward GEMM with operands that do not toggle and with realistic ones, then exit")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="launch a 1 GiB device copy and every kernel of the step twice, then exit "
                         "(run under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2507_16099_amd as fp8
    import synthetic_inputs as si

    if not os.path.exists(fp8.library_path()):
        from paper_2507_16099_amd import build as _b
        _b.build()
    fp8.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.sweep:
        print(json.dumps(_sweep(torch, fp8, dev, max(5, args.steps // 2))))
        return 0

    if args.decode:
        print(json.dumps(_decode(torch, fp8, dev, max(10, args.steps))))
        return 0

    if args.block:
        print(json.dumps(_block(torch, fp8, dev, max(5, args.steps // 2))))
        return 0

    if args.configs:
        print(json.dumps(_configs(torch, fp8, dev, max(10, args.steps))))
        return 0

    if args.data_probe:
        print(json.dumps(_data_probe(torch, fp8, dev, max(10, args.steps))))
        return 0

    wl = si.WORKLOADS[args.workload or si.BENCH_WORKLOAD]
    M, K, N = wl.M, wl.K, wl.N
    rowwise = wl.recipe == si.ROWWISE
    recipe = fp8.Recipe(gran=fp8.FP8_ROW if rowwise else fp8.FP8_TENSOR,
                        flags=fp8.FP8_POW2_SCALE if wl.pow2 else 0)

    # synthetic inputs of the workload's distributions, generated on the device
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed)

    def normal(shape, std):
        return (torch.randn(shape, generator=g, device=dev, dtype=torch.float32) * std).to(torch.bfloat16)

    def draw(dist, shape):
        if dist[0] == "normal":
            return normal(shape, dist[1])
        # Student-t with hot columns
        z = torch.randn(shape, generator=g, device=dev)
        chi = torch.distributions.Chi2(torch.tensor(float(dist[1]), device=dev)).sample(shape)
        v = z / torch.sqrt(chi / dist[1])
        ncol = int(round(dist[2] * shape[1]))
        if ncol:
            cols = torch.randperm(shape[1], generator=g, device=dev)[:ncol]
            v[:, cols] *= dist[3]
        return v.to(torch.bfloat16)

    x = draw(wl.x_dist, (M, K))
    w = draw(wl.w_dist, (N, K))
    dy = draw(wl.dy_dist, (M, N))
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    dw = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
    ws_f = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, recipe, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, recipe, True), dtype=torch.uint8, device=dev)

    def stateless_step():
        fp8.fp8_linear_fwd(x, w, recipe, y=y, workspace=ws_f)
        if wl.backward:
            fp8.fp8_linear_bwd(dy, x, w, recipe, dx=dx, dw=dw, workspace=ws_b)

    # The timed step: forward and backward share one workspace (FP8_SAVE_FOR_BWD), so the fp8 copies of
    # X and W that the backward needs are made by the forward from the same read as its own.  Every
    # step still quantizes X, W and dY from their bfloat16 originals (dynamic scaling); codes, scales and
    # results are identical to the stateless calls (tested bit for bit).
    if wl.backward:
        recipe_s = fp8.Recipe(gran=recipe.gran, flags=recipe.flags | fp8.FP8_SAVE_FOR_BWD)
        ws_s = torch.empty(fp8.fp8_linear_workspace_bytes(M, K, N, recipe_s, True), dtype=torch.uint8, device=dev)

        def step():
            fp8.fp8_linear_fwd(x, w, recipe_s, y=y, workspace=ws_s)
            fp8.fp8_linear_bwd(dy, (M, K), (N, K), recipe_s, dx=dx, dw=dw, workspace=ws_s)
    else:
        step = stateless_step

    if args.traffic_probe:
        # reference for the counters: a plain copy of known size (1 GiB read + 1 GiB written)
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
            step()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": wl.name, "copy_bytes_each_way": 1 << 30}))
        return 0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    n_gemm = 3 if wl.backward else 1
    flop_step = n_gemm * 2.0 * M * N * K
    value = flop_step / (ms_per_step * 1e-3) / 1e12

    result = {
        "metric": "fp8 scaled-GEMM TFLOP/s + cast GB/s; fp8 linear fwd+bwd vs bf16, 1 GPU",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3fn/e5m2 x fp32-accumulate -> bf16", "data": "synthetic",
        "config": {"workload": wl.name, "M": M, "K": K, "N": N, "recipe": wl.recipe, "pow2_scales": wl.pow2,
                   "pass": "fwd+bwd" if wl.backward else "fwd", "flop_per_step": flop_step,
                   "workspace": "shared by forward and backward (FP8_SAVE_FOR_BWD)" if wl.backward else "forward only"},
    }
    if wl.backward:
        ms0 = _event_time_ms(stateless_step, max(3, args.steps // 2), 2, torch)
        result["stateless_step"] = {"ms_per_step": round(ms0, 4), "TFLOP/s": round(flop_step / (ms0 * 1e-3) / 1e12, 1),
                                    "note": "separate workspaces: the backward re-reads X and W for its own copies"}

    # ------------------------------------------------ per-kernel legs
    if not args.no_kernel_legs:
        it, wu = max(5, args.steps), 3
        kernels = {}
        gran = fp8.FP8_ROW if rowwise else fp8.FP8_TENSOR
        fl = recipe.flags
        T = fp8.FP8_TRANSPOSE_OUT
        E4, E5 = fp8.FP8_E4M3FN, fp8.FP8_E5M2

        # operands for the GEMM legs (the same calls the linear makes)
        xq, sx = fp8.fp8_quantize(x, gran, E4, fl)
        wq, sw = fp8.fp8_quantize(w, gran, E4, fl)

        def gemm_leg(name, a, fa, sa, b, fb, sb, out):
            m, k = a.shape
            n = b.shape[0]
            ms = _event_time_ms(lambda: fp8.fp8_scaled_mm(a, fa, sa, gran, b, fb, sb, gran, 0, out=out), it, wu, torch)
            tf = 2.0 * m * n * k / (ms * 1e-3) / 1e12
            kernels[name] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_of_fp8_peak": round(tf / FP8_PEAK_TFLOPS, 4)}
            return ms, tf

        # Quantization legs stream through ROTATING copies of their input (and their
        # own outputs), enough of them that consecutive launches never touch the same
        # bytes within 1.5 GB: X and W alone (128 MB, 112 MB here) would otherwise be
        # served by the 256 MB last-level cache instead of HBM.
        def rotated(t):
            n = max(2, -(-1_500_000_000 // (t.numel() * t.element_size())))
            return [t] + [t.clone() for _ in range(n - 1)]

        def cast_leg(name, src, quant, elems, bytes_per_elem):
            """quant(input, q_out, scale_out) -> launches; q/scale buffers rotate with the input."""
            ins = rotated(src)
            outs = [quant(ins[0], None, None)]
            outs += [tuple(torch.empty_like(o) for o in outs[0]) for _ in ins[1:]]
            state = {"i": 0}

            def fn():
                i = state["i"] = (state["i"] + 1) % len(ins)
                quant(ins[i], *outs[i])
            ms = _event_time_ms(fn, max(it, 2 * len(ins)), len(ins), torch)
            gbs = elems * bytes_per_elem / (ms * 1e-3) / 1e9
            kernels[name] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "bytes_per_elem": bytes_per_elem,
                             "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "rotating_buffers": len(ins)}
            return outs[0]

        def q_fn(g_, fmt, flags):
            def run(inp, q, sc):
                if q is None:
                    return fp8.fp8_quantize(inp, g_, fmt, flags)
                return fp8.fp8_quantize(inp, g_, fmt, flags, out=q, scale_out=sc)
            return run

        # practical HBM ceiling: a plain device copy (read + write), same rotation
        def copy_leg():
            src = rotated(x)
            dst = [torch.empty_like(t) for t in src]
            state = {"i": 0}

            def fn():
                i = state["i"] = (state["i"] + 1) % len(src)
                dst[i].copy_(src[i])
            ms = _event_time_ms(fn, max(it, 2 * len(src)), len(src), torch)
            gbs = 2 * x.numel() * x.element_size() / (ms * 1e-3) / 1e9
            kernels["plain_copy_ceiling"] = {"ms": round(ms, 4), "GB/s": round(gbs, 1), "bytes_per_elem": 4,
                                             "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                                             "note": "torch copy_ of X, read + write; not part of the path"}
        copy_leg()

        fwd_ms, fwd_tf = gemm_leg("gemm_fwd", xq, E4, sx, wq, E4, sw, y)
        fwd_clock = _shader_clock_under_load(lambda: fp8.fp8_scaled_mm(xq, E4, sx, gran, wq, E4, sw, gran, 0, out=y), torch, 1.0)
        tag = "row" if rowwise else "tensor"
        bpe = 3 if rowwise else 5
        cast_leg(f"quant_x_{tag}", x, q_fn(gran, E4, fl), M * K, bpe)
        cast_leg(f"quant_w_{tag}", w, q_fn(gran, E4, fl), N * K, bpe)

        def amax_run(inp, a, _unused=None):
            if a is None:
                return (fp8.fp8_amax(inp, fp8.FP8_TENSOR),)
            fp8.fp8_amax(inp, fp8.FP8_TENSOR, out=a)
        cast_leg("amax_x_tensor", x, amax_run, M * K, 2)

        def cast_run(inp, q, _unused=None):
            if q is None:
                return (fp8.fp8_cast(inp, sx, gran, E4, 0),)
            fp8.fp8_cast(inp, sx, gran, E4, 0, out=q)
        cast_leg("cast_x_given_scale", x, cast_run, M * K, 3)
        if wl.backward:
            cgran = fp8.FP8_COL if rowwise else fp8.FP8_TENSOR
            gq, sg = cast_leg(f"quant_dy_{tag}", dy, q_fn(gran, E5, fl), M * N, bpe)
            wt, swt = cast_leg("quant_w_col_t", w, q_fn(cgran, E4, fl | T), N * K, 5)
            gemm_leg("gemm_dx", gq, E5, sg, wt, E4, swt, dx)
            del gq, wt
            gqt, sgt = cast_leg("quant_dy_col_t", dy, q_fn(cgran, E5, fl | T), M * N, 5)
            xt, sxt = cast_leg("quant_x_col_t", x, q_fn(cgran, E4, fl | T), M * K, 5)
            gemm_leg("gemm_dw", gqt, E5, sgt, xt, E4, sxt, dw)
            del gqt, xt
        torch.cuda.empty_cache()

        if wl.backward and rowwise:
            # rowwise_gw_hp recipe: dW in bfloat16 from the unquantized tensors (same flops, bf16 matrix-core peak)
            ms = _event_time_ms(lambda: fp8.fp8_grad_weight_hp(dy, x, dw), it, wu, torch)
            tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
            kernels["gemm_dw_bf16_hp"] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1),
                                          "frac_of_bf16_peak": round(tf / BF16_PEAK_TFLOPS, 4)}
            hp = fp8.Recipe(gran=fp8.FP8_ROW, flags=recipe.flags | fp8.FP8_GRAD_WEIGHT_HP)

            def hp_step():
                fp8.fp8_linear_fwd(x, w, hp, y=y, workspace=ws_f)
                fp8.fp8_linear_bwd(dy, x, w, hp, dx=dx, dw=dw, workspace=ws_b)
            hp_ms = _event_time_ms(hp_step, max(3, args.steps // 2), 2, torch)
            result["rowwise_gw_hp"] = {"ms_per_step": round(hp_ms, 4),
                                       "TFLOP/s": round(flop_step / (hp_ms * 1e-3) / 1e12, 1),
                                       "note": "same step with the weight gradient kept in bfloat16 (Appendix A)"}

        # LayerNorm in front of the linear with the cast fused into its epilogue (the block of the paper's
        # microbenchmark appendix), against the unfused pair: a framework LayerNorm, then the rowwise quantize
        if rowwise and K % 8 == 0 and K <= 16384:
            gamma = (torch.rand(K, device=dev) + 0.5).to(torch.bfloat16)
            beta = (torch.rand(K, device=dev) - 0.5).to(torch.bfloat16)

            def lnq(inp, *o):
                if o[0] is None:
                    r5 = fp8.fp8_layernorm_quantize(inp, gamma, beta, 1e-5, E4, fl & fp8.FP8_POW2_SCALE, want_stats=False)
                    return (r5[0], r5[1], r5[2])
                fp8.fp8_layernorm_quantize(inp, gamma, beta, 1e-5, E4, fl & fp8.FP8_POW2_SCALE, out=(o[0], o[1], o[2], None, None))
            cast_leg("layernorm_quant_x_fused", x, lnq, M * K, 5)
            xs_ln = rotated(x)
            qs_ln = [fp8.fp8_quantize(t_, gran, E4, fl) for t_ in xs_ln]
            st_ln = {"i": 0}

            def unfused():
                i = st_ln["i"] = (st_ln["i"] + 1) % len(xs_ln)
                hh = torch.nn.functional.layer_norm(xs_ln[i], (K,), gamma, beta, 1e-5)
                fp8.fp8_quantize(hh, gran, E4, fl, out=qs_ln[i][0], scale_out=qs_ln[i][1])
            ms = _event_time_ms(unfused, max(it, 2 * len(xs_ln)), len(xs_ln), torch)
            kernels["layernorm_then_quant_x_unfused"] = {"ms": round(ms, 4), "bytes_per_elem": 7,
                                                         "GB/s": round(M * K * 7 / (ms * 1e-3) / 1e9, 1),
                                                         "comparator": "torch layer_norm (bf16) + fp8_quantize rowwise"}
            del xs_ln, qs_ln
            torch.cuda.empty_cache()

        # MX (microscaling) forward: block quantization of X and W, block-scaled GEMM
        if K % 128 == 0:
            mq = lambda inp, q, e: fp8.fp8_mx_quantize(inp, E4) if q is None else fp8.fp8_mx_quantize(inp, E4, q, e)
            xm, xe = cast_leg("mx_quant_x", x, mq, M * K, 3)
            wm, we = fp8.fp8_mx_quantize(w, E4)
            ms = _event_time_ms(lambda: fp8.fp8_mx_scaled_mm(xm, E4, xe, wm, E4, we, 0, out=y), it, wu, torch)
            tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
            kernels["mx_gemm_fwd"] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_of_fp8_peak": round(tf / FP8_PEAK_TFLOPS, 4),
                                      "note": "scales in plain rows [rows, K/32]"}
            if K % 512 == 0:
                # the same product with the scale bytes in slabs of sixteen blocks (negative ld_e at the public entry points)
                xm2, xe2 = fp8.fp8_mx_quantize(x, E4, slabs=True)
                wm2, we2 = fp8.fp8_mx_quantize(w, E4, slabs=True)
                ms = _event_time_ms(lambda: fp8.fp8_mx_scaled_mm(xm2, E4, xe2, wm2, E4, we2, 0, out=y), it, wu, torch)
                tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
                kernels["mx_gemm_fwd_scale_slabs"] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1),
                                                      "frac_of_fp8_peak": round(tf / FP8_PEAK_TFLOPS, 4),
                                                      "note": "scales in slabs [K/512, rows, 16]"}
                del xm2, xe2, wm2, we2
            wsm = torch.empty(fp8.fp8_mx_linear_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
            ms = _event_time_ms(lambda: fp8.fp8_mx_linear_fwd(x, w, y=y, workspace=wsm), max(3, args.steps // 2), 2, torch)
            result["mx_linear_fwd"] = {"ms": round(ms, 4), "TFLOP/s": round(2.0 * M * N * K / (ms * 1e-3) / 1e12, 1),
                                       "note": "forward with both operands in MX blocks of 32 along K (E8M0 scales applied by the matrix cores)"}
            del xm, xe, wm, we
            # blockwise FP8 (1 x 128 tiles of X, 128 x 128 blocks of W, power-of-two scales): same GEMM, other quantizers
            bq1 = lambda inp, q, e: fp8.fp8_block_quantize(inp, 1, E4) if q is None else fp8.fp8_block_quantize(inp, 1, E4, q, e)
            bq128 = lambda inp, q, e: fp8.fp8_block_quantize(inp, 128, E4) if q is None else fp8.fp8_block_quantize(inp, 128, E4, q, e)
            cast_leg("block_quant_x_1x128", x, bq1, M * K, 3)
            cast_leg("block_quant_w_128x128", w, bq128, N * K, 3)
            ms = _event_time_ms(lambda: fp8.fp8_block_linear_fwd(x, w, y=y, workspace=wsm), max(3, args.steps // 2), 2, torch)
            result["block_linear_fwd"] = {"ms": round(ms, 4), "TFLOP/s": round(2.0 * M * N * K / (ms * 1e-3) / 1e12, 1),
                                          "note": "forward with X in tiles of 1 x 128 and W in blocks of 128 x 128 (blockwise FP8, power-of-two "
                                                  "scales applied by the matrix cores)"}
            if wl.backward and M % 128 == 0 and N % 128 == 0:
                mqt = lambda inp, q, e: fp8.fp8_mx_quantize_t(inp, E4) if q is None else fp8.fp8_mx_quantize_t(inp, E4, q, e)
                cast_leg("mx_quant_dy_t", dy, mqt, M * N, 3)

                mq_both = lambda inp, *o: fp8.fp8_mx_quantize_row_col(inp, E4) if o[0] is None else fp8.fp8_mx_quantize_row_col(inp, E4, out=o)
                cast_leg("mx_quant_dy_row_and_col_t", dy, mq_both, M * N, 4)
                cast_leg("mx_quant_x_t", x, mqt, M * K, 3)
                if M % 512 == 0:
                    # the same with the scale bytes in slabs (the layout the linear entry points use between their
                    # quantizers and products): the dwords of neighbouring output rows are 16 bytes apart instead of a scale row apart
                    mqt_s = lambda inp, q, e: fp8.fp8_mx_quantize_t(inp, E4, slabs=True) if q is None else fp8.fp8_mx_quantize_t(inp, E4, q, e)
                    cast_leg("mx_quant_dy_t_scale_slabs", dy, mqt_s, M * N, 3)
                    cast_leg("mx_quant_x_t_scale_slabs", x, mqt_s, M * K, 3)
                    bqt_s = lambda inp, q, e: fp8.fp8_block_quantize_t(inp, 1, E4, slabs=True) if q is None else fp8.fp8_block_quantize_t(inp, 1, E4, q, e)
                    cast_leg("block_quant_dy_t_128x1_scale_slabs", dy, bqt_s, M * N, 3)
                torch.cuda.empty_cache()
                wsb = torch.empty(fp8.fp8_mx_linear_bwd_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)

                def mx_step():
                    fp8.fp8_mx_linear_fwd(x, w, y=y, workspace=wsm)
                    fp8.fp8_mx_linear_bwd(dy, x, w, dx=dx, dw=dw, workspace=wsb)
                ms = _event_time_ms(mx_step, max(3, args.steps // 2), 2, torch)
                result["mx_linear_fwd_bwd"] = {"ms_per_step": round(ms, 4), "TFLOP/s": round(flop_step / (ms * 1e-3) / 1e12, 1),
                                               "note": "forward + backward with every operand in MX blocks along the contracted axis "
                                                       "(5 block-quantization passes, the gradient in both orientations from one read, + 3 block-scaled GEMMs)"}

                def block_step():
                    fp8.fp8_block_linear_fwd(x, w, y=y, workspace=wsm)
                    fp8.fp8_block_linear_bwd(dy, x, w, dx=dx, dw=dw, workspace=wsb)
                bqt = lambda inp, q, e: fp8.fp8_block_quantize_t(inp, 1, E4) if q is None else fp8.fp8_block_quantize_t(inp, 1, E4, q, e)
                cast_leg("block_quant_dy_t_128x1", dy, bqt, M * N, 3)
                ms = _event_time_ms(block_step, max(3, args.steps // 2), 2, torch)
                result["block_linear_fwd_bwd"] = {"ms_per_step": round(ms, 4), "TFLOP/s": round(flop_step / (ms * 1e-3) / 1e12, 1),
                                                  "note": "forward + backward of the blockwise recipe: 5 one-pass block quantizations (tiles of 1 x 128 "
                                                          "along each product's contraction axis, the weight in 128 x 128 blocks, the gradient in both "
                                                          "orientations from one read) + 3 block-scaled GEMMs"}
                del wsb
            del wsm

        # vendor FP8 GEMM on the forward operands (context only; never linked into the library)
        try:
            a8 = xq.view(torch.float8_e4m3fn)
            b8 = wq.view(torch.float8_e4m3fn).t()
            if rowwise:
                kw = dict(scale_a=(1.0 / sx).reshape(M, 1), scale_b=(1.0 / sw).reshape(1, N))
            else:
                kw = dict(scale_a=(1.0 / sx).reshape(()), scale_b=(1.0 / sw).reshape(()))
            vend = lambda: torch._scaled_mm(a8, b8, out_dtype=torch.bfloat16, **kw)
            vend()
            vms = _event_time_ms(vend, it, wu, torch)
            result["vendor_fp8_gemm_fwd"] = {"ms": round(vms, 4), "TFLOP/s": round(2.0 * M * N * K / (vms * 1e-3) / 1e12, 1),
                                             "comparator": "torch._scaled_mm (vendor library), benchmark only"}
        except Exception as exc:  # the comparator is optional; the path under test never depends on it
            result["vendor_fp8_gemm_fwd"] = {"error": f"{type(exc).__name__}: {str(exc)[:120]}"}
        # bf16 comparator: the same three products by the vendor BLAS through torch
        def bf16_step():
            torch.matmul(x, w.t(), out=y)
            if wl.backward:
                torch.matmul(dy, w, out=dx)
                torch.matmul(dy.t(), x, out=dw)
        bf_ms = _event_time_ms(bf16_step, max(3, args.steps // 2), 2, torch)
        fp8_ms = _event_time_ms(step, max(3, args.steps // 2), 2, torch)
        result["kernels"] = kernels
        result["vs_bf16"] = {"bf16_ms_per_step": round(bf_ms, 4), "fp8_ms_per_step": round(fp8_ms, 4),
                             "speedup": round(bf_ms / fp8_ms, 3),
                             "bf16_TFLOP/s": round(flop_step / (bf_ms * 1e-3) / 1e12, 1),
                             "comparator": "torch.matmul bf16 (vendor BLAS), benchmark only"}
        result["roofline"] = {"kernel": "forward scaled GEMM (gemm_fp8_stream_kernel<e4m3,e4m3>)", "bound": "mfma",
                              "achieved": round(fwd_tf, 1), "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                              "frac": round(fwd_tf / FP8_PEAK_TFLOPS, 4), "traffic": _profiled_traffic(wl.name),
                              "flop_per_launch": 2.0 * M * N * K, "avg_launch_ms": round(fwd_ms, 4),
                              "shader_clock_MHz_under_load": fwd_clock,
                              "note": "the shader clock is what rocm-smi reports while this kernel runs back to back (nominal 2400 MHz: "
                                      "the published peak assumes it); on operands that do not toggle the same launch holds 2.4 GHz and "
                                      "0.71 of the peak (bench.py --data-probe)"}

    # ------------------------------------------------ CPU oracle baseline
    if not args.no_cpu_baseline:
        from oracle import fp8_oracle as orc
        ms_rows = M if args.cpu_full else min(M, args.cpu_sample_rows)
        sub = si.scaled_down(wl, ms_rows, K, N)
        hx, hw, hdy = sub.x(), sub.w(), sub.dy()
        orec = orc.Recipe(gran=orc.ROW if rowwise else orc.TENSOR, pow2=wl.pow2)
        orc.lib()
        c0 = time.perf_counter()
        orc.linear_fwd(hx, hw, orec)
        if wl.backward:
            orc.linear_bwd_dx(hdy, hw, orec)
            orc.linear_bwd_dw(hdy, hx, orec)
        c1 = time.perf_counter()
        cflop = n_gemm * 2.0 * ms_rows * N * K
        # the cast path by itself: the oracle's rowwise (or tensorwise) quantization of the FULL weight tensor
        # (the largest tensor that is the same in the sample and in the whole workload), 3 bytes per element
        q0 = time.perf_counter()
        orc.quantize(hw, orc.ROW if rowwise else orc.TENSOR, orc.E4M3FN)
        q1 = time.perf_counter()
        full_s = (c1 - c0) * M / ms_rows
        sample = (f"the whole workload ({M} tokens): quantize + {n_gemm} GEMMs, {c1 - c0:.1f} s of CPU time" if ms_rows == M else
                  f"same workload with M reduced to {ms_rows} tokens (full K, N): quantize + {n_gemm} GEMMs, "
                  f"{c1 - c0:.1f} s of CPU time; the whole step extrapolates to {full_s:.0f} s, beyond the 10-30 s of CPU "
                  f"work that a default run allows (bench.py --cpu-full times it in full)")
        result["cpu_baseline"] = {"value": round(cflop / (c1 - c0) / 1e12, 6), "unit": "TFLOP/s",
                                  "cores": orc.num_threads(), "kind": "oracle", "sample": sample,
                                  "cast": {"value": round(3.0 * N * K / (q1 - q0) / 1e9, 3), "unit": "GB/s",
                                           "sample": f"amax + scale + cast of the full weight tensor [{N}, {K}] "
                                                     f"(3 bytes per element), {q1 - q0:.2f} s"}}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
