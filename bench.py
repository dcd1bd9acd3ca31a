#!/usr/bin/env python3
"""Benchmark of the lmKAN layer hot path on one MI355X.

A step is one forward + one backward (gradients w.r.t. inputs and coefficients) of the
headline layer: 1024 -> 1024, G = 16, batch 8192, float32 coefficients, synthetic seeded
inputs already resident in HBM.  Prints ONE JSON line.
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

PEAK_FP32_VECTOR_TFLOPS = 157.3     # MI355X: 256 CU x 128 FMA/clk x 2 flop x 2.4 GHz
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# file (profiles/bench_cfg3_f32_hbm_counters.md: counters scaled by what a plain 1 GiB copy reads,
# x2.000 and x1.000).  Counters cannot be read from inside the timed process, so the figure is stored
# here per (workload, storage, kernel); anything not measured reports null.
MEASURED_TRAFFIC_BYTES = {
    ("cfg3_1024x1024_G16", "f32", "backward_input_slab_kernel"): 1.581e9,
    ("cfg3_1024x1024_G16", "f32", "forward_slab_kernel"): 1.076e9,
    ("cfg3_1024x1024_G16", "f32", "backward_coef_stream_kernel"): 2.823e9,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)      # the paper's protocol: 10 warm-up + 20 timed
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--storage", default="f32", choices=["f32", "f16", "bf16"])
    ap.add_argument("--workload", default="cfg3_1024x1024_G16")
    ap.add_argument("--grid", type=int, default=0,
                    help="override the workload's number of grid intervals G (for sweeps over G)")
    ap.add_argument("--graph", action="store_true",
                    help="time the step as a replayed HIP graph (one launch per step instead of a dozen)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=8192)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run one plain device copy of 1 GiB (torch's copy kernel): "
                         "the known-size reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def stack_inference(args, pkg, wl, torch, np, dev):
    """cfg2 as it runs at inference (App. F.1): the four layers chained, the evaluation-mode batch
    normalisation after each hidden layer folded into that layer's table, forward only.  A step is
    one batch through the whole stack; workspace and activations are allocated once."""
    layers = wl.CFG2_LAYERS
    B = layers[0].batch
    g = torch.Generator(device="cpu").manual_seed(77)
    x = wl.make_x(layers[0], dev)
    descs, tables, outs = [], [], []
    need = 256
    for i, w in enumerate(layers):
        paper = pkg.LayerDesc(w.n_in, w.n_out, w.grid)
        P = wl.make_coef(w, dev)
        if i + 1 < len(layers):     # seeded stand-ins for the running statistics, as in the full-size test
            scale = (torch.rand((w.n_out,), generator=g) * 0.4 + 0.8) / (w.coef_std * (w.n_in / 2) ** 0.5)
            shift = torch.randn((w.n_out,), generator=g) * 0.2
            pkg.lmkan_fold(paper, P, 1.0, None, None, scale.to(dev), shift.to(dev))
        tables.append(pkg.lmkan_pack(paper, P))
        d = pkg.LayerDesc(w.n_in, w.n_out, w.grid, coef_layout=pkg.LMKAN_LAYOUT_PACKED)
        descs.append(d)
        outs.append(torch.empty((B, w.n_out), dtype=torch.float32, device=dev))
        need = max(need, pkg.lmkan_workspace_bytes(d, B, False))
    ws = torch.empty(need, dtype=torch.uint8, device=dev)

    def step():
        a = x
        for d, t, y in zip(descs, tables, outs):
            pkg.lmkan_forward(d, a, t, y=y, workspace=ws)
            a = y

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    fma = sum(4.0 * B * (w.n_in // 2) * w.n_out for w in layers)
    print(json.dumps({
        "metric": "lmKAN stack inference samples/sec (cfg2: 64->256->256->256->1, forward only, 1 GPU)",
        "value": round(B / (ms * 1e-3), 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"cfg2_stack_inference: batch={B} G=16, normalisation folded into the tables, "
                               "activations pass through device memory between the layers"},
        "tflops": round(2 * fma / (ms * 1e-3) / 1e12, 3)}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2509_07103_amd as pkg
    from paper_2509_07103_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    L = pkg.lib()
    if args.workload == "cfg2_stack_inference":
        return stack_inference(args, pkg, wl, torch, np, dev)
    conv = args.workload in wl.CONV_BY_NAME     # a convolution stage: rows = windows of the images
    w = wl.CONV_BY_NAME[args.workload] if conv else wl.BY_NAME[args.workload]
    if args.grid:
        import dataclasses
        w = dataclasses.replace(w, grid=args.grid, name=f"{w.name}@G={args.grid}")
    dt_code = {"f32": pkg.LMKAN_F32, "f16": pkg.LMKAN_F16, "bf16": pkg.LMKAN_BF16}[args.storage]
    B, K, n_out = w.batch, w.n_in // 2, w.n_out

    # ---- inputs, resident in HBM before anything is timed -------------------------------
    x = wl.make_image(w, dev) if conv else wl.make_x(w, dev)
    gy = wl.make_grad_y(w, dev)
    if w.name.startswith("cfg5") and args.storage == "bf16":
        P_stored = wl.make_coef_bf16_chunked(w, dev)      # no room for a float32 master beside it
    else:
        P_master = wl.make_coef(w, dev)
        P_stored = wl.store(P_master, args.storage).contiguous()
        if args.storage != "f32":
            del P_master
    paper = pkg.LayerDesc(w.n_in, n_out, w.grid, coef_dtype=dt_code)
    t0 = time.perf_counter()
    P_packed = pkg.lmkan_pack(paper, P_stored)
    torch.cuda.synchronize()
    pack_ms = (time.perf_counter() - t0) * 1e3
    desc = pkg.LayerDesc(w.n_in, n_out, w.grid, coef_dtype=dt_code, coef_layout=pkg.LMKAN_LAYOUT_PACKED)

    y = torch.empty((B, n_out), dtype=torch.float32, device=dev)
    gx = torch.empty_like(x)
    gP = torch.empty(paper.coef_shape(), dtype=torch.float32, device=dev)
    need = max(pkg.lmkan_workspace_bytes(desc, B, False), pkg.lmkan_workspace_bytes(desc, B, True), 256)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    d = desc.c()

    if conv:
        geom = pkg.Conv2d(w.n, w.h, w.w, w.c_in, w.kh, w.kw, w.stride).c()
        assert pkg.lmkan_conv2d_rows(pkg.Conv2d(w.n, w.h, w.w, w.c_in, w.kh, w.kw, w.stride))[0] == B

    def forward():
        if conv:
            st = L.lmkan_conv2d_forward(C.byref(d), C.byref(geom), x.data_ptr(), P_packed.data_ptr(), y.data_ptr(),
                                        ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
        else:
            st = L.lmkan_forward(C.byref(d), B, x.data_ptr(), P_packed.data_ptr(), y.data_ptr(),
                                 ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
        assert st == 0, pkg.lmkan_status_string(st)

    def backward_only(gx_ptr, gp_ptr):
        if conv:
            st = L.lmkan_conv2d_backward(C.byref(d), C.byref(geom), x.data_ptr(), P_packed.data_ptr(),
                                         gy.data_ptr(), gx_ptr, gp_ptr, ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
        else:
            st = L.lmkan_backward(C.byref(d), B, x.data_ptr(), P_packed.data_ptr(), gy.data_ptr(),
                                  gx_ptr, gp_ptr, ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
        assert st == 0, pkg.lmkan_status_string(st)

    def backward():
        backward_only(gx.data_ptr(), gP.data_ptr())

    def step():
        forward()
        backward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:      # the same step recorded once as a HIP graph and replayed (launch-bound layers)
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph):
            step()
        run_step = hip_graph.replay
        run_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- per-call durations with events on the launch stream ------------------------------
    def event_ms(fn, reps):
        e0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        e1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        for i in range(reps):
            e0[i].record()
            fn()
            e1[i].record()
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in zip(e0, e1)]))

    reps = max(3, min(args.steps, 20))
    null = C.c_void_p(0)

    def kernel_ms(fn, reps):
        """Duration of the call's main kernel alone: the library records the two events around it
        on the launch stream (lmkan_time_next_kernel), leaving out the passes before and after."""
        pairs = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            e1.record()         # the events exist from here on; the library records them again
            pkg.lmkan_time_next_kernel(e0, e1)
            fn()
            pairs.append((e0, e1))
        pkg.lmkan_time_next_kernel(None, None)
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in pairs]))

    fwd_ms = event_ms(forward, reps)
    bwd_ms = event_ms(backward, reps)
    gx_ms = event_ms(lambda: backward_only(gx.data_ptr(), null), reps)
    gp_ms = event_ms(lambda: backward_only(null, gP.data_ptr()), reps)

    fma = 4.0 * B * K * n_out       # Alg. 1: four multiply-adds per (sample, pair, output);
    fma_fwd = fma                   # each of the three passes does that many
    fma_bwd = 2.0 * fma
    s_bytes = 4 if args.storage == "f32" else 2
    # each call = its main kernel plus the small preamble-record / zero-fill / sort / transpose
    # launches; which kernel serves a call follows the library's own dispatch rules
    ok = n_out % 4 == 0 and B >= 256
    if n_out <= 8:
        fwd_name, gx_name = "forward_small_kernel", "backward_input_small_kernel"
    elif ok and w.grid <= 16:
        fwd_name, gx_name = "forward_slab_kernel", "backward_input_slab_kernel"
    elif ok and w.grid <= 34:
        fwd_name, gx_name = "forward_slab_narrow_kernel", "backward_input_slab_narrow_kernel"
    else:
        fwd_name, gx_name = "forward_generic_kernel", "backward_generic_kernel(grad_x)"
    gp_name = ("backward_coef_small_kernel" if n_out <= 8 else "backward_coef_stream_kernel" if n_out % 4 == 0
               else "backward_generic_kernel(grad_coef)")
    calls = {fwd_name: fwd_ms, gx_name: gx_ms, gp_name: gp_ms}
    kernels = {fwd_name: kernel_ms(forward, reps),
               gx_name: kernel_ms(lambda: backward_only(gx.data_ptr(), null), reps),
               gp_name: kernel_ms(lambda: backward_only(null, gP.data_ptr()), reps)}
    dom_name = max(kernels, key=kernels.get)
    dom_ms = kernels[dom_name]
    # algorithmic work of one such launch: 4 B K n_out multiply-adds; compulsory HBM bytes: the
    # table (read, or written in float32 by the coefficient gradient) + x + one y-sized tensor
    table_bytes = (w.grid + 1) ** 2 * K * n_out * (4 if "coef" in dom_name else s_bytes)
    algo_bytes = table_bytes + x.numel() * 4 + B * n_out * 4
    t_alu = 2.0 * fma / (PEAK_FP32_VECTOR_TFLOPS * 1e12)
    t_hbm = algo_bytes / (PEAK_HBM_GBS * 1e9)
    if t_hbm > t_alu:
        achieved = algo_bytes / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4)}
    else:
        achieved = 2.0 * fma / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "alu", "achieved": round(achieved, 3), "peak": PEAK_FP32_VECTOR_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_VECTOR_TFLOPS, 4)}
    roofline.update({"traffic": MEASURED_TRAFFIC_BYTES.get((w.name, args.storage, dom_name)),
                     "traffic_unit": "bytes per launch (HBM read + write)", "kernel": dom_name,
                     "kernel_ms": round(dom_ms, 4),
                     "kernels_ms": {k: round(v, 4) for k, v in kernels.items()},
                     "all_ms": {k: round(v, 4) for k, v in calls.items()},
                     "note": "kernel_ms / kernels_ms: the kernel alone, events recorded by the library around "
                             "its launch; all_ms: whole calls (kernel + preamble, sort, fill, transpose passes)"})

    out = {
        # the benchmark's metric; `value` is the samples/sec of a forward + backward step, the gather rate
        # and its ratio to the HBM peak are in "forward"
        "metric": f"lmKAN layer samples/sec + achieved gather GB/s vs HBM peak ({w.n_in}->{n_out}, 1 GPU)",
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": (f"convolution {w.kh}x{w.kw} stride {w.stride} on [{w.n}][{w.h}][{w.w}][{w.c_in}] images, "
                                f"a sample = one window; " if conv else "") +
                               f"{w.name}: n_in={w.n_in} n_out={n_out} G={w.grid} batch={B} "
                               f"coef_storage={args.storage} x~{w.x_kind} coef~N(0,{w.coef_std})",
                   "pass": "forward+backward(grad_x,grad_coef)", "coef_layout": "packed",
                   "launch": "hip graph replay" if args.graph else "stream launches",
                   "pack_ms_once": round(pack_ms, 3)},
        "forward": {"ms": round(fwd_ms, 4), "samples_per_s": round(B / (fwd_ms * 1e-3), 1),
                    "gather_GBps": round(fma_fwd * s_bytes / (fwd_ms * 1e-3) / 1e9, 1),
                    "gather_vs_hbm_peak": round(fma_fwd * s_bytes / (fwd_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3),
                    "tflops": round(2 * fma_fwd / (fwd_ms * 1e-3) / 1e12, 3)},
        "backward": {"ms": round(bwd_ms, 4), "samples_per_s": round(B / (bwd_ms * 1e-3), 1),
                     "tflops": round(2 * fma_bwd / (bwd_ms * 1e-3) / 1e12, 3)},
        "roofline": roofline,
    }

    # ---- Hessian regulariser of the same table (Sec. 3.5): value + gradient, HBM-bound ----------
    hval = torch.empty(1, dtype=torch.float64, device=dev)

    def hessian():
        st = L.lmkan_hessian_reg(C.byref(d), P_packed.data_ptr(), 1.0, hval.data_ptr(), gP.data_ptr(),
                                 torch.cuda.current_stream().cuda_stream)
        assert st == 0, pkg.lmkan_status_string(st)

    hess_ms = event_ms(hessian, reps)
    hess_bytes = (w.grid + 1) ** 2 * K * n_out * (s_bytes + 4)      # table read once, gradient written once
    out["hessian_reg"] = {"ms": round(hess_ms, 4), "GBps": round(hess_bytes / (hess_ms * 1e-3) / 1e9, 1),
                          "vs_hbm_peak": round(hess_bytes / (hess_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3),
                          "note": "value + gradient of the off-diagonal Hessian regulariser; not part of the step"}

    # ---- yardstick of App. G: a dense float32 linear layer of the same shape (library GEMM) ------------
    # The paper normalises its kernel by this ratio (about 8 on its H100 for large batches).  Context only.
    if not conv and w.n_in * n_out * 4 <= 1 << 28:
        xw = torch.randn((w.n_in, n_out), dtype=torch.float32, device=dev)
        yl = torch.empty((B, n_out), dtype=torch.float32, device=dev)
        for _ in range(3):      # library set-up and kernel selection happen on the first calls
            torch.matmul(x, xw, out=yl)
        torch.cuda.synchronize()
        lin_ms = event_ms(lambda: torch.matmul(x, xw, out=yl), reps)
        out["dense_linear"] = {"ms": round(lin_ms, 4), "forward_ratio": round(fwd_ms / lin_ms, 2),
                               "note": "torch.matmul float32 [B,n_in]x[n_in,n_out]; lmKAN forward time / this"}
        del xw, yl

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline: the oracle as it stands, on a bounded row sample ---------------------
    if not args.no_cpu_baseline:
        import oracle
        o = oracle.get()
        rows = min(args.cpu_rows, B)
        if conv:    # the oracle's own gathering of the windows into rows, timed with the rest
            n_img = -(-rows // (B // w.n))
            xh = o.conv2d_patches(x[:n_img].cpu().numpy(), w.kh, w.kw, w.stride)[:rows]
        else:
            xh = x[:rows].cpu().numpy()
        gyh = gy[:rows].cpu().numpy()
        Pc = P_stored.cpu().contiguous()
        Ph = Pc.numpy() if args.storage == "f32" else Pc.view(torch.int16).numpy().view(np.uint16)
        code = {"f32": 0, "f16": 1, "bf16": 2}[args.storage]
        t0 = time.perf_counter()
        o.forward(xh, Ph, w.grid, dtype=code, threads=1)
        o.backward_input(xh, Ph, gyh, w.grid, dtype=code, threads=1)
        for k in range(K):
            o.backward_coef_pair(xh, gyh, w.grid, k)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(rows / cpu_s, 3), "unit": "samples/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"first {rows} rows of the same batch through oracle forward, "
                                         f"backward_input and backward_coef_pair for all {K} pairs "
                                         f"(full-size table), {cpu_s:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
