#!/usr/bin/env python3
"""Benchmark of the lmKAN layer hot path on one MI355X.

A step is one forward + one backward (gradients w.r.t. inputs and coefficients) of the
headline layer: 1024 -> 1024, G = 16, batch 8192, float32 coefficients, synthetic seeded
inputs already resident in HBM.  Prints ONE JSON line: the headline step, the kernel that
dominates it against its roofline (with what this machine was measured to deliver on the
primitive streams, and the HBM traffic of that kernel from the committed rocprofv3 counter
summary), the other four configurations in short runs, and the CPU oracle on a row sample.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_VECTOR_TFLOPS = 157.3     # MI355X: 256 CU x 128 FMA/clk x 2 flop x 2.4 GHz
PEAK_HBM_GBS = 8000.0
HEADLINE = "cfg3_1024x1024_G16"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)      # the paper's protocol: 10 warm-up + 20 timed
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--storage", default="f32", choices=["f32", "f16", "bf16"])
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--grid", type=int, default=0,
                    help="override the workload's number of grid intervals G (for sweeps over G)")
    ap.add_argument("--graph", action="store_true",
                    help="time the step as a replayed HIP graph (one launch per step instead of a dozen)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="leave out the short runs of the other configurations")
    ap.add_argument("--cpu-rows", type=int, default=4096)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run one plain device copy of 1 GiB (torch's copy kernel): "
                         "the known-size reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def kernel_names(w, n_out, B, storage, packed):
    """Main kernel of a forward call, of a grad_x-only call and of a grad_coef-only call, and of a call
    for both gradients when one kernel forms both: mirrors the library's dispatch (lmkan_api.hip)."""
    # (the forward pass alone takes the slab kernels from pairs x outputs >= 1024 on; every workload
    # of this file has 256 rows or more, where both rules say yes)
    ok = (n_out % 4 == 0 or packed) and (B >= 256 or (w.n_in // 2) * n_out >= 8192)
    both = None
    if n_out == 1 or (n_out <= 8 and not (ok and w.grid <= 34)):
        fwd, gx, gp = "forward_small_kernel", "backward_input_small_kernel", "backward_coef_small_kernel"
        # one output on rows: the tables of 64 pairs (or of all) fit LDS, the kernel locates by itself
        fit = ((160 * 1024 - 1024) // 4) // ((w.grid + 1) ** 2 | 1)
        if n_out == 1 and not getattr(w, "kh", 0) and (fit >= w.n_in // 2 or fit >= 64):
            fwd, gx, gp = "forward_head_kernel", "backward_input_head_kernel", "backward_coef_head_kernel"
    elif ok and w.grid <= 16:
        f16 = storage == "f16" and (packed or n_out % 8 == 0)
        fwd = "forward_slab_f16_kernel" if f16 else "forward_slab_kernel"
        gx = ("backward_input_slab_f16_kernel" if f16 else
              "backward_input_lane_kernel" if storage == "f32" else "backward_input_slab_kernel")
        gp = "backward_coef_stream_kernel"
    elif ok and w.grid <= 34:
        fwd, gx, gp = "forward_slab_narrow_kernel", "backward_input_slab_narrow_kernel", "backward_coef_stream_kernel"
        # 32-output tiles of a packed table as it is stored, where two such slabs fit LDS
        if packed and storage != "f32":
            fwd, gx = "forward_lane32_kernel", "backward_input_lane32_kernel"
        elif packed and 2 * (w.grid + 1) ** 2 * 128 + 256 <= 160 * 1024:
            fwd, gx = "forward_lane32_f32_kernel", "backward_input_lane32_f32_kernel"
        elif B >= 16 * w.grid * w.grid:
            both = "backward_fused_kernel"
    elif ok:
        # one 16-output slab at a time fits LDS up to G = 48
        fwd = "forward_slab_narrow_kernel" if (w.grid + 1) ** 2 * 64 <= 160 * 1024 - 512 else "forward_generic_kernel"
        gx, gp = "backward_fused_kernel", "backward_coef_stream_kernel"
        both = "backward_fused_kernel"
    else:
        fwd, gx = "forward_generic_kernel", "backward_generic_kernel(grad_x)"
        gp = "backward_coef_stream_kernel"
    return fwd, gx, gp, both


def profile_traffic(workload, storage, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary of this workload
    (profiles/bench_<workload>_<storage>_hbm_counters.md, a table whose last column is read + written
    bytes).  Counters cannot be read from inside the timed process; a kernel the summary does not list
    reports null with the reason, so a renamed or replaced kernel cannot keep a stale figure."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_{storage}_hbm_counters.md")
    if not os.path.exists(path):
        return None, f"no counter summary profiles/{os.path.basename(path)}"
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 2 and cells[0] == kernel:
            m = re.fullmatch(r"([0-9.]+)\s*([kMG]?)B", cells[-1])
            if m:
                return float(m.group(1)) * {"": 1, "k": 1e3, "M": 1e6, "G": 1e9}[m.group(2)], os.path.basename(path)
    return None, f"{kernel} is not listed in profiles/{os.path.basename(path)}"


class Bench:
    def __init__(self):
        import numpy as np
        import torch

        import paper_2509_07103_amd as pkg
        from paper_2509_07103_amd import workloads as wl
        self.np, self.torch, self.pkg, self.wl = np, torch, pkg, wl
        self.dev = torch.device("cuda:0")
        self.L = pkg.lib()

    # ---- timing helpers ---------------------------------------------------------------------
    def event_ms(self, fn, reps):
        torch = self.torch
        e0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        e1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        for i in range(reps):
            e0[i].record()
            fn()
            e1[i].record()
        torch.cuda.synchronize()
        return float(self.np.mean([a.elapsed_time(b) for a, b in zip(e0, e1)]))

    def kernel_ms(self, fn, reps):
        """Duration of the call's main kernel alone: the library records the two events around it on
        the launch stream (lmkan_time_next_kernel), leaving out the passes before and after."""
        torch, pkg = self.torch, self.pkg
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
        return float(self.np.mean([a.elapsed_time(b) for a, b in pairs]))

    # ---- one layer (or convolution stage) -----------------------------------------------------
    def layer(self, name, storage, steps, warmup, grid=0, graph=False, detailed=False, keep=False):
        np, torch, pkg, wl, dev, L = self.np, self.torch, self.pkg, self.wl, self.dev, self.L
        conv = name in wl.CONV_BY_NAME      # a convolution stage: rows = windows of the images
        w = wl.CONV_BY_NAME[name] if conv else wl.BY_NAME[name]
        if grid:
            import dataclasses
            w = dataclasses.replace(w, grid=grid, name=f"{w.name}@G={grid}")
        dt_code = {"f32": pkg.LMKAN_F32, "f16": pkg.LMKAN_F16, "bf16": pkg.LMKAN_BF16}[storage]
        B, K, n_out = w.batch, w.n_in // 2, w.n_out

        # inputs, resident in HBM before anything is timed
        x = wl.make_image(w, dev) if conv else wl.make_x(w, dev)
        gy = wl.make_grad_y(w, dev)
        if w.name.startswith("cfg5") and storage == "bf16":
            P_stored = wl.make_coef_bf16_chunked(w, dev)      # no room for a float32 master beside it
        else:
            P_master = wl.make_coef(w, dev)
            P_stored = wl.store(P_master, storage).contiguous()
            del P_master
        paper = pkg.LayerDesc(w.n_in, n_out, w.grid, coef_dtype=dt_code)
        # a one-output table stays in the layout of Alg. 1 (contiguous over the pairs there; packing
        # would pad it to 64 columns)
        packed = n_out != 1
        t0 = time.perf_counter()
        P_packed = pkg.lmkan_pack(paper, P_stored) if packed else P_stored
        torch.cuda.synchronize()
        pack_ms = (time.perf_counter() - t0) * 1e3 if packed else 0.0
        if not keep:
            del P_stored
        layout = pkg.LMKAN_LAYOUT_PACKED if packed else pkg.LMKAN_LAYOUT_PAPER
        desc = pkg.LayerDesc(w.n_in, n_out, w.grid, coef_dtype=dt_code, coef_layout=layout)

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
            s = torch.cuda.current_stream().cuda_stream
            if conv:
                st = L.lmkan_conv2d_forward(C.byref(d), C.byref(geom), x.data_ptr(), P_packed.data_ptr(), y.data_ptr(),
                                            ws.data_ptr(), need, s)
            else:
                st = L.lmkan_forward(C.byref(d), B, x.data_ptr(), P_packed.data_ptr(), y.data_ptr(), ws.data_ptr(),
                                     need, s)
            assert st == 0, pkg.lmkan_status_string(st)

        # the backward call of a step runs on the same x and the same workspace as its forward call:
        # it is told that the records are there (LMKAN_FLAG_WORKSPACE_HAS_RECORDS) and skips the
        # preamble pass; the calls timed on their own below do everything themselves
        d_reuse = pkg.LayerDesc(w.n_in, n_out, w.grid, coef_dtype=dt_code, coef_layout=layout,
                                flags=pkg.LMKAN_FLAG_WORKSPACE_HAS_RECORDS).c()
        has_records = pkg.lmkan_workspace_bytes(desc, B, False) > 0

        def backward_only(gx_ptr, gp_ptr, desc_c=d):
            s = torch.cuda.current_stream().cuda_stream
            if conv:
                st = L.lmkan_conv2d_backward(C.byref(desc_c), C.byref(geom), x.data_ptr(), P_packed.data_ptr(),
                                             gy.data_ptr(), gx_ptr, gp_ptr, ws.data_ptr(), need, s)
            else:
                st = L.lmkan_backward(C.byref(desc_c), B, x.data_ptr(), P_packed.data_ptr(), gy.data_ptr(), gx_ptr,
                                      gp_ptr, ws.data_ptr(), need, s)
            assert st == 0, pkg.lmkan_status_string(st)

        null = C.c_void_p(0)

        def backward():
            backward_only(gx.data_ptr(), gP.data_ptr())

        def step():
            forward()
            backward_only(gx.data_ptr(), gP.data_ptr(), d_reuse if has_records else d)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        run_step = step
        if graph:      # the same step recorded once as a HIP graph and replayed (launch-bound layers)
            hip_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(hip_graph):
                step()
            run_step = hip_graph.replay
            run_step()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run_step()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

        reps = max(3, min(steps, 20))
        fwd_ms = self.event_ms(forward, reps)
        bwd_ms = self.event_ms(backward, reps)
        gx_ms = self.event_ms(lambda: backward_only(gx.data_ptr(), null), reps)
        gp_ms = self.event_ms(lambda: backward_only(null, gP.data_ptr()), reps)

        fma = 4.0 * B * K * n_out       # Alg. 1: four multiply-adds per (sample, pair, output); each of the
        s_bytes = 4 if storage == "f32" else 2      # three passes (forward, grad_x, grad_coef) does that many
        fwd_name, gx_name, gp_name, both_name = kernel_names(w, n_out, B, storage, packed)
        # the kernels that run in a step, each timed alone; a kernel that forms both gradients does
        # twice the multiply-adds
        kernels = {fwd_name: (self.kernel_ms(forward, reps), fma)}
        if both_name:
            kernels[both_name + "(grad_x+grad_coef)"] = (self.kernel_ms(backward, reps), 2 * fma)
        else:
            kernels[gx_name] = (self.kernel_ms(lambda: backward_only(gx.data_ptr(), null), reps), fma)
            kernels[gp_name] = (self.kernel_ms(lambda: backward_only(null, gP.data_ptr()), reps), fma)
        dom_name = max(kernels, key=lambda k: kernels[k][0])
        dom_ms, dom_fma = kernels[dom_name]
        # algorithmic work of one such launch: its multiply-adds; compulsory HBM bytes: the table (read,
        # or written in float32 by the coefficient gradient, or both) + x + one y-sized tensor
        nodes = (w.grid + 1) ** 2
        if "grad_x+grad_coef" in dom_name:
            table_bytes = nodes * K * n_out * (s_bytes + 4)
        else:
            table_bytes = nodes * K * n_out * (4 if "coef" in dom_name else s_bytes)
        algo_bytes = table_bytes + x.numel() * 4 + B * n_out * 4
        t_alu = 2.0 * dom_fma / (PEAK_FP32_VECTOR_TFLOPS * 1e12)
        t_hbm = algo_bytes / (PEAK_HBM_GBS * 1e9)
        if t_hbm > t_alu:
            achieved = algo_bytes / (dom_ms * 1e-3) / 1e9
            roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(achieved / PEAK_HBM_GBS, 4)}
        else:
            achieved = 2.0 * dom_fma / (dom_ms * 1e-3) / 1e12
            roofline = {"bound": "alu", "achieved": round(achieved, 3), "peak": PEAK_FP32_VECTOR_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_VECTOR_TFLOPS, 4)}
        traffic, source = profile_traffic(w.name, storage, dom_name.split("(")[0])
        roofline.update({"traffic": traffic, "traffic_unit": "bytes per launch (HBM read + write)",
                         "traffic_source": source, "kernel": dom_name, "kernel_ms": round(dom_ms, 4),
                         "algorithmic_bytes": algo_bytes, "algorithmic_fma": dom_fma,
                         "kernels_ms": {k: round(v[0], 4) for k, v in kernels.items()},
                         "calls_ms": {"forward": round(fwd_ms, 4), "backward(grad_x,grad_coef)": round(bwd_ms, 4),
                                      "backward(grad_x)": round(gx_ms, 4), "backward(grad_coef)": round(gp_ms, 4)},
                         "note": "kernel_ms / kernels_ms: the kernel alone, events recorded by the library around "
                                 "its launch; calls_ms: whole calls (kernel + preamble, sort, fill, transpose, "
                                 "combine passes)"})
        summary = {
            "workload": f"{w.name}: n_in={w.n_in} n_out={n_out} G={w.grid} batch={B} coef_storage={storage}",
            "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
            "samples_per_s": round(B / (ms_per_step * 1e-3), 1),
            "forward_ms": round(fwd_ms, 4), "grad_x_ms": round(gx_ms, 4), "grad_coef_ms": round(gp_ms, 4),
            "backward_ms": round(bwd_ms, 4),
            "forward_algorithmic_gather_GBps": round(fma * s_bytes / (fwd_ms * 1e-3) / 1e9, 1),
            "roofline": {k: roofline[k] for k in ("bound", "achieved", "peak", "unit", "frac", "kernel", "kernel_ms",
                                                  "traffic")},
        }
        if not detailed:
            return summary
        out = {
            # the benchmark's metric; `value` is the samples/sec of a forward + backward step
            "metric": f"lmKAN layer samples/sec + achieved gather GB/s vs HBM peak ({w.n_in}->{n_out}, 1 GPU)",
            "value": round(B / (ms_per_step * 1e-3), 1),
            "unit": "samples/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": round(ms_per_step, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            # the arithmetic type: products and sums are float32 whatever the table is stored in
            "dtype": "f32", "coef_storage": storage, "data": "synthetic",
            "config": {"workload": (f"convolution {w.kh}x{w.kw} stride {w.stride} on [{w.n}][{w.h}][{w.w}][{w.c_in}] "
                                    f"images, a sample = one window; " if conv else "") +
                                   f"{w.name}: n_in={w.n_in} n_out={n_out} G={w.grid} batch={B} "
                                   f"coef_storage={storage} x~{w.x_kind} coef~N(0,{w.coef_std})",
                       "pass": "forward+backward(grad_x,grad_coef); " +
                               ("the backward call reuses the preamble records its forward call left in the workspace"
                                if has_records else "the forward call locates its inputs itself and leaves no records"),
                       "coef_layout": "packed" if packed else "alg1",
                       "launch": "hip graph replay" if graph else "stream launches",
                       "pack_ms_once": round(pack_ms, 3)},
            "forward": {"ms": round(fwd_ms, 4), "samples_per_s": round(B / (fwd_ms * 1e-3), 1),
                        # 4 B K n_out coefficient operands x their size / time: what the multiply-adds pull
                        # through LDS and L2 together, not bytes that crossed the HBM interface
                        "algorithmic_gather_GBps": round(fma * s_bytes / (fwd_ms * 1e-3) / 1e9, 1),
                        "compulsory_hbm_GBps": round((nodes * K * n_out * s_bytes + x.numel() * 4 + B * n_out * 4) /
                                                     (fwd_ms * 1e-3) / 1e9, 1),
                        "hbm_peak_GBps": PEAK_HBM_GBS,
                        "tflops": round(2 * fma / (fwd_ms * 1e-3) / 1e12, 3)},
            "backward": {"ms": round(bwd_ms, 4), "samples_per_s": round(B / (bwd_ms * 1e-3), 1),
                         "tflops": round(4 * fma / (bwd_ms * 1e-3) / 1e12, 3)},
            "roofline": roofline,
        }

        # Hessian regulariser of the same table (Sec. 3.5): value + gradient, HBM-bound
        hval = torch.empty(1, dtype=torch.float64, device=dev)

        def hessian():
            st = L.lmkan_hessian_reg(C.byref(d), P_packed.data_ptr(), 1.0, hval.data_ptr(), gP.data_ptr(),
                                     torch.cuda.current_stream().cuda_stream)
            assert st == 0, pkg.lmkan_status_string(st)

        hess_ms = self.event_ms(hessian, reps)
        hess_bytes = nodes * K * n_out * (s_bytes + 4)      # table read once, gradient written once
        out["hessian_reg"] = {"ms": round(hess_ms, 4), "GBps": round(hess_bytes / (hess_ms * 1e-3) / 1e9, 1),
                              "vs_hbm_peak": round(hess_bytes / (hess_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3),
                              "note": "value + gradient of the off-diagonal Hessian regulariser; not part of the step"}
        if keep:
            self.kept = dict(w=w, conv=conv, x=x, gy=gy, P_stored=P_stored, storage=storage)
        return out

    # ---- cfg2 as it runs at inference -----------------------------------------------------------
    def stack_inference(self, steps, warmup):
        """cfg2 as it runs at inference (App. F.1): the four layers chained, the evaluation-mode batch
        normalisation after each hidden layer folded into that layer's table, forward only.  A step is
        one batch through the whole stack; workspace and activations are allocated once."""
        torch, pkg, wl, dev = self.torch, self.pkg, self.wl, self.dev
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
            # (the one-output table of the last layer stays in the layout of Alg. 1)
            tables.append(pkg.lmkan_pack(paper, P) if w.n_out != 1 else P)
            d = pkg.LayerDesc(w.n_in, w.n_out, w.grid,
                              coef_layout=pkg.LMKAN_LAYOUT_PACKED if w.n_out != 1 else pkg.LMKAN_LAYOUT_PAPER)
            descs.append(d)
            outs.append(torch.empty((B, w.n_out), dtype=torch.float32, device=dev))
            need = max(need, pkg.lmkan_workspace_bytes(d, B, False))
        ws = torch.empty(need, dtype=torch.uint8, device=dev)

        def step():
            a = x
            for d, t, y in zip(descs, tables, outs):
                pkg.lmkan_forward(d, a, t, y=y, workspace=ws)
                a = y

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        fma = sum(4.0 * B * (w.n_in // 2) * w.n_out for w in layers)
        t_alu_ms = 2.0 * fma / (PEAK_FP32_VECTOR_TFLOPS * 1e12) * 1e3
        return {"workload": f"cfg2_stack_inference: 64->256->256->256->1, batch={B} G=16, normalisation folded "
                            "into the tables, activations pass through device memory between the layers, forward only",
                "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4),
                "samples_per_s": round(B / (ms * 1e-3), 1), "tflops": round(2 * fma / (ms * 1e-3) / 1e12, 3),
                "roofline": {"bound": "alu", "frac": round(t_alu_ms / ms, 4), "peak": PEAK_FP32_VECTOR_TFLOPS,
                             "unit": "TFLOP/s", "achieved": round(2 * fma / (ms * 1e-3) / 1e12, 3),
                             "kernel": "four lmkan_forward calls (whole step)"}}

    # ---- what the machine delivers on the primitive streams -----------------------------------
    def machine(self):
        torch, pkg = self.torch, self.pkg
        scratch = torch.empty(1 << 30, dtype=torch.uint8, device=self.dev)
        out = {name: round(pkg.lmkan_microbench(code, scratch), 2) for name, code in pkg.MICROBENCH.items()}
        props = torch.cuda.get_device_properties(self.dev)
        out["compute_units"] = props.multi_processor_count
        per_clk = 2 * out["compute_units"] * out["nominal_clock_GHz"] * 1e9 / 1e12
        out["fma_vector_TFLOPs"] = round(out["fma_per_clk_cu"] * per_clk, 1)
        out["fma_mfma_4x4x1_TFLOPs"] = round(out["mfma_fma_per_clk_cu"] * per_clk, 1)
        out["note"] = ("lmkan_microbench on this box, this run: per clock at the nominal clock; packed float32 vector "
                       "instructions are switched off in this build, so the published vector peak (128 multiply-adds "
                       "per clock and compute unit) is not reachable by vector code here")
        return out

    # ---- CPU baseline: the oracle as it stands, on a bounded row sample -----------------------
    def cpu_baseline(self, rows_max):
        import concurrent.futures as cf

        import oracle
        np, torch = self.np, self.torch
        k = self.kept
        w, x, gy, P_stored, storage = k["w"], k["x"], k["gy"], k["P_stored"], k["storage"]
        o = oracle.get()
        B, K = w.batch, w.n_in // 2
        rows = min(rows_max, B)
        if k["conv"]:    # the oracle's own gathering of the windows into rows, timed with the rest
            n_img = -(-rows // (B // w.n))
            xh = o.conv2d_patches(x[:n_img].cpu().numpy(), w.kh, w.kw, w.stride)[:rows]
        else:
            xh = x[:rows].cpu().numpy()
        gyh = gy[:rows].cpu().numpy()
        Pc = P_stored.cpu().contiguous()
        Ph = Pc.numpy() if storage == "f32" else Pc.view(torch.int16).numpy().view(np.uint16)
        code = {"f32": 0, "f16": 1, "bf16": 2}[storage]
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)

        def run(threads):
            t0 = time.perf_counter()
            o.forward(xh, Ph, w.grid, dtype=code, threads=threads)
            o.backward_input(xh, Ph, gyh, w.grid, dtype=code, threads=threads)
            if threads == 1:
                for kk in range(K):
                    o.backward_coef_pair(xh, gyh, w.grid, kk)
            else:       # pair slices are independent; the C routine runs without the interpreter lock
                with cf.ThreadPoolExecutor(max_workers=threads) as pool:
                    list(pool.map(lambda kk: o.backward_coef_pair(xh, gyh, w.grid, kk), range(K)))
            return time.perf_counter() - t0

        one = run(1)
        many = run(cores) if cores > 1 else one
        sample = (f"first {rows} rows of the same batch through oracle forward, backward_input and "
                  f"backward_coef_pair for all {K} pairs (full-size table)")
        return {"value": round(rows / many, 3), "unit": "samples/s", "cores": cores, "kind": "oracle",
                "sample": f"{sample}, {many:.1f} s on {cores} threads",
                "one_core": {"value": round(rows / one, 3), "unit": "samples/s", "cores": 1, "seconds": round(one, 1)},
                "host_cores_available": cores, "host_cores_total": os.cpu_count()}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    b = Bench()
    if args.workload == "cfg2_stack_inference":
        r = b.stack_inference(args.steps, args.warmup)
        r.update({"metric": "lmKAN stack inference samples/sec (cfg2: 64->256->256->256->1, forward only, 1 GPU)",
                  "value": r["samples_per_s"], "unit": "samples/s", "n_gpus": 1, "higher_is_better": True,
                  "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                  "config": {"workload": r.pop("workload")}})
        print(json.dumps(r))
        return
    want_cpu = not args.no_cpu_baseline
    out = b.layer(args.workload, args.storage, args.steps, args.warmup, grid=args.grid, graph=args.graph,
                  detailed=True, keep=want_cpu)
    out["roofline"]["measured"] = b.machine()
    headline = args.workload == HEADLINE and not args.grid
    if headline and not args.no_configs:
        # the other four configurations of the benchmark spec, short runs (5 warm-up + 15 timed steps each;
        # the 46 ms steps of cfg5: 2 + 5)
        wl = b.wl
        configs = {}
        for name, storage in ((wl.CFG1.name, "f32"), (wl.CFG4.name, "f32"), (wl.CFG5.name, "bf16"),
                              (wl.CFG3.name, "f16")):
            torch.cuda.empty_cache()
            short = name == wl.CFG5.name
            configs[f"{name}_{storage}"] = b.layer(name, storage, 5 if short else 15, 2 if short else 5)
        torch.cuda.empty_cache()
        configs["cfg2_stack_inference"] = b.stack_inference(15, 5)
        for w in wl.CFG2_LAYERS:
            torch.cuda.empty_cache()
            configs[f"{w.name}_f32"] = b.layer(w.name, "f32", 15, 5)
        out["configs"] = configs
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=b.dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if want_cpu:
        out["cpu_baseline"] = b.cpu_baseline(args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
