#!/usr/bin/env python3
"""Benchmark of the ABFT-protected GEMM path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload square|dlrm|resnet50] [--no-extras]

A step is one pass of the whole protected path over one batch of synthetic input:
every linear layer of the workload runs through ``abft_gemm`` / ``abft_conv`` with the
scheme the intensity-guided selector picks for it (activation checksum, matrix
product with fused checksum epilogue, comparison).  Inputs are resident in HBM before
the timed region.  One JSON line is printed: whole-pass protected TFLOP/s, the ABFT
overhead against the same kernels run unprotected, the roofline figure of the dominant
kernel (HIP events around that kernel inside the timed region) and the CPU oracle
timed on a bounded sample.  Short extra legs report the other benchmark configurations.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

from paper_2104_09455_amd import binding as B  # noqa: E402
from paper_2104_09455_amd import workloads as wl  # noqa: E402

PEAK = {"f16": 2516.6e12, "bf16": 2516.6e12, "i8": 5033.2e12}  # dense MFMA, op/s
HBM = 8.0e12
DT = {"f16": B.F16, "bf16": B.BF16, "i8": B.I8}
TORCH_IN = {"f16": torch.float16, "bf16": torch.bfloat16, "i8": torch.int8}
TORCH_OUT = {"f16": torch.float16, "bf16": torch.bfloat16, "i8": torch.int32}
ESIZE = {"f16": 2, "bf16": 2, "i8": 1}
CSIZE = {"f16": 2, "bf16": 2, "i8": 4}
# HBM traffic of the dominant kernel per launch, from the rocprofv3 counter runs summarised under
# profiles/*_hbm_traffic.md: (FETCH_SIZE KiB, WRITE_SIZE KiB) per dispatch and the scale factors the
# copy probe of the same runs gave (2.0 and 1.0).  Keyed by (layer, M, N, K, dtype, mode).
TRAFFIC_KIB = {
    ("top1", 256, 1024, 1024, "f16", "thread"): (3129.5, 518.1),
    ("sq8192", 8192, 8192, 8192, "f16", "global"): (786912.9, 134962.9),
}
TRAFFIC_SCALE = (2.0, 1.0)


# --------------------------------------------------------------------------- #
# HIP events straight from the runtime (torch events only see torch's own stream)
# --------------------------------------------------------------------------- #
class Hip:
    def __init__(self):
        self.rt = ctypes.CDLL("libamdhip64.so")
        self.rt.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.rt.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.rt.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def event(self):
        e = ctypes.c_void_p()
        assert self.rt.hipEventCreate(ctypes.byref(e)) == 0
        return e.value

    def record(self, e, stream):
        assert self.rt.hipEventRecord(e, stream) == 0

    def elapsed_ms(self, e0, e1):
        assert self.rt.hipEventSynchronize(e1) == 0
        ms = ctypes.c_float()
        assert self.rt.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
        return ms.value

    def destroy(self, e):
        self.rt.hipEventDestroy(e)


# --------------------------------------------------------------------------- #
# one protected layer with its device buffers
# --------------------------------------------------------------------------- #
class LayerRun:
    def __init__(self, layer: wl.Layer, dtype: str, gen: torch.Generator, dist_a="uniform_01", dist_b="weights"):
        self.layer, self.dtype = layer, dtype
        self.dt = DT[dtype]
        M, N, K = layer.M, layer.N, layer.K
        dev = "cuda:0"
        a_shape = (layer.conv.batch, layer.conv.H, layer.conv.W, layer.conv.Cin) if layer.conv else (M, K)
        if dtype == "i8":
            self.A = torch.randint(-128, 128, a_shape, generator=gen, device=dev, dtype=torch.int32).to(torch.int8)
            self.B = torch.randint(-128, 128, (N, K), generator=gen, device=dev, dtype=torch.int32).to(torch.int8)
        else:
            a = torch.rand(a_shape, generator=gen, device=dev) if dist_a == "uniform_01" else (
                torch.randn(a_shape, generator=gen, device=dev) if dist_a == "normal" else
                torch.rand(a_shape, generator=gen, device=dev) * 2 - 1)
            b = torch.randn((N, K), generator=gen, device=dev)
            if dist_b == "weights":
                b = b * 0.02
            self.A, self.B = a.to(TORCH_IN[dtype]), b.to(TORCH_IN[dtype])  # B stored N x K (ABFT_B_NK)
        self.C = torch.zeros((M, N), dtype=TORCH_OUT[dtype], device=dev)
        self.flag = torch.zeros(1, dtype=torch.int32, device=dev)
        es = ESIZE[dtype]
        aligned = ((layer.conv.Cin if layer.conv else K) * es) % 16 == 0 and (K * es) % 16 == 0
        _, rn = B.abft_region_shape(M, N, K, self.dt, aligned)
        self.beta = torch.zeros(B.abft_beta_bytes(K, N, rn) // 8, dtype=torch.float64, device=dev)
        B.abft_weight_checksum(K, N, self.B, K, B.B_NK, self.dt, self.beta, block_n=rn)  # offline step (Sec. 2.5)
        self.pick = B.abft_select(M, N, K, self.dt)
        self.conv = None
        if layer.conv:
            c = layer.conv
            self.conv = B.Conv(c.batch, c.H, c.W, c.Cin, c.KH, c.KW, c.stride, c.pad)
            self.wsb = max(B.abft_conv_workspace_bytes(self.conv, N, self.dt, m) for m in (B.NONE, B.GLOBAL, B.THREAD))
        else:
            self.wsb = max(B.abft_workspace_bytes(M, N, K, self.dt, m) for m in (B.NONE, B.GLOBAL, B.THREAD))
        self.ws = torch.zeros(max(self.wsb, 256), dtype=torch.uint8, device=dev)
        self.flops = 2.0 * M * N * K
        self.bytes = ESIZE[dtype] * (M * K + K * N) + CSIZE[dtype] * M * N
        self.ai = self.flops / self.bytes

    def run(self, mode, stream=None):
        L = self.layer
        if self.conv is not None:
            B.abft_conv(self.conv, L.N, self.A, self.B, L.K, B.B_NK, self.C, L.N, self.dt, mode, beta=self.beta,
                        workspace=self.ws, workspace_bytes=self.wsb, fault_flag=self.flag, stream=stream)
        else:
            B.abft_gemm(L.M, L.N, L.K, self.A, L.K, self.B, L.K, B.B_NK, self.C, L.N, self.dt, mode,
                        beta=self.beta, workspace=self.ws, workspace_bytes=self.wsb, fault_flag=self.flag,
                        stream=stream)


def time_mode(hip: Hip, lr: LayerRun, mode: int, reps: int, warm: int, stream=None) -> float:
    """Mean device microseconds of one call (all kernels of the scheme): `reps` calls are captured
    into a HIP graph on a side stream and the graph is replayed, so that the figure is the GPU's
    time and not the Python caller's (a ctypes call costs more than a small layer's kernels)."""
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cap):
        for _ in range(max(1, warm)):
            lr.run(mode, cap.cuda_stream)
    cap.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=cap):
        for _ in range(reps):
            lr.run(mode, cap.cuda_stream)
    g.replay()
    torch.cuda.synchronize()
    n = 5 if reps >= 20 else 3
    t0 = time.perf_counter()
    for _ in range(n):
        g.replay()
    torch.cuda.synchronize()
    us = 1e6 * (time.perf_counter() - t0) / (n * reps)
    del g
    return us


ALL_ROWS = []   # every per-layer measurement of this run, for the selector study


def layer_table(hip, runs, reps, warm, stream, modes=(B.NONE, B.GLOBAL, B.THREAD)):
    rows = []
    for lr in runs:
        # enough calls per graph replay that the replay's own launch cost (some 10 us) disappears
        # in the per-call figure: about 1.5 ms of estimated device work, at most 100 calls
        est_us = max(lr.flops / PEAK[lr.dtype], lr.bytes / HBM) * 1e6 * 2 + 3.0
        n_calls = max(reps, min(100, int(1500.0 / est_us) + 1))
        t = {m: time_mode(hip, lr, m, n_calls, warm, stream) for m in modes}
        pick_t = t[lr.pick]
        roof = min(PEAK[lr.dtype], lr.ai * HBM)
        rows.append({
            "layer": lr.layer.name, "M": lr.layer.M, "N": lr.layer.N, "K": lr.layer.K,
            "ai": round(lr.ai, 1), "pick": B.MODE_NAMES[lr.pick],
            "us_none": round(t[B.NONE], 2), "us_global": round(t[B.GLOBAL], 2), "us_thread": round(t[B.THREAD], 2),
            "ovh_global_pct": round(100 * (t[B.GLOBAL] / t[B.NONE] - 1), 2),
            "ovh_thread_pct": round(100 * (t[B.THREAD] / t[B.NONE] - 1), 2),
            "ovh_pick_pct": round(100 * (pick_t / t[B.NONE] - 1), 2),
            "tflops_pick": round(lr.flops / pick_t / 1e6, 2),
            "roofline_frac_pick": round(lr.flops / (pick_t * 1e-6) / roof, 4),
        })
        # the other wavefront-level schemes of the paper's design space (Sec. 5.1, 5.2.1, 5.2.2; Table 1):
        # replication with single accumulation, one-sided with half-precision checksum adds, two-sided
        for m in (B.REPLICA, B.THREAD_HALF, B.TWOSIDED):
            if m in t:
                rows[-1]["us_" + B.MODE_NAMES[m]] = round(t[m], 2)
                rows[-1]["ovh_" + B.MODE_NAMES[m] + "_pct"] = round(100 * (t[m] / t[B.NONE] - 1), 2)
        ALL_ROWS.append(dict(rows[-1], dtype=lr.dtype))
    return rows


def selector_study(rows):
    """The analytic rule (global iff AI > CMR, Sec. 5.3) against the measured per-layer optimum over
    every layer measured in this run, and the threshold that would have served these layers best
    (scan over the observed intensities; the rule stays 'global above the threshold')."""
    fp = [r for r in rows if r["dtype"] != "i8"]
    if not fp:
        return None
    def cost(th):
        t = sum(r["us_global"] if r["ai"] > th else r["us_thread"] for r in fp)
        miss = sum(1 for r in fp if ((r["us_global"] <= r["us_thread"]) != (r["ai"] > th)))
        return t, miss
    best_t = sum(min(r["us_global"], r["us_thread"]) for r in fp)
    t_none = sum(r["us_none"] for r in fp)
    cands = [0.0] + sorted({r["ai"] for r in fp})
    fit = min(cands, key=lambda th: cost(th)[0])
    ta, ma = cost(314.6)
    tf, mf = cost(fit)
    return {"layers": len(fp), "spec_cmr": 314.6,
            "analytic": {"mispredicted": ma, "ovh_pct": round(100 * (ta / t_none - 1), 2)},
            "fitted": {"threshold": fit, "mispredicted": mf, "ovh_pct": round(100 * (tf / t_none - 1), 2)},
            "per_layer_best_ovh_pct": round(100 * (best_t / t_none - 1), 2),
            "global_faster_on": sum(1 for r in fp if r["us_global"] <= r["us_thread"])}


def summarize(rows):
    tn = sum(r["us_none"] for r in rows)
    tg = sum(r["us_global"] for r in rows)
    tt = sum(r["us_thread"] for r in rows)
    tp = sum(r["us_global"] if r["pick"] == "global" else r["us_thread"] for r in rows)
    best = sum(min(r["us_global"], r["us_thread"]) for r in rows)
    fl = sum(2.0 * r["M"] * r["N"] * r["K"] for r in rows)
    return {"layers": len(rows), "us_none": round(tn, 1), "ovh_global_pct": round(100 * (tg / tn - 1), 2),
            "ovh_thread_pct": round(100 * (tt / tn - 1), 2), "ovh_selector_pct": round(100 * (tp / tn - 1), 2),
            "ovh_profiled_best_pct": round(100 * (best / tn - 1), 2),
            "tflops_selector": round(fl / tp / 1e6, 2)}


# --------------------------------------------------------------------------- #
# caveats of the latency-bound layers, measured rather than argued
# --------------------------------------------------------------------------- #
def cold_cache_leg(layer: wl.Layer, dtype: str, gen, copies=320):
    """The layer with its operands rotating through `copies` distinct copies (more than the 256 MB
    Infinity Cache), so that every call streams its weights and activations from HBM: device
    microseconds per call, unprotected and thread-level, and the HBM rate they amount to."""
    M, N, K = layer.M, layer.N, layer.K
    dev = "cuda:0"
    a = torch.rand((copies, M, K), generator=gen, device=dev).to(TORCH_IN[dtype])
    b = (torch.randn((copies, N, K), generator=gen, device=dev) * 0.02).to(TORCH_IN[dtype])
    c = torch.zeros((M, N), dtype=TORCH_OUT[dtype], device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    es = ESIZE[dtype]
    out = {"copies": copies, "MB_per_copy": round((M * K + N * K) * es / 1e6, 2)}
    for mode in (B.NONE, B.THREAD):
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())

        def calls():
            for i in range(copies):
                B.abft_gemm(M, N, K, a.data_ptr() + i * M * K * es, K, b.data_ptr() + i * N * K * es, K, B.B_NK,
                            c, N, DT[dtype], mode, fault_flag=flag, stream=cap.cuda_stream)
        with torch.cuda.stream(cap):
            calls()
        cap.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=cap):
            calls()
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        us = 1e6 * (time.perf_counter() - t0) / (3 * copies)
        out["us_" + B.MODE_NAMES[mode]] = round(us, 2)
        out["hbm_GBps_" + B.MODE_NAMES[mode]] = round(((M * K + N * K) * es + M * N * CSIZE[dtype]) / us / 1e3, 1)
        del g
    out["false_alarms"] = int(flag.item())
    return out


def measured_ceilings(hip, gen):
    """Own ceilings: an element-wise copy kernel's HBM rate and the best unprotected product."""
    n = 1 << 28  # 1 GiB of fp32
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(2):
        torch.mul(src, 1.0, out=dst)
    e0, e1 = hip.event(), hip.event()
    st = torch.cuda.current_stream().cuda_stream or None
    hip.record(e0, st)
    for _ in range(5):
        torch.mul(src, 1.0, out=dst)
    hip.record(e1, st)
    ms = hip.elapsed_ms(e0, e1) / 5
    hip.destroy(e0)
    hip.destroy(e1)
    del src, dst
    torch.cuda.empty_cache()
    copy_gbps = 2 * n * 4 / (ms * 1e-3) / 1e9
    lr = LayerRun(wl.Layer("sq8192", 8192, 8192, 8192), "f16", gen, "normal", "normal")
    us = time_mode(hip, lr, B.NONE, 5, 2)
    tf = lr.flops / us / 1e6
    out = {"copy_GBps": round(copy_gbps, 1), "best_unprotected_fp16_TFLOPs": round(tf, 1),
           "measured_cmr_fp16": round(tf * 1e12 / (copy_gbps * 1e9), 1),
           "spec_cmr_fp16": round(PEAK["f16"] / HBM, 1)}
    try:
        out["mfma_from_registers_TFLOPs"] = mfma_shapes_leg()
    except Exception as e:
        out["mfma_from_registers_TFLOPs"] = {"error": repr(e)}
    try:
        out["sustained_clock_and_library_context"] = clock_context(lr)
    except Exception as e:  # (no rocm-smi, no permission: context only)
        out["sustained_clock_and_library_context"] = {"error": repr(e)}
    del lr
    torch.cuda.empty_cache()
    return out


def mfma_shapes_leg(secs=1.0):
    """What the matrix units sustain from registers alone (abft_mfma_probe: no memory traffic at all),
    per MFMA shape, on random fp16 operands and on zeros: the measurement behind the 16x16x32 shapes
    of the 256 x 256 tile.  Under the board's power limit the rate depends on the operands' values."""
    nbytes = B.abft_mfma_probe_bytes()
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    res = {}
    for dist in ("random", "zeros"):
        ops_t = (torch.rand(nbytes // 2, device="cuda:0") * 0.02 - 0.01).to(torch.float16) if dist == "random" \
            else torch.zeros(nbytes // 2, dtype=torch.float16, device="cuda:0")
        for shape in (32, 16):
            iters = 20000
            B.abft_mfma_probe(shape, B.F16, 200, ops_t, sink)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rate = 0.0
            while time.perf_counter() - t0 < secs:       # (the last batch: the clock has settled by then)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ops = sum(B.abft_mfma_probe(shape, B.F16, iters, ops_t, sink) for _ in range(10))
                e1.record()
                torch.cuda.synchronize()
                rate = ops / (e0.elapsed_time(e1) * 1e-3) / 1e12
            res[f"{'32x32x16' if shape == 32 else '16x16x32'}_{dist}"] = round(rate, 1)
        del ops_t
    return res


def clock_context(lr, secs=1.5):
    """Context for the fraction of the matrix unit's peak: the peak is quoted at 2.4 GHz, and a long
    run of dense products holds a lower clock under the board's power limit, which depends on the
    operands' values.  For the unprotected 8192^3 fp16 product on N(0,1) operands and on zeros:
    this library's rate and the shader clock rocm-smi shows meanwhile, and beside them the ROCm
    GEMM library's rate on the same operands (through torch.matmul; context only, no part of the
    path)."""
    import re
    import subprocess
    import threading
    samples, stop = [], [False]

    def poll():
        while not stop[0]:
            try:
                o = subprocess.run(["/opt/rocm/bin/rocm-smi", "--showclocks"], capture_output=True, text=True,
                                   timeout=5).stdout
                m = re.search(r"sclk clock level: \S+ \((\d+)Mhz\)", o)
                if m:
                    samples.append((time.perf_counter(), int(m.group(1))))
            except Exception:
                pass
            time.sleep(0.05)

    def run_for(fn, label, res):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 0
        e0.record()
        while time.perf_counter() - t0 < secs:
            for _ in range(50):
                fn()
            n += 50
            torch.cuda.synchronize()
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        us = e0.elapsed_time(e1) * 1e3 / n
        clk = [c for (t, c) in samples if t0 + 0.5 < t < t1]
        tf = lr.flops / us / 1e6
        res[label + "_TFLOPs"] = round(tf, 1)
        if clk:
            mhz = sum(clk) / len(clk)
            res[label + "_sclk_MHz"] = round(mhz)
            res[label + "_frac_of_peak_at_that_clock"] = round(tf / (PEAK["f16"] / 1e12 * mhz / 2400.0), 3)

    res = {}
    th = threading.Thread(target=poll, daemon=True)
    th.start()
    try:
        bt = lr.B.t()
        for dist in ("normal", "zeros"):
            if dist == "zeros":
                lr.A.zero_()
                lr.B.zero_()
            run_for(lambda: lr.run(B.NONE, None), f"this_library_{dist}", res)
            run_for(lambda: torch.matmul(lr.A, bt), f"rocm_gemm_library_{dist}", res)
    finally:
        stop[0] = True
        th.join(timeout=10)
    return res


# --------------------------------------------------------------------------- #
# CPU baseline: the oracle, as it stands, on a bounded sample of the workload
# --------------------------------------------------------------------------- #
def chain_leg(gen, batch=256, steps=300):
    """DLRM's two MLPs as chains (Sec. 2.4 step 4): ReLU fused into the store of every layer but
    each MLP's last, layer l's output handed to layer l + 1 as its input.  Two forms, both timed as
    device time of a whole pass replayed from a graph: one kernel launch per layer
    (abft_plan_run_all), and one launch per chain (abft_plan_run_chain: bottom MLP behind its K = 13
    layer, top MLP), each with the selector's schemes, all-global and unprotected."""
    layers = wl.dlrm_layers(batch)
    rs = [LayerRun(l, "f16", gen) for l in layers]
    plan = B.abft_plan_create([B.Layer(r.layer.M, r.layer.N, r.layer.K, r.dt, B.B_NK, 0, B.Conv(), r.B.data_ptr(),
                                       r.layer.K) for r in rs], profile=False)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    ins, last = [], []
    for i, r in enumerate(rs):
        head = i == 0 or not r.layer.name.startswith(rs[i - 1].layer.name[:3])   # first layer of an MLP
        ins.append(r.A if head else rs[i - 1].C)
        if i > 0 and head:
            last.append(i - 1)
    last.append(len(rs) - 1)
    for i in range(len(rs)):
        B.abft_plan_set_activation(plan, i, B.ACT_NONE if i in last else B.ACT_RELU)
    io = B.PlanIO(ins, [r.layer.K for r in rs], [r.C for r in rs], [r.layer.N for r in rs])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    n_bot = last[0] + 1                      # layers of the bottom MLP

    def per_layer(st):
        B.abft_plan_run_all(plan, io, flag, -1, st)

    def one_launch(st):
        # bottom MLP: its first layer (K = 13) on its own, the rest as one chain; top MLP: one chain
        B.abft_plan_run(plan, 0, rs[0].A, rs[0].layer.K, rs[0].C, rs[0].layer.N, flag, st)
        B.abft_plan_run_chain(plan, 1, n_bot - 1, rs[0].C, rs[0].layer.N, [r.C for r in rs[1:n_bot]],
                              [r.layer.N for r in rs[1:n_bot]], flag, st)
        B.abft_plan_run_chain(plan, n_bot, len(rs) - n_bot, rs[n_bot].A, rs[n_bot].layer.K, [r.C for r in rs[n_bot:]],
                              [r.layer.N for r in rs[n_bot:]], flag, st)

    def pass_us(fn):
        with torch.cuda.stream(side):
            fn(side.cuda_stream)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            fn(side.cuda_stream)
        for _ in range(10):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return 1e6 * (time.perf_counter() - t0) / steps

    res = {"batch": batch, "layers": [r.layer.name for r in rs], "relu_after": [r.layer.name for i, r in enumerate(rs) if i not in last]}
    try:
        for label, mode in (("selector", B.AUTO), ("global", B.GLOBAL), ("none", B.NONE)):
            for i in range(len(rs)):
                B.abft_plan_set_mode(plan, i, mode)
            res["us_" + label] = round(pass_us(per_layer), 2)
            res["us_" + label + "_one_launch_per_chain"] = round(pass_us(one_launch), 2)
        for form in ("", "_one_launch_per_chain"):
            res["ovh_selector_pct" + form] = round(100 * (res["us_selector" + form] / res["us_none" + form] - 1), 2)
            res["ovh_global_pct" + form] = round(100 * (res["us_global" + form] / res["us_none" + form] - 1), 2)
        res["false_alarms"] = int(flag.item())
        res["chain_status"] = B.abft_plan_chain_status(plan)
    finally:
        B.abft_plan_destroy(plan)
    return res


def handover_leg(gen, M=2048, widths=(4096, 4096, 4096, 4096, 4096), dtype="f16", steps=100):
    """A chain of mid-size, compute-bound fully-connected layers (ReLU between them) under the global
    scheme, where a stand-alone call pays 10-20 % for forming the activation checksum inside the
    product: every layer on its own (abft_plan_run) against the chain run layer by layer with each
    layer's activation checksums handed over by the epilogue of the layer before it (Sec. 2.4 step
    4; abft_plan_run_chain).  Device time of a whole pass, eager launches on one stream."""
    nl = len(widths) - 1
    rs = [LayerRun(wl.Layer(f"fc{i}", M, widths[i + 1], widths[i]), dtype, gen) for i in range(nl)]
    plan = B.abft_plan_create([B.Layer(M, widths[i + 1], widths[i], rs[i].dt, B.B_NK, 0, B.Conv(), rs[i].B.data_ptr(),
                                       widths[i]) for i in range(nl)], profile=False)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for i in range(nl):
        B.abft_plan_set_activation(plan, i, B.ACT_RELU if i + 1 < nl else B.ACT_NONE)
    Cs, ldc = [r.C for r in rs], [int(w) for w in widths[1:]]

    def alone():
        for i in range(nl):
            B.abft_plan_run(plan, i, rs[0].A if i == 0 else Cs[i - 1], widths[i], Cs[i], ldc[i], flag)

    def chain():
        B.abft_plan_run_chain(plan, 0, nl, rs[0].A, widths[0], Cs, ldc, flag)

    def pass_us(fn):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = float("inf")
        for _ in range(3):
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, 1e3 * e0.elapsed_time(e1) / steps)
        return best

    def brackets():
        """HIP events right around each layer's product kernel inside the chain (one layer per pass)."""
        hip = Hip()
        io = B.PlanIO([rs[0].A] + Cs[:-1], list(widths[:-1]), Cs, ldc)
        out = []
        for layer in range(nl):
            e0, e1 = hip.event(), hip.event()
            B.abft_set_kernel_events(e0, e1)
            tot = 0.0
            for it in range(15):
                B.abft_plan_run_all(plan, io, flag, layer)
                torch.cuda.synchronize()
                if it >= 5:
                    tot += 1e3 * hip.elapsed_ms(e0, e1)
            B.abft_set_kernel_events(None, None)
            hip.destroy(e0)
            hip.destroy(e1)
            out.append(round(tot / 10, 1))
        return out

    res = {"M": M, "widths": list(widths), "dtype": dtype}
    try:
        for label, mode in (("none", B.NONE), ("global", B.GLOBAL)):
            for i in range(nl):
                B.abft_plan_set_mode(plan, i, mode)
            res["us_" + label + "_alone"] = round(pass_us(alone), 2)
            before = B.abft_handover_launches()
            res["us_" + label + "_chain"] = round(pass_us(chain), 2)
            if mode == B.GLOBAL:
                res["layers_with_handed_over_checksums"] = (B.abft_handover_launches() - before) // (3 * steps + 5)
            # (the first layer's bracket also holds the start from an idle GPU)
            res["kernel_bracket_us_per_layer_" + label + "_chain"] = brackets()
        res["ovh_global_alone_pct"] = round(100 * (res["us_global_alone"] / res["us_none_alone"] - 1), 2)
        res["ovh_global_chain_pct"] = round(100 * (res["us_global_chain"] / res["us_none_chain"] - 1), 2)
        res["false_alarms"] = int(flag.item())
    finally:
        B.abft_plan_destroy(plan)
    return res


def cpu_baseline(runs, budget_s=12.0):
    """The oracle as it stands on a bounded sample of the workload: row blocks of A (whole images
    for a convolution) through the fp64 / int64 triple-loop product and the checksum scheme the
    selector picks, layer after layer until about budget_s seconds of CPU work are spent."""
    import oracle
    from oracle import build as obuild
    if not os.path.exists(os.path.join(ROOT, "oracle", "libabft_oracle.so")):
        obuild.build()

    def host(t, dtype):
        t = t.cpu()
        return t.numpy() if dtype == "i8" else t.view(torch.int16).numpy().view(np.float16 if dtype == "f16" else np.uint16)

    t_used, flops, desc = 0.0, 0.0, []
    for lr in runs:
        L = lr.layer
        if t_used >= budget_s:
            break
        Bw = np.ascontiguousarray(host(lr.B, lr.dtype).T)  # K x N, the oracle's orientation
        done = 0
        # blocks of about 2e9 multiply-adds, at most 4096 rows of a layer
        step = int(max(1, min(L.M, 2e9 // (L.N * L.K))))
        while done < min(L.M, 4096) and t_used < budget_s:
            if lr.conv is not None:
                c = L.conv
                per = c.OH * c.OW
                img0 = done // per
                imgs = max(1, min(c.batch - img0, math.ceil(step / per)))
                xs = host(lr.A[img0:img0 + imgs], lr.dtype)
                t0 = time.perf_counter()
                Aw = oracle.im2col(xs, lr.dtype, c.KH, c.KW, c.stride, c.pad)
            else:
                Aw = host(lr.A[done:done + step], lr.dtype)
                t0 = time.perf_counter()
            Cw = oracle.gemm(Aw, Bw, lr.dtype)
            if lr.pick == B.GLOBAL:
                oracle.global_check(Aw, Bw, Cw, lr.dtype)
            else:
                tm, tn, _ = B.abft_tile_shape(L.M, L.N, L.K, lr.dt, True)
                oracle.thread_check(Aw, Bw, Cw, lr.dtype, tm, tn)
            t_used += time.perf_counter() - t0
            flops += 2.0 * Aw.shape[0] * L.N * L.K
            done += Aw.shape[0]
        desc.append(f"{L.name}:{done}/{L.M} rows")
    return {"value": round(flops / t_used / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.threads(),
            "kind": "oracle", "seconds": round(t_used, 2),
            "sample": "fp64 triple-loop GEMM + the selected checksum scheme on " + ", ".join(desc[:12]) +
                      (" ..." if len(desc) > 12 else "")}


# --------------------------------------------------------------------------- #
# the comparison tolerance, stated as a number per configuration
# --------------------------------------------------------------------------- #
def _report_of(lr: "LayerRun", mode: int):
    rep = torch.zeros(ctypes.sizeof(B.Report), dtype=torch.uint8, device="cuda:0")
    lr.flag.zero_()
    L = lr.layer
    if lr.conv is not None:
        B.abft_conv(lr.conv, L.N, lr.A, lr.B, L.K, B.B_NK, lr.C, L.N, lr.dt, mode, beta=lr.beta, workspace=lr.ws,
                    workspace_bytes=lr.wsb, fault_flag=lr.flag, report=rep)
    else:
        B.abft_gemm(L.M, L.N, L.K, lr.A, L.K, lr.B, L.K, B.B_NK, lr.C, L.N, lr.dt, mode, beta=lr.beta,
                    workspace=lr.ws, workspace_bytes=lr.wsb, fault_flag=lr.flag, report=rep)
    torch.cuda.synchronize()
    return B.Report.from_buffer_copy(rep.cpu().numpy().tobytes()), int(lr.flag.item())


def tolerance_row(lr: "LayerRun", mode: int, label: str):
    """tau of the comparison with the largest residual / tau in one clean run, as the device formed
    it: tau = coeff * ||C_S||_F + bias_coeff * ||C_S||_1 over the region S (workgroup tile for the
    global scheme, wavefront tile for the thread-level one).  min_flagged_over_rms: the smallest
    change of one element of C that must be flagged (2 tau), in units of the region's rms(C)."""
    L = lr.layer
    if lr.dtype == "i8":
        return {"config": label, "dtype": "i8", "scheme": B.MODE_NAMES[mode], "tau": 0.0,
                "note": "exact integer comparison: every single-bit flip changes the sum"}
    rep, flagged = _report_of(lr, mode)
    aligned = ((L.conv.Cin if L.conv else L.K) * 2) % 16 == 0
    rm, rn = (B.abft_region_shape(L.M, L.N, L.K, lr.dt, aligned) if mode == B.GLOBAL
              else B.abft_tile_shape(L.M, L.N, L.K, lr.dt, aligned)[:2])
    n_el = min(rm, L.M) * min(rn, L.N)
    rms = rep.frob / math.sqrt(n_el) if n_el else 0.0
    return {"config": label, "dtype": lr.dtype, "scheme": B.MODE_NAMES[mode], "region": [rm, rn], "K": L.K,
            "coeff": B.abft_tolerance_coeff(L.K, lr.dt, mode), "bias_coeff": B.abft_tolerance_bias_coeff(L.K, lr.dt, mode),
            "tau": float(f"{rep.tau:.4g}"), "frob_region": float(f"{rep.frob:.4g}"), "rms_region": float(f"{rms:.4g}"),
            "clean_residual_over_tau": round(rep.worst_ratio, 3),
            "min_flagged_over_rms": float(f"{(2 * rep.tau / rms) if rms else 0.0:.3g}"), "comparisons": rep.tiles,
            "false_alarm": flagged}


def tolerance_leg(gen):
    """One row per benchmark configuration (representative layers; the scheme the selector picks)."""
    rows = []
    def add(layer, dtype, label, da="uniform_01", db="weights", modes=None):
        lr = LayerRun(layer, dtype, gen, da, db)
        for m in (modes or (lr.pick,)):
            rows.append(tolerance_row(lr, m, label))
        del lr
        torch.cuda.empty_cache()
    add(wl.Layer("sq64", 64, 64, 64), "f16", "configs[0] 64^3 U[-1,1]", "uniform_pm1", "uniform_pm1", (B.GLOBAL, B.THREAD))
    add(wl.Layer("sq64", 64, 64, 64), "i8", "configs[0] 64^3 int8", modes=(B.GLOBAL,))
    for b in (1, 16, 256):
        add(wl.dlrm_layers(b)[4], "f16", f"configs[1] DLRM top1 batch {b}")
    for b in (1, 64):
        layers = wl.resnet50_layers(b)
        add(layers[0], "f16", f"configs[2] ResNet-50 conv1 batch {b}")
        add(layers[28], "f16", f"configs[2] ResNet-50 {layers[28].name} batch {b}")
        add(layers[-2], "f16", f"configs[2] ResNet-50 {layers[-2].name} batch {b}")
    for n, dts in ((4096, ("f16", "bf16")), (8192, ("f16", "bf16", "i8"))):
        for d in dts:
            add(wl.Layer(f"sq{n}", n, n, n), d, f"configs[3] {n}^3 N(0,1)", "normal", "normal")
    for m in (1, 256, 512, 8192):
        add(wl.Layer(f"m{m}", m, 4096, 4096), "f16", f"configs[4] M={m}, N=K=4096 N(0,1)", "normal", "normal")
    return rows


def noise_study(gen):
    """How large the clean residual of a comparison gets on this GPU, in the units the tolerance is
    written in: max over seeds and regions of |lhs - rhs| / (2^-24 sqrt(K) ||C_S||_F) (the random-walk
    part; the tolerance allows 8) and, for the global scheme, of |lhs - rhs| / (2^-24 K ||C_S||_1) (the
    same-sign drift; the tolerance adds 1e-3 of it).  From the device's own report of the worst region."""
    u = 2.0 ** -24
    out = []
    shapes = ((256, 256, 64), (256, 256, 1024), (1024, 1024, 1024), (1024, 1024, 8192), (4096, 4096, 4096),
              (2048, 2048, 16384), (8192, 8192, 8192))
    dists = (("normal", "normal"), ("uniform_pm1", "uniform_pm1"), ("uniform_01", "weights"), ("uniform_01", "uniform_01"))
    for dtype in ("f16", "bf16"):
        for da, db in dists:
            for (M, N, K) in shapes:
                seeds = 2 if M >= 4096 else 6
                for mode in (B.GLOBAL, B.THREAD):
                    walk = drift = ratio = 0.0
                    flags = 0
                    for sd in range(seeds):
                        lr = LayerRun(wl.Layer("n", M, N, K), dtype, gen, da, db)
                        rep, fl = _report_of(lr, mode)
                        res = abs(rep.lhs - rep.rhs)
                        walk = max(walk, res / (u * math.sqrt(K) * rep.frob) if rep.frob else 0.0)
                        if mode == B.GLOBAL and rep.l1:
                            drift = max(drift, res / (u * K * rep.l1))
                        ratio = max(ratio, rep.worst_ratio)
                        flags += fl
                        del lr
                    out.append({"dtype": dtype, "A": da, "B": db, "M": M, "N": N, "K": K, "scheme": B.MODE_NAMES[mode],
                                "residual_over_u_sqrtK_frob": round(walk, 3), "residual_over_u_K_l1": float(f"{drift:.3g}"),
                                "residual_over_tau": round(ratio, 3), "false_alarms": flags})
                    torch.cuda.empty_cache()
    return out


# --------------------------------------------------------------------------- #
def build_workload(name, gen):
    if name == "dlrm":
        return "configs[1]: DLRM MLPs (bottom 13-512-256-64, top 512-1024-1024-512-256-1), fp16, batch 256", \
            [LayerRun(l, "f16", gen) for l in wl.dlrm_layers(256)], "f16"
    if name == "resnet50":
        return "configs[2]: ResNet-50 53 conv layers as implicit GEMM, fp16, 224x224, batch 64", \
            [LayerRun(l, "f16", gen) for l in wl.resnet50_layers(64)], "f16"
    if name == "square":
        return "configs[3]: square GEMM M=N=K=8192, fp16 N(0,1)", \
            [LayerRun(wl.Layer("sq8192", 8192, 8192, 8192), "f16", gen, "normal", "normal")], "f16"
    raise SystemExit(f"unknown workload {name}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="square", choices=["dlrm", "resnet50", "square"])
    ap.add_argument("--noise-study", action="store_true",
                    help="only measure the clean residuals of the comparisons against the units of the tolerance "
                         "and print them as one JSON line")
    ap.add_argument("--no-extras", action="store_true", help="skip the short legs for the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--all-layers", action="store_true", help="print every row of the per-layer table")
    ap.add_argument("--probe", default=None, metavar="M,N,K[,DTYPE]",
                    help="only run one fully-connected layer of that shape ten times under every scheme (each scheme "
                         "is a kernel of its own name, so hardware counters of a profiler separate them) and print "
                         "the device times as one JSON line")
    ap.add_argument("--chain", default=None, metavar="M,WIDTH,LAYERS[,DTYPE]",
                    help="only run the chain leg for LAYERS fully-connected layers of WIDTH x WIDTH at batch M "
                         "(stand-alone layers against the chain with handed-over activation checksums) and print "
                         "it as one JSON line")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="first run 5 plain element-wise copy kernels that read MIB MiB and write MIB MiB each "
                         "(calibrates hardware byte counters under a profiler)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()  # fails loudly if libabft.so was not built
    torch.cuda.set_device(0)
    hip = Hip()
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(20210409)
    stream = torch.cuda.current_stream().cuda_stream or None

    if args.copy_probe > 0:
        src = torch.ones(args.copy_probe * (1 << 18), dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)  # one vectorized element-wise kernel: reads and writes MIB MiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.noise_study:
        print(json.dumps({"noise_study": noise_study(gen)}))
        return

    if args.chain:
        parts = args.chain.split(",")
        m, width, nl = (int(x) for x in parts[:3])
        print(json.dumps({"chain": handover_leg(gen, m, (width,) * (nl + 1), parts[3] if len(parts) > 3 else "f16", steps=20)}))
        return

    if args.probe:
        parts = args.probe.split(",")
        M, N, K = (int(x) for x in parts[:3])
        dt = parts[3] if len(parts) > 3 else "f16"
        lr = LayerRun(wl.Layer("probe", M, N, K), dt, gen, "normal", "normal")
        res = {"probe": [M, N, K, dt]}
        modes = [B.NONE, B.GLOBAL, B.THREAD, B.REPLICA] + ([] if dt == "i8" else [B.THREAD_HALF, B.TWOSIDED])
        for mode in modes:
            for _ in range(3):
                lr.run(mode, stream)
            torch.cuda.synchronize()
            e0, e1 = hip.event(), hip.event()
            hip.record(e0, stream)
            for _ in range(10):
                lr.run(mode, stream)
            hip.record(e1, stream)
            res["us_" + B.MODE_NAMES[mode]] = round(1e3 * hip.elapsed_ms(e0, e1) / 10, 2)
        res["false_alarms"] = int(lr.flag.item())
        print(json.dumps(res))
        return

    label, runs, dtype = build_workload(args.workload, gen)
    defaults = {"dlrm": (1000, 100), "resnet50": (20, 3), "square": (20, 3)}[args.workload]
    steps = args.steps if args.steps is not None else defaults[0]
    warmup = args.warmup if args.warmup is not None else defaults[1]

    # ---- per-layer table (also warms everything up and finds the dominant kernel)
    reps = 50 if args.workload == "dlrm" else 10
    rows = layer_table(hip, runs, reps, 3, stream)
    # the dominant kernel: the layer with the most algorithmic work against its own roofline
    dom_i = max(range(len(runs)), key=lambda i: max(runs[i].flops / PEAK[runs[i].dtype], runs[i].bytes / HBM))
    dom = runs[dom_i]

    # ---- a plan over the workload: per-layer scheme by the selector, offline weight checksums
    def plan_layer(lr):
        L = lr.layer
        conv = lr.conv if lr.conv is not None else B.Conv()
        return B.Layer(L.M, L.N, L.K, lr.dt, B.B_NK, 1 if lr.conv is not None else 0, conv, lr.B.data_ptr(), L.K)
    plan = B.abft_plan_create([plan_layer(lr) for lr in runs], profile=False)
    io = B.PlanIO([lr.A for lr in runs], [lr.layer.K for lr in runs], [lr.C for lr in runs],
                  [lr.layer.N for lr in runs])
    flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    assert [B.abft_plan_mode(plan, i) for i in range(len(runs))] == [lr.pick for lr in runs]

    # ---- the timed region: exactly `steps` protected passes, one library call per pass (the
    # library launches every layer's kernels back to back; this is faster than replaying a
    # captured graph of the same pass).  HIP events bracket the dominant layer's GEMM kernel
    # inside the library, on the stream it is launched on.
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    sp = side.cuda_stream

    def run_range(lo, hi):
        for i in range(lo, hi):
            B.abft_plan_run(plan, i, runs[i].A, runs[i].layer.K, runs[i].C, runs[i].layer.N, flag, sp)

    for _ in range(warmup):
        B.abft_plan_run_all(plan, io, flag, -1, stream)
    ev = [(hip.event(), hip.event()) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        B.abft_set_kernel_events(ev[s][0], ev[s][1])
        B.abft_plan_run_all(plan, io, flag, dom_i, stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    B.abft_set_kernel_events(None, None)
    ms_per_step = 1000.0 * wall / steps
    total_flops = sum(lr.flops for lr in runs)
    value = total_flops / (wall / steps) / 1e12
    flagged = int(flag.item())

    kern_us = float(np.mean([1000.0 * hip.elapsed_ms(a, b) for a, b in ev]))
    for a, b in ev:
        hip.destroy(a)
        hip.destroy(b)
    compute_bound = dom.ai > PEAK[dtype] / HBM
    if compute_bound:
        achieved = dom.flops / (kern_us * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK[dtype] / 1e12, "unit": "TFLOP/s",
                "frac": round(achieved / (PEAK[dtype] / 1e12), 4), "traffic": None}
    else:
        achieved = dom.bytes / (kern_us * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM / 1e9, "unit": "GB/s",
                "frac": round(achieved / (HBM / 1e9), 4), "traffic": None}
    tk = TRAFFIC_KIB.get((dom.layer.name, dom.layer.M, dom.layer.N, dom.layer.K, dtype, B.MODE_NAMES[dom.pick]))
    if tk is not None:
        roof["traffic"] = int((tk[0] * TRAFFIC_SCALE[0] + tk[1] * TRAFFIC_SCALE[1]) * 1024)
    # the dominant layer's whole call alone (its product kernel, plus the activation-checksum pass
    # where the global scheme runs one), replayed back to back from a graph (per-layer table): what a
    # kernel trace shows; the bracket in the timed region also holds the dispatch gap of an eager launch
    alone_us = rows[dom_i]["us_" + B.MODE_NAMES[dom.pick]]
    if tk is not None:
        roof["traffic_source"] = "looked up: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under profiles/ (not read in this run)"
    roof.update({"kernel": f"gemm_kernel[{B.MODE_NAMES[dom.pick]}] on {dom.layer.name} "
                           f"(M={dom.layer.M},N={dom.layer.N},K={dom.layer.K})",
                 "avg_launch_us": round(kern_us, 3),
                 "call_device_us": alone_us,
                 "achieved_call_device": round((dom.flops / 1e12 if compute_bound else dom.bytes / 1e9) / (alone_us * 1e-6), 2),
                 "frac_call_device": round((dom.flops / PEAK[dtype] if compute_bound else dom.bytes / HBM) / (alone_us * 1e-6), 4),
                 "algorithmic_per_launch": dom.flops if compute_bound else dom.bytes})

    # whole passes replayed from one graph each: protected (selector's picks), then unprotected
    # (same kernels, mode NONE) for the whole-model overhead; outside the timed region
    def graph_pass_ms():
        with torch.cuda.stream(side):
            run_range(0, len(runs))
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            run_range(0, len(runs))
        for _ in range(max(3, warmup // 10)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return 1000.0 * (time.perf_counter() - t0) / steps

    graph_ms = graph_none_ms = None
    try:
        graph_ms = graph_pass_ms()
        for i in range(len(runs)):
            B.abft_plan_set_mode(plan, i, B.NONE)
        graph_none_ms = graph_pass_ms()
    except Exception as e:  # reported, never fatal
        graph_ms = repr(e)
    # the unprotected pass launched like the timed region
    for i in range(len(runs)):
        B.abft_plan_set_mode(plan, i, B.NONE)
    for _ in range(warmup):
        B.abft_plan_run_all(plan, io, flag, -1, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.abft_plan_run_all(plan, io, flag, -1, stream)
    torch.cuda.synchronize()
    wall_none = time.perf_counter() - t0
    # the analytic selector with another scheme of the paper's design space standing in for the
    # exact one-sided checksum on the layers it assigns to the thread level (same granularity of
    # checks): replication with single accumulation (Sec. 5.1), the paper's own half-precision
    # one-sided checksum (Sec. 5.2.2) and two-sided ABFT (Sec. 5.2.1), the last two with their
    # widened tolerance
    def selector_with(thread_level_mode):
        try:
            for i, lr in enumerate(runs):
                B.abft_plan_set_mode(plan, i, thread_level_mode if lr.pick == B.THREAD else lr.pick)
            for _ in range(warmup):
                B.abft_plan_run_all(plan, io, flag, -1, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                B.abft_plan_run_all(plan, io, flag, -1, stream)
            torch.cuda.synchronize()
            wall_r = time.perf_counter() - t0
            return {"value": round(total_flops / (wall_r / steps) / 1e12, 3), "unit": "TFLOP/s",
                    "ms_per_step": round(1000.0 * wall_r / steps, 5),
                    "overhead_pct_whole_pass": round(100 * (wall_r / wall_none - 1), 2),
                    "false_alarms": int(flag.item())}
        except Exception as e:  # reported, never fatal
            return {"error": repr(e)}
    # the selector's own pass once more, launched as the unprotected pass was (no event bracket
    # around the dominant kernel: two event records per pass are a sixth of a DLRM pass)
    again = selector_with(B.THREAD)
    repl = selector_with(B.REPLICA)
    half = selector_with(B.THREAD_HALF) if dtype != "i8" else None
    twos = selector_with(B.TWOSIDED) if dtype != "i8" else None
    for i in range(len(runs)):
        B.abft_plan_set_mode(plan, i, B.AUTO)
    B.abft_plan_destroy(plan)

    # the paper's own selection procedure (Sec. 5.3: profile both schemes per layer before
    # deployment, keep the faster): a second plan made that way, timed like the first
    prof = None
    try:
        plan2 = B.abft_plan_create([plan_layer(lr) for lr in runs], profile=True)
        picks2 = [B.abft_plan_mode(plan2, i) for i in range(len(runs))]
        for _ in range(warmup):
            B.abft_plan_run_all(plan2, io, flag, -1, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            B.abft_plan_run_all(plan2, io, flag, -1, stream)
        torch.cuda.synchronize()
        wall2 = time.perf_counter() - t0
        B.abft_plan_destroy(plan2)
        prof = {"value": round(total_flops / (wall2 / steps) / 1e12, 3), "unit": "TFLOP/s",
                "ms_per_step": round(1000.0 * wall2 / steps, 5),
                "overhead_pct_whole_pass": round(100 * (wall2 / wall_none - 1), 2),
                "modes_picked": {m: sum(1 for x in picks2 if B.MODE_NAMES[x] == m) for m in ("global", "thread")},
                # where the analytic rule and the profile disagree (device times from the layer table)
                "disagrees_with_analytic": [
                    {"layer": r["layer"], "ai": r["ai"], "analytic": r["pick"], "profiled": B.MODE_NAMES[x],
                     "us_global": r["us_global"], "us_thread": r["us_thread"]}
                    for r, x in zip(rows, picks2) if B.MODE_NAMES[x] != r["pick"]][:12],
                "n_disagree": sum(1 for r, x in zip(rows, picks2) if B.MODE_NAMES[x] != r["pick"])}
    except Exception as e:  # reported, never fatal
        prof = {"error": repr(e)}

    out = {
        "metric": "protected GEMM TFLOP/s and ABFT overhead % vs unprotected MFMA GEMM per layer",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": label, "layers": len(runs), "selector": "analytic (AI vs CMR)",
                   "modes_picked": {m: sum(1 for lr in runs if B.MODE_NAMES[lr.pick] == m) for m in ("global", "thread")}},
        "launch": "one abft_plan_run_all call per pass",
        "overhead_pct_whole_pass": round(100 * (wall / wall_none - 1), 2),
        "overhead_pct_whole_pass_without_event_bracket": again.get("overhead_pct_whole_pass"),
        "overhead_pct_summed_layers": summarize(rows)["ovh_selector_pct"],
        "false_alarms": flagged,
        "profiled_selector": prof,
        "analytic_selector_with_replication_at_thread_level": repl,
        "analytic_selector_with_half_precision_checksum_at_thread_level": half,
        "analytic_selector_with_two_sided_checksum_at_thread_level": twos,
        "graph_replay": None if not isinstance(graph_ms, float) else {
            "ms_per_step": round(graph_ms, 5), "tflops": round(total_flops / (graph_ms * 1e-3) / 1e12, 3),
            "unprotected_ms_per_step": None if graph_none_ms is None else round(graph_none_ms, 5)},
        "graph_replay_error": graph_ms if isinstance(graph_ms, str) else None,
        "roofline": roof,
        "tolerance": None,
        "summary": summarize(rows),
        "layers": rows if (len(rows) <= 16 or args.all_layers) else rows[:3] + [{"...": f"{len(rows) - 6} more"}] + rows[-3:],
        "paper_context": "NVIDIA T4, FP16: DLRM MLP-Bottom/Top batch 1 overhead 5.16/5.61 % (intensity-guided) vs "
                         "23.50/18.16 % (global); ResNet-50 HD 4.21 % vs 8.49 %; square 2048^3 global 1 %, thread 14 %",
    }

    try:
        out["tolerance"] = tolerance_leg(gen)
    except Exception as e:  # reported, never fatal
        out["tolerance"] = {"error": repr(e)}

    if not args.no_extras:
        extra = {}
        try:
            for n, dts in ((4096, ("f16", "bf16")), (8192, ("f16", "bf16", "i8"))):
                for d in dts:
                    if args.workload == "square" and (n, d) == (8192, "f16"):
                        continue   # the headline itself
                    if True:
                        lr = LayerRun(wl.Layer(f"sq{n}", n, n, n), d, gen, "normal", "normal")
                        r = layer_table(hip, [lr], 20 if n <= 4096 else 10, 3, stream)[0]
                        extra[f"square{n}_{d}"] = {k: r[k] for k in ("pick", "us_none", "ovh_global_pct", "ovh_thread_pct",
                                                                      "tflops_pick", "roofline_frac_pick")}
                        del lr
                        torch.cuda.empty_cache()
            if args.workload != "dlrm":
                for b in (1, 16, 256):
                    rs = [LayerRun(l, "f16", gen) for l in wl.dlrm_layers(b)]
                    extra[f"dlrm_b{b}"] = summarize(layer_table(hip, rs, 50, 3, stream))
            else:
                for b in (1, 16):
                    rs = [LayerRun(l, "f16", gen) for l in wl.dlrm_layers(b)]
                    extra[f"dlrm_b{b}"] = summarize(layer_table(hip, rs, 50, 3, stream))
            if args.workload != "resnet50":
                for b in (1, 64):
                    rs = [LayerRun(l, "f16", gen) for l in wl.resnet50_layers(b)]
                    extra[f"resnet50_b{b}"] = summarize(layer_table(hip, rs, 5, 2, stream))
                    del rs
                    torch.cuda.empty_cache()
            sweep = []
            for m in wl.sweep_m():
                lr = LayerRun(wl.Layer(f"m{m}", m, 4096, 4096), "f16", gen, "normal", "normal")
                r = layer_table(hip, [lr], 10, 2, stream, modes=(B.NONE, B.GLOBAL, B.THREAD, B.THREAD_HALF, B.TWOSIDED))[0]
                sweep.append({k: r[k] for k in ("M", "ai", "pick", "us_none", "ovh_global_pct", "ovh_thread_pct",
                                                "ovh_thread_half_pct", "ovh_twosided_pct")})
            extra["sweep_N4096_K4096"] = sweep
            # the paper's Fig. 11 sizes (its T4 numbers: thread-level 2-14 %, global 27 % at 32^3 down to 1 % at 2048^3,
            # replication above 70 % at the two largest sizes)
            fig11 = []
            for n in wl.square_sizes_paper():
                lr = LayerRun(wl.Layer(f"sq{n}", n, n, n), "f16", gen, "normal", "normal")
                r = layer_table(hip, [lr], 20, 2, stream, modes=(B.NONE, B.GLOBAL, B.THREAD, B.REPLICA, B.THREAD_HALF, B.TWOSIDED))[0]
                fig11.append({k: r[k] for k in ("M", "ai", "pick", "us_none", "ovh_global_pct", "ovh_thread_pct",
                                                "ovh_replica_pct", "ovh_thread_half_pct", "ovh_twosided_pct")})
            extra["squares_fig11"] = fig11
            extra["measured_ceilings"] = measured_ceilings(hip, gen)
            extra["dlrm_mlp_chains_relu"] = [chain_leg(gen, b) for b in (1, 16, 256)]
            extra["midsize_chain_handed_over_checksums"] = [
                handover_leg(gen, m, w, dt) for m, w, dt in ((1024, (4096,) * 5, "f16"), (2048, (4096,) * 5, "f16"),
                                                             (4096, (4096,) * 5, "f16"), (2048, (2048,) * 5, "f16"),
                                                             (2048, (4096,) * 5, "bf16"))]
            extra["selector_study_fp16_bf16"] = selector_study(ALL_ROWS)
            extra["dlrm_top1_cold_cache"] = cold_cache_leg(wl.Layer("top1", 256, 1024, 1024), "f16", gen)
        except Exception as e:  # extras never invalidate the main measurement
            extra["error"] = repr(e)
        out["extra"] = extra

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(runs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
