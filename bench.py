#!/usr/bin/env python3
"""Benchmark of the 2:4-sparse convolution on one MI355X.

A step is one launch of ss_conv2d_fwd (implicit unfold + sparse contraction + fused bias/ReLU
epilogue) on the ResNet-50-style 3x3 layer (N=32, 256->256, 14x14, fp16), with every operand
already resident in device memory; the weight compressor is a one-off per weight update and is
timed separately.  The dense twin is timed the same way for the speed-up ratio, and the CPU
oracle is timed on the host cores as a reported baseline.  Prints ONE JSON line; beside the
headline it carries the rest of the protocol ("protocol": configs[0] latency, configs[2]
bandwidth, cold-cache points, per-layer sums of configs[3] and configs[4]) and the rate against
the issue peak measured in the same run.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--table | --tail | --trunk | --fused | --q8 | --probes]
        --table  per-layer report of configs 0-2, the ResNet-50 stack and ConvNeXt-T stage 1 (--cold, --only)
        --tail   the fused residual / activation tail against a separate pass
        --trunk  the ResNet-50 convolution trunk chained in one HIP graph, images/s
        --fused  a k x k convolution and the 1x1 after it (or the two 1x1 of a ConvNeXt block) in one kernel
        --q8     the int8 / FP8 precision points
        --probes calibration: register-only issue rate of the matrix instructions, LDS bandwidth of a compute unit
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

import numpy as np

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

SPARSE_PEAK_TFLOPS = 5000.0   # 2:4-sparse fp16/bf16 MFMA, dense-equivalent = 2 x the 2.5 PFLOP/s dense peak
DENSE_PEAK_TFLOPS = 2500.0
SPARSE_INT8_PEAK_TOPS = 10000.0     # 2 x the published dense int8 peak (5.0 POP/s), dense-equivalent
HBM_PEAK_GBS = 8000.0
# Memory-side bytes per launch of the sparse kernel on configs[1], from the rocprofv3 counter runs summarised in
# profiles/conv_kernel_hbm_traffic.md: 2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE (factors from a streaming copy).
CFG1_TRAFFIC_BYTES = int((2.0 * 4336.1 + 1.0 * 3136.0) * 1024)


def _to_dev(bits, dtype, torch, ss):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(ss.torch_dtype(dtype))


class LayerRun:
    """Device-resident operands of one layer and closures that launch the sparse / dense path."""

    def __init__(self, L, torch, ss, wl, copies: int = 1, values: bool = True):
        self.L = L
        self.desc = ss.make_desc(L.cout, L.cin, L.kh, L.kw, L.dtype, L.korder)
        tdt = ss.torch_dtype(L.dtype)
        if values:
            d = wl.make_inputs(L)
            self.host = d
            W = _to_dev(d["W"], L.dtype, torch, ss)
            M = None if d["M"] is None else torch.from_numpy(d["M"]).cuda()
            x0 = _to_dev(d["x"], L.dtype, torch, ss)
            self.bias = torch.from_numpy(d["bias"]).cuda()
        else:   # timing only: shapes and value distribution matter, not the exact draw
            g = torch.Generator(device="cuda").manual_seed(L.seed)
            W = (torch.randn((L.cout, L.K), generator=g, device="cuda") * (2.0 / L.K) ** 0.5).to(tdt)
            M = None
            if L.mask != "none":
                pat = torch.tensor([[1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 0, 1], [0, 1, 1, 0], [0, 1, 0, 1], [0, 0, 1, 1]],
                                   dtype=torch.uint8, device="cuda")
                M = pat[torch.randint(0, 6, (L.cout, L.K // 4), generator=g, device="cuda")].reshape(L.cout, L.K).contiguous()
            x0 = torch.randn((L.N, L.H, L.W, L.cin), generator=g, device="cuda")
            x0 = (x0.clamp_(min=0) if L.relu_input else x0).to(tdt)
            self.bias = torch.randn(L.cout, generator=g, device="cuda") * 0.1
        self.W, self.M = W, M
        self.packed = ss.ss_mask_compress(self.desc, W, M) if M is not None else None
        self.dense = ss.ss_dense_pack(self.desc, W, M)
        self.xs = [x0] + [x0.clone() for _ in range(copies - 1)]
        st, pd = (L.stride,) * 2, (L.pad,) * 2
        self.calls_s, self.calls_d, self.ys = [], [], []
        for xi in self.xs:
            cd, y = ss.prepare_conv2d(self.desc, xi, self.dense, self.bias, st, pd, L.act, sparse=False)
            self.calls_d.append(cd)
            self.ys.append(y)
            if self.packed is not None:
                cs, _ = ss.prepare_conv2d(self.desc, xi, self.packed, self.bias, st, pd, L.act, y=y, sparse=True)
                self.calls_s.append(cs)
        self.i = 0

    def sparse(self):
        self.i = (self.i + 1) % len(self.xs)
        self.calls_s[self.i]()

    def densef(self):
        self.i = (self.i + 1) % len(self.xs)
        self.calls_d[self.i]()


class Q8Run:
    """The 8-bit variant of a layer (channels-last flattening), int8 or FP8 E4M3: device operands drawn on the GPU
    for timing (weights ~ N(0, 40) and activations ReLU(N(0, 32)), clipped and cast; random 2:4 patterns; a
    per-channel scale)."""

    def __init__(self, L, torch, ss, wl, dtype=None, korder=None):
        self.L = L
        dtype = ss.SS_I8 if dtype is None else dtype
        if korder is None:
            korder = wl.K_RSC if L.kh * L.kw > 1 else L.korder
        self.desc = ss.make_desc(L.cout, L.cin, L.kh, L.kw, dtype, korder)
        g = torch.Generator(device="cuda").manual_seed(L.seed)

        def cast(t):
            if dtype == ss.SS_I8:
                return t.clamp_(-127, 127).round_().to(torch.int8)
            return t.clamp_(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8)
        W = cast(torch.randn((L.cout, L.K), generator=g, device="cuda") * 40)
        pat = torch.tensor([[1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 0, 1], [0, 1, 1, 0], [0, 1, 0, 1], [0, 0, 1, 1]],
                           dtype=torch.uint8, device="cuda")
        M = pat[torch.randint(0, 6, (L.cout, L.K // 4), generator=g, device="cuda")].reshape(L.cout, L.K).contiguous()
        x = torch.randn((L.N, L.H, L.W, L.cin), generator=g, device="cuda") * 32
        x = cast(x.clamp_(min=0) if L.relu_input else x)
        self.scale = torch.full((L.cout,), 1.0 / (40 * 32 * (L.K / 2) ** 0.5), device="cuda")
        self.bias = torch.randn(L.cout, generator=g, device="cuda") * 0.1
        self.packed = ss.ss_mask_compress(self.desc, W, M)
        self.dense = ss.ss_dense_pack(self.desc, W, M)
        st, pd = (L.stride,) * 2, (L.pad,) * 2
        self.densef, self.y = ss.prepare_conv2d_q8(self.desc, x, self.dense, self.scale, self.bias, st, pd, L.act, sparse=False)
        self.sparse, _ = ss.prepare_conv2d_q8(self.desc, x, self.packed, self.scale, self.bias, st, pd, L.act, y=self.y)
        self.keep = (W, M, x)


def q8_point(torch, ss, wl, L, steps, warmup, reps=3, dtype=None, korder=None):
    """Sparse / dense-twin time of the 8-bit variant of a layer and its rate in dense-equivalent TOP/s (the published
    dense peaks of int8 and fp8 are the same, 5.0 P/s, so one sparse peak serves both)."""
    run = Q8Run(L, torch, ss, wl, dtype, korder)
    ts = median_time(torch, run.sparse, steps, warmup, reps=reps)
    td = median_time(torch, run.densef, steps, warmup, reps=reps)
    tops = L.dense_equiv_flop / ts / 1e9
    return {"sparse_us": ts * 1e3, "dense_twin_us": td * 1e3, "speedup": td / ts, "tops": tops,
            "frac_sparse_8bit_peak": tops / SPARSE_INT8_PEAK_TOPS}


def print_q8_table(torch, ss, wl, steps, warmup):
    """8-bit integer variants of the benchmark layers and of the masked ResNet-50 layers (batch 64), next to the
    16-bit path on the same shape (channels-last flattening for both, so the comparison is like for like)."""
    import dataclasses
    layers = [wl.CONFIG1, wl.with_batch(wl.CONFIG1, 500), wl.with_batch(wl.CONFIG1, 512), wl.CONFIG2]
    layers += [L for L in wl.resnet50_layers(64) if L.mask != "none" and L.cin % 16 == 0]
    print(f"{'layer':34s} {'N':>4s} {'int8 us':>9s} {'twin us':>9s} {'x':>5s} {'TOP/s':>8s} {'16-bit us':>10s} {'int8 gain':>9s}"
          f" {'fp8 us':>8s} {'twin us':>8s} {'x':>5s}")
    tot8 = tot16 = totd = totf = totfd = 0.0
    for i, L in enumerate(layers):
        r = q8_point(torch, ss, wl, L, steps, warmup)
        rf = q8_point(torch, ss, wl, L, steps, warmup, dtype=ss.SS_F8)
        L16 = dataclasses.replace(L, korder=wl.K_RSC if L.kh * L.kw > 1 else L.korder)
        run16 = LayerRun(L16, torch, ss, wl, values=False)
        t16 = median_time(torch, run16.sparse, steps, warmup, reps=3) * 1e3
        del run16
        print(f"{L.name:34s} {L.N:4d} {r['sparse_us']:9.1f} {r['dense_twin_us']:9.1f} {r['speedup']:5.2f} {r['tops']:8.0f} "
              f"{t16:10.1f} {t16 / r['sparse_us']:9.2f} {rf['sparse_us']:8.1f} {rf['dense_twin_us']:8.1f} {rf['speedup']:5.2f}", flush=True)
        if i < 3:       # the benchmark layer in the paper's own flattening (taps inside a block: byte transpose)
            rc = q8_point(torch, ss, wl, L, steps, warmup, korder=wl.K_CRS)
            rfc = q8_point(torch, ss, wl, L, steps, warmup, dtype=ss.SS_F8, korder=wl.K_CRS)
            print(f"{'  ... channel-slowest flattening':34s} {L.N:4d} {rc['sparse_us']:9.1f} {rc['dense_twin_us']:9.1f} {rc['speedup']:5.2f} "
                  f"{rc['tops']:8.0f} {'':>10s} {'':>9s} {rfc['sparse_us']:8.1f} {rfc['dense_twin_us']:8.1f} {rfc['speedup']:5.2f}", flush=True)
        if i >= 4:      # the ResNet-50 layers
            tot8 += r["sparse_us"] * L.count
            totd += r["dense_twin_us"] * L.count
            tot16 += t16 * L.count
            totf += rf["sparse_us"] * L.count
            totfd += rf["dense_twin_us"] * L.count
    print(f"ResNet-50 masked layers, batch 64: int8 sparse {tot8 / 1e3:.3f} ms, int8 dense twin {totd / 1e3:.3f} ms, "
          f"16-bit sparse {tot16 / 1e3:.3f} ms, fp8 sparse {totf / 1e3:.3f} ms, fp8 dense twin {totfd / 1e3:.3f} ms")


def time_graph(torch, fn, steps: int, warmup: int) -> float:
    """Milliseconds per launch with the `steps` launches captured in one HIP graph, so that the
    host's launch rate does not bound a kernel that runs for a few microseconds."""
    for _ in range(max(warmup, 1)):
        fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for _ in range(steps):
                fn()
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    time_graph.last_wall_ms = wall_ms / steps
    return e0.elapsed_time(e1) / steps


def time_launches(torch, fn, steps: int, warmup: int) -> float:
    """Milliseconds per launch: `steps` back-to-back launches between two events on the launch stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def median_time(torch, fn, steps, warmup, reps=5, graph=True):
    timer = time_graph if graph else time_launches
    return float(np.median([timer(torch, fn, steps, warmup if r == 0 else 2) for r in range(reps)]))


def cpu_baseline(L, wl, min_seconds: float = 10.0, max_runs: int = 200):
    """The oracle as it stands, timed on the host cores on the same workload: the full layer, repeated until about ten
    seconds of CPU work have been spent (one run of configs[1] takes a fraction of a second), rate over all runs."""
    import oracle
    d = wl.make_inputs(L)
    runs, total = 0, 0.0
    while runs < max_runs and (runs == 0 or total < min_seconds):
        t0 = time.perf_counter()
        oracle.conv2d(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, dtype=L.dtype,
                      bias=d["bias"], stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act)
        total += time.perf_counter() - t0
        runs += 1
    return {"value": L.dense_equiv_flop * runs / total / 1e12, "unit": "TFLOP/s (dense-equivalent)", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": total, "runs": runs,
            "sample": f"the full workload ({L.name}: all {L.P * L.cout} outputs) x {runs} runs ({total:.1f} s of wall time), fp64 direct convolution"}


def layer_report(torch, ss, wl, L, steps, warmup, cold=False):
    copies = 1
    if cold:   # rotate through > 512 MB of distinct activations so nothing stays cache-resident
        per = 2 * L.N * L.H * L.W * L.cin + 2 * L.P * L.cout
        copies = max(2, min(64, int(600e6 // per) + 1))
    run = LayerRun(L, torch, ss, wl, copies=copies, values=False)
    out = {"layer": L.name, "count": L.count, "gflop": L.dense_equiv_flop / 1e9, "masked": L.mask != "none"}
    td = median_time(torch, run.densef, steps, warmup, reps=3)
    out["dense_us"] = td * 1e3
    if L.mask != "none":
        ts = median_time(torch, run.sparse, steps, warmup, reps=3)
        out["sparse_us"] = ts * 1e3
        out["speedup"] = td / ts
        out["tflops"] = L.dense_equiv_flop / ts / 1e9
        out["gbs"] = L.algorithmic_bytes(True) / ts / 1e6
        out["t_floor_us"] = max(L.dense_equiv_flop / SPARSE_PEAK_TFLOPS / 1e6, L.algorithmic_bytes(True) / HBM_PEAK_GBS / 1e3)
    else:
        out["tflops"] = L.dense_equiv_flop / td / 1e9
        out["gbs"] = L.algorithmic_bytes(False) / td / 1e6
        out["t_floor_us"] = max(L.dense_equiv_flop / DENSE_PEAK_TFLOPS / 1e6, L.algorithmic_bytes(False) / HBM_PEAK_GBS / 1e3)
    del run
    torch.cuda.empty_cache()
    return out


def print_table(torch, ss, wl, steps, warmup, cold, only=""):
    rows = []
    groups = [("configs 0-2", [wl.CONFIG0, wl.CONFIG1, wl.CONFIG2]), ("ResNet-50 conv stack, batch 64, bf16", wl.resnet50_layers()),
              ("ConvNeXt-T stage 1, batch 128, bf16", wl.convnext_t_stage1_layers())]
    for title, layers in groups:
        layers = [L for L in layers if only in L.name]
        if not layers:
            continue
        print(f"## {title}" + (" (cold: rotating buffers)" if cold else " (warm: buffers reused)"), flush=True)
        print(f"{'layer':34s} {'x':>2s} {'GFLOP':>8s} {'sparse us':>10s} {'dense us':>9s} {'speedup':>7s} {'TFLOP/s':>8s} {'GB/s':>7s} {'floor us':>8s} {'frac':>5s}")
        tot_s = tot_d = tot_f = 0.0
        for L in layers:
            r = layer_report(torch, ss, wl, L, steps, warmup, cold)
            rows.append(r)
            t_used = r.get("sparse_us", r["dense_us"])
            tot_s += L.count * t_used
            tot_d += L.count * r["dense_us"]
            tot_f += L.count * r["t_floor_us"]
            print(f"{L.name:34s} {L.count:2d} {r['gflop']:8.2f} {r.get('sparse_us', float('nan')):10.2f} {r['dense_us']:9.2f} "
                  f"{r.get('speedup', float('nan')):7.2f} {r['tflops']:8.1f} {r['gbs']:7.0f} {r['t_floor_us']:8.2f} {r['t_floor_us'] / t_used:5.2f}", flush=True)
        print(f"{'total (x count)':34s}    {'':8s} {tot_s:10.1f} {tot_d:9.1f} {tot_d / tot_s:7.2f} {'':8s} {'':7s} {tot_f:8.1f} {tot_f / tot_s:5.2f}", flush=True)
        if "ConvNeXt" in title and (not only or only in "cnx_dw_7x7_96"):
            # the block's grouped convolution stays dense in the paper and runs through the dedicated depthwise kernel
            N, H, C = layers[0].N, layers[0].H, 96
            x = torch.randn((N, H, H, C), device="cuda").to(torch.bfloat16)
            w = (torch.randn((7, 7, C), device="cuda") * (2.0 / 49) ** 0.5).to(torch.bfloat16)
            b = torch.randn(C, device="cuda") * 0.1
            y = torch.empty_like(x)
            t = median_time(torch, lambda: ss.ss_dwconv2d_fwd(x, w, b, (3, 3), y=y), steps, warmup, reps=3) * 1e3
            nbytes, flop = 2 * x.numel() * 2, 2.0 * x.numel() * 49
            print(f"{'cnx_dw_7x7_96 (dense, depthwise)':34s} {3:2d} {flop / 1e9:8.2f} {'':>10s} {t:9.2f} {'':>7s} {flop / t / 1e6:8.1f} "
                  f"{nbytes / t / 1e3:7.0f} {nbytes / HBM_PEAK_GBS / 1e3:8.2f} {nbytes / HBM_PEAK_GBS / 1e3 / t:5.2f}", flush=True)
    return rows


def print_tail_table(torch, ss, wl, steps, warmup):
    """Fused layer tail (conv + bias + residual, activation, one rounding) against the same conv followed by a
    separate elementwise pass over the output, on the layers that close a residual block."""
    import dataclasses
    res_layers = [L for L in wl.resnet50_layers() if "_c3_" in L.name]
    cnx = {L.name: L for L in wl.convnext_t_stage1_layers()}
    cases = [(dataclasses.replace(L, act=wl.ACT_RELU), True) for L in res_layers]
    cases += [(dataclasses.replace(cnx["cnx_pw_96_384"], act=wl.ACT_GELU), False),       # expansion: GELU, no residual
              (dataclasses.replace(cnx["cnx_pw_384_96"], act=wl.ACT_NONE), True)]        # projection: + block input
    print("## fused tail: y = act(conv + bias + residual) in one kernel vs conv, then a separate add / activation pass")
    print(f"{'layer':24s} {'act':>5s} {'res':>4s} {'conv only us':>12s} {'fused us':>9s} {'separate us':>12s} {'saved us':>9s} {'fused GB/s':>10s}")
    names = {wl.ACT_NONE: "none", wl.ACT_RELU: "relu", wl.ACT_GELU: "gelu"}
    for L, with_res in cases:
        run = LayerRun(dataclasses.replace(L, act=wl.ACT_NONE), torch, ss, wl, values=False)
        x, y = run.xs[0], run.ys[0]
        r = torch.randn_like(y) if with_res else None
        st, pd = (L.stride,) * 2, (L.pad,) * 2
        fused, y2 = ss.prepare_conv2d(run.desc, x, run.packed, run.bias, st, pd, L.act, sparse=True, residual=r)

        def separate():
            run.calls_s[0]()
            if r is not None:
                y.add_(r)
            if L.act == wl.ACT_RELU:
                y.relu_()
            elif L.act == wl.ACT_GELU:
                y.copy_(torch.nn.functional.gelu(y))
        t_conv = median_time(torch, run.calls_s[0], steps, warmup) * 1e3
        t_fused = median_time(torch, fused, steps, warmup) * 1e3
        t_sep = median_time(torch, separate, steps, warmup) * 1e3
        nbytes = L.algorithmic_bytes(True) + (y.numel() * 2 if with_res else 0)
        print(f"{L.name:24s} {names[L.act]:>5s} {'yes' if with_res else 'no':>4s} {t_conv:12.2f} {t_fused:9.2f} {t_sep:12.2f} "
              f"{t_sep - t_fused:9.2f} {nbytes / t_fused / 1e3:10.0f}", flush=True)
        del run, fused, y2, r
        torch.cuda.empty_cache()


def print_fused_table(torch, ss, wl, steps, warmup, batch=64):
    """The 3x3 -> 1x1 (+ residual, ReLU) pairs of the ResNet-50 bottlenecks: one fused kernel against the two separate
    calls (the second with its fused tail), sparse path and dense twin."""
    import dataclasses
    layers = {L.name: L for L in wl.resnet50_layers(batch)}
    layers.update({L.name: L for L in wl.convnext_t_stage1_layers()})
    # (first layer, second layer, activation after the first, activation after the second + residual)
    pairs = [("s1_c2_3x3_64_64", "s1_c3_1x1_64_256", wl.ACT_RELU, wl.ACT_RELU),
             ("s2_c2_3x3_128_128", "s2_c3_1x1_128_512", wl.ACT_RELU, wl.ACT_RELU),
             ("s2_c2_3x3_128_128_s2", "s2_c3_1x1_128_512", wl.ACT_RELU, wl.ACT_RELU),
             ("s3_c2_3x3_256_256", "s3_c3_1x1_256_1024", wl.ACT_RELU, wl.ACT_RELU),
             ("s3_c2_3x3_256_256_s2", "s3_c3_1x1_256_1024", wl.ACT_RELU, wl.ACT_RELU),
             ("cnx_pw_96_384", "cnx_pw_384_96", wl.ACT_GELU, wl.ACT_NONE)]      # the ConvNeXt block's inverted bottleneck, batch 128
    print(f"{'pair':44s} {'fused us':>9s} {'separate us':>12s} {'gain':>6s} {'twin fused':>11s} {'twin separate':>14s}")
    for n1, n2, act1, act2 in pairs:
        L1, L2 = layers[n1], layers[n2]
        tdt = ss.torch_dtype(L1.dtype)
        g = torch.Generator(device="cuda").manual_seed(1)
        pat = torch.tensor([[1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 0, 1], [0, 1, 1, 0], [0, 1, 0, 1], [0, 0, 1, 1]], dtype=torch.uint8, device="cuda")

        def weights(L):
            W = (torch.randn((L.cout, L.K), generator=g, device="cuda") * (2.0 / L.K) ** 0.5).to(tdt)
            M = pat[torch.randint(0, 6, (L.cout, L.K // 4), generator=g, device="cuda")].reshape(L.cout, L.K).contiguous()
            d = ss.make_desc(L.cout, L.cin, L.kh, L.kw, L.dtype, L.korder)
            return d, ss.ss_mask_compress(d, W, M), ss.ss_dense_pack(d, W, M), torch.randn(L.cout, generator=g, device="cuda") * 0.1
        d1, p1, q1, b1 = weights(L1)
        d2, p2, q2, b2 = weights(L2)
        x = torch.randn((L1.N, L1.H, L1.W, L1.cin), generator=g, device="cuda").clamp_(min=0).to(tdt)
        res = torch.randn((L1.N, L1.Ho, L1.Wo, L2.cout), generator=g, device="cuda").to(tdt)
        st, pd = (L1.stride,) * 2, (L1.pad,) * 2
        out = {}
        for sparse, w1, w2 in ((True, p1, p2), (False, q1, q2)):
            fused, _ = ss.prepare_conv2d_pw_fused(d1, x, w1, b1, st, pd, act1, d2, w2, b2, res, act2, sparse=sparse)
            c1, t = ss.prepare_conv2d(d1, x, w1, b1, st, pd, act1, sparse=sparse)
            c2, _ = ss.prepare_conv2d(d2, t, w2, b2, (1, 1), (0, 0), act2, sparse=sparse, residual=res)

            def separate():
                c1()
                c2()
            out[sparse] = (median_time(torch, fused, steps, warmup, reps=3) * 1e3, median_time(torch, separate, steps, warmup, reps=3) * 1e3)
        print(f"{n1 + ' -> ' + n2:44s} {out[True][0]:9.1f} {out[True][1]:12.1f} {out[True][1] / out[True][0]:6.2f} "
              f"{out[False][0]:11.1f} {out[False][1]:14.1f}", flush=True)


def print_trunk(torch, ss, wl, batch=64, image=224):
    """End-to-end ResNet-50 convolution trunk (53 convolutions + max pool, real dataflow, fused residual tails),
    replayed as one HIP graph: images per second on the sparse path and on the dense twin."""
    from paper_2411_00288_amd import resnet50
    print(f"## ResNet-50 convolution trunk, batch {batch}, {image}x{image} (+ a zero fourth channel), bf16, synthetic weights: stem (dense) -> max pool -> "
          "16 bottlenecks; 48 convolutions 2:4-masked, stem and 4 shortcut convolutions dense; add + ReLU fused into conv3; "
          "3x3 + conv3 of the first two stages in one kernel")
    for sparse in (True, False):
        t = resnet50.Trunk(batch=batch, image=image, dtype=wl.BF16, sparse=sparse)
        t.input.copy_(torch.randn(t.input.shape, device="cuda").to(torch.bfloat16))
        t.input[..., 3:] = 0
        ms = median_time(torch, t.forward, 5, 2, reps=5)
        stem = median_time(torch, t.launches[0], 20, 3, reps=3)
        print(f"{'2:4 sparse path' if sparse else 'dense twin     '}: {ms:8.3f} ms per batch  {batch / ms * 1e3:9.0f} images/s  "
              f"{t.dense_equiv_flop() / ms / 1e9:7.1f} TFLOP/s dense-equivalent   (stem alone {stem * 1e3:6.1f} us)", flush=True)
        del t
        torch.cuda.empty_cache()


def single_launch_us(torch, fn, reps=50):
    """Latency of one isolated launch: device idle before, event pair around the launch, median over `reps`."""
    ts = []
    for _ in range(reps):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3)
    return float(np.median(ts))


def protocol_report(torch, ss, wl, steps, warmup):
    """The rest of the measurement protocol beside the headline layer: configs[0] latency, configs[2] bandwidth, cold
    points, and the per-layer sums of configs[3] (ResNet-50 convolutions, batch 64) and configs[4] (ConvNeXt-T stage
    1, batch 128) against their roofline floors."""
    out = {}
    run0 = LayerRun(wl.CONFIG0, torch, ss, wl, values=False)
    out["configs0"] = {"workload": wl.CONFIG0.name, "graph_us": median_time(torch, run0.sparse, steps, warmup, reps=3) * 1e3,
                       "single_launch_us": single_launch_us(torch, run0.sparse),
                       "dense_twin_graph_us": median_time(torch, run0.densef, steps, warmup, reps=3) * 1e3}
    del run0
    r2 = layer_report(torch, ss, wl, wl.CONFIG2, steps, warmup)
    out["configs2"] = {"workload": wl.CONFIG2.name, "sparse_us": r2["sparse_us"], "dense_twin_us": r2["dense_us"],
                       "speedup": r2["speedup"], "algorithmic_gbs": r2["gbs"], "frac_hbm_peak": r2["gbs"] / HBM_PEAK_GBS,
                       "tflops": r2["tflops"], "floor_us": r2["t_floor_us"]}
    cold = {}
    for name, L in (("configs1", wl.CONFIG1), ("configs2", wl.CONFIG2)):
        r = layer_report(torch, ss, wl, L, min(steps, 128), min(warmup, 20), cold=True)
        cold[name] = {"sparse_us": r["sparse_us"], "dense_twin_us": r["dense_us"], "algorithmic_gbs": r["gbs"], "tflops": r["tflops"]}
    out["cold"] = dict(cold, note="rotating through more than 512 MB of distinct activation / output buffers")
    for key, title, layers in (("configs3", "ResNet-50 convolutions, batch 64, bf16, each layer on its own buffers", wl.resnet50_layers()),
                               ("configs4", "ConvNeXt-T stage 1 masked layers, batch 128, bf16", wl.convnext_t_stage1_layers())):
        tot_s = tot_d = tot_f = 0.0
        per = []
        for L in layers:
            r = layer_report(torch, ss, wl, L, min(steps, 50), min(warmup, 10))
            t_used = r.get("sparse_us", r["dense_us"])
            tot_s += L.count * t_used
            tot_d += L.count * r["dense_us"]
            tot_f += L.count * r["t_floor_us"]
            per.append({"layer": L.name, "count": L.count, "us": round(t_used, 2), "dense_twin_us": round(r["dense_us"], 2),
                        "floor_us": round(r["t_floor_us"], 2), "gbs": round(r["gbs"]), "tflops": round(r["tflops"], 1)})
        out[key] = {"workload": title, "sum_sparse_us": tot_s, "sum_dense_twin_us": tot_d, "sum_floor_us": tot_f,
                    "speedup": tot_d / tot_s, "frac_of_floor": tot_f / tot_s, "layers": per}
    return out


def print_probes(torch, ss):
    """Calibration probes of the library (include/ss_debug.h): what the chip delivers when nothing else is in the way."""
    print("## register-only issue rate of the matrix instruction (two waves per SIMD on every compute unit), dense-equivalent TFLOP/s")
    for name, dt in (("fp16", ss.SS_F16), ("bf16", ss.SS_BF16)):
        print(f"{name}: 2:4-sparse 32x32x32 {ss.ss_debug_issue_peak(dt, True):8.1f}   dense 32x32x16 {ss.ss_debug_issue_peak(dt, False):8.1f}", flush=True)
    print("## LDS bandwidth of one compute unit, 16 bytes per lane and instruction, eight instructions in flight per wave; "
          "B/clk at the nominal 2.4 GHz")
    for write, what, rows in ((0, "fragment reads", (592, 576, 272, 144)), (1, "lane-linear writes", (16,)),
                              (2, "... as 8-byte writes", (16,)), (3, "... as 4-byte writes", (16,)),
                              (4, "half reading, half writing", (592,))):
        for rb in rows:
            vals = [ss.ss_debug_lds_bandwidth(write, w, rb) for w in ((2, 4) if write == 4 else (1, 2, 4))]
            row = f"{what:20s}" + (f" rows of {rb:3d} B" if not write else "              ")
            print(row + "  " + "  ".join(f"{w} wave(s)/SIMD: {v:6.1f} GB/s = {v / 2.4:5.1f} B/clk" for w, v in zip(((2, 4) if write == 4 else (1, 2, 4)), vals)), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--table", action="store_true", help="per-layer report for all configurations instead of the JSON line")
    ap.add_argument("--cold", action="store_true", help="with --table: rotate buffers so activations are not cache-resident")
    ap.add_argument("--only", default="", help="with --table: only layers whose name contains this string")
    ap.add_argument("--trunk", action="store_true", help="end-to-end ResNet-50 convolution trunk (images/s) instead of the JSON line")
    ap.add_argument("--q8", action="store_true", help="report of the 8-bit integer precision point instead of the JSON line")
    ap.add_argument("--fused", action="store_true", help="report of the fused 3x3 -> 1x1 bottleneck pairs instead of the JSON line")
    ap.add_argument("--tail", action="store_true", help="report of the fused residual / activation tail instead of the JSON line")
    ap.add_argument("--profile-run", action="store_true",
                    help="for rocprofv3: one 512 MiB streaming copy (calibrates the traffic counters), then 20 sparse and "
                         "20 dense-twin launches of the benchmark layer, eagerly; prints nothing but a done line")
    ap.add_argument("--workload", default="cfg1", choices=["cfg1", "cfg1_n500", "cfg1_n512", "cfg2", "s1_c3", "s3_c3", "stem"],
                    help="with --profile-run: which layer to launch")
    ap.add_argument("--probes", action="store_true", help="calibration probes (matrix-instruction issue rate, LDS bandwidth) instead of the JSON line")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-protocol", action="store_true", help="skip the configs[0], [2], [3], [4] and cold-cache legs of the JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the method has no multi-GPU path; batch sharding needs no "
              "exchange). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2411_00288_amd as ss
    from paper_2411_00288_amd import workloads as wl
    torch.cuda.set_device(0)

    if args.probes:
        print_probes(torch, ss)
        return
    if args.trunk:
        print_trunk(torch, ss, wl)
        return
    if args.fused:
        print_fused_table(torch, ss, wl, min(args.steps, 100), min(args.warmup, 20))
        return
    if args.q8:
        print_q8_table(torch, ss, wl, min(args.steps, 200), min(args.warmup, 50))
        return
    if args.tail:
        print_tail_table(torch, ss, wl, min(args.steps, 200), min(args.warmup, 50))
        return
    if args.table:
        print_table(torch, ss, wl, min(args.steps, 200), min(args.warmup, 50), args.cold, args.only)
        return

    L = wl.CONFIG1
    if args.profile_run:
        L = {"cfg1": wl.CONFIG1, "cfg1_n500": wl.with_batch(wl.CONFIG1, 500), "cfg1_n512": wl.with_batch(wl.CONFIG1, 512),
             "cfg2": wl.CONFIG2,
             "s1_c3": [l for l in wl.resnet50_layers() if l.name == "s1_c3_1x1_64_256"][0],
             "s3_c3": [l for l in wl.resnet50_layers() if l.name == "s3_c3_1x1_256_1024"][0],
             "stem": wl.resnet50_layers()[0]}[args.workload]
    run = LayerRun(L, torch, ss, wl, values=not args.profile_run)

    if args.profile_run:
        src = torch.ones(256 << 20, dtype=torch.float16, device="cuda")     # 512 MiB read + 512 MiB written:
        dst = torch.empty_like(src)                                        # larger than every cache level
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)                                       # a plain streaming copy kernel
        torch.cuda.synchronize()
        del src, dst
        if L.mask != "none":
            for _ in range(20):
                run.sparse()
            torch.cuda.synchronize()
        for _ in range(20):
            run.densef()
        torch.cuda.synchronize()
        print(f"profile-run done ({L.name}): 1 streaming copy of 536870912 bytes, 20 sparse, 20 dense launches", flush=True)
        return

    # ---- the timed region: exactly `steps` launches of the sparse convolution, recorded in one HIP
    # graph (a launch lasts a few microseconds, less than the host needs to issue one), replayed
    # once between two events on the launch stream and bracketed by device synchronisation.
    kern_ms = time_graph(torch, run.sparse, args.steps, args.warmup)
    wall_ms = time_graph.last_wall_ms                  # host clock around the same replay (includes one synchronisation)
    ms = kern_ms                                       # one clock for `value` and `roofline.achieved`: the event pair
    value = L.dense_equiv_flop / ms / 1e9              # dense-equivalent TFLOP/s
    eager_ms = time_launches(torch, run.sparse, args.steps, 2)   # host-issued launches, for reference

    # ---- companions (not part of `value`)
    t_dense = median_time(torch, run.densef, args.steps, min(args.warmup, 200))
    t_sparse = median_time(torch, run.sparse, args.steps, 2)
    Lbig = wl.with_batch(L, 512)                      # same layer, 16x the batch: asymptotic utilisation
    big = LayerRun(Lbig, torch, ss, wl, values=False)
    tb_s = median_time(torch, big.sparse, 20, 3, reps=3)
    tb_d = median_time(torch, big.densef, 20, 3, reps=3)
    del big
    # N = 500: 1532 tiles of 256x64 = 2.99 x the 512 workgroups the chip holds, i.e. three full rounds (N = 512 needs
    # a fourth round that is 6 % full)
    Leven = wl.with_batch(L, 500)
    even = LayerRun(Leven, torch, ss, wl, values=False)
    te_s = median_time(torch, even.sparse, 20, 3, reps=3)
    te_d = median_time(torch, even.densef, 20, 3, reps=3)
    del even
    # the 8-bit precision points on the same shape and flattening, N = 32 and N = 500
    q8_small = q8_point(torch, ss, wl, L, min(args.steps, 200), min(args.warmup, 50), korder=L.korder)
    q8_big = q8_point(torch, ss, wl, Leven, 20, 3, korder=L.korder)
    f8_small = q8_point(torch, ss, wl, L, min(args.steps, 200), min(args.warmup, 50), dtype=ss.SS_F8, korder=L.korder)
    f8_big = q8_point(torch, ss, wl, Leven, 20, 3, dtype=ss.SS_F8, korder=L.korder)
    tc = time_launches(torch, lambda: ss.ss_mask_compress(run.desc, run.W, run.M, packed=run.packed), 20, 3)
    Wu, Uz = run.W.clone(), torch.zeros_like(run.W)     # a zero update: the packed weights stay what they are
    tu = time_launches(torch, lambda: ss.ss_mask_update_compress(run.desc, Wu, Uz, run.M, packed=run.packed), 20, 3)

    achieved = L.dense_equiv_flop / kern_ms / 1e9
    issue_peak = ss.ss_debug_issue_peak(ss.SS_F16, True)          # measured: register-only issue rate of the instruction
    issue_peak_dense = ss.ss_debug_issue_peak(ss.SS_F16, False)
    protocol = {} if args.no_protocol else protocol_report(torch, ss, wl, min(args.steps, 200), min(args.warmup, 50))
    out = {
        "metric": "dense-equiv TFLOP/s of 2:4 sparse conv2d; speedup vs same-design dense conv",
        "value": value, "unit": "TFLOP/s (dense-equivalent)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "wall_ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "configs[1]: 3x3 conv 256->256, 14x14, N=32, stride 1, pad 1, fp16 NHWC, "
                               "argmax-of-logits 2:4 mask along Cin*kh*kw, fused bias+ReLU", "K": L.K, "P": L.P},
        "speedup_vs_dense_twin": t_dense / t_sparse,
        "sparse_us": t_sparse * 1e3, "dense_twin_us": t_dense * 1e3,
        "scaled_batch": {"workload": "same layer at N=512", "sparse_us": tb_s * 1e3, "dense_twin_us": tb_d * 1e3,
                         "tflops": Lbig.dense_equiv_flop / tb_s / 1e9, "speedup": tb_d / tb_s,
                         "frac_sparse_peak": Lbig.dense_equiv_flop / tb_s / 1e9 / SPARSE_PEAK_TFLOPS},
        "scaled_batch_full_rounds": {"workload": "same layer at N=500 (three full rounds of workgroups)", "sparse_us": te_s * 1e3,
                                     "dense_twin_us": te_d * 1e3, "tflops": Leven.dense_equiv_flop / te_s / 1e9,
                                     "speedup": te_d / te_s,
                                     "frac_sparse_peak": Leven.dense_equiv_flop / te_s / 1e9 / SPARSE_PEAK_TFLOPS},
        "int8": {"workload": "same shape, mask and flattening with int8 operands, fp16 output", "n32": q8_small,
                 "n500": q8_big, "peak_tops": SPARSE_INT8_PEAK_TOPS},
        "fp8": {"workload": "same shape, mask and flattening with FP8 E4M3 operands, fp16 output", "n32": f8_small,
                "n500": f8_big, "peak_tflops": SPARSE_INT8_PEAK_TOPS},
        "compress_us": tc * 1e3, "update_compress_us": tu * 1e3, "eager_launch_us": eager_ms * 1e3,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": SPARSE_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / SPARSE_PEAK_TFLOPS, "traffic": CFG1_TRAFFIC_BYTES,
                     "traffic_unit": "bytes per launch (algorithmic: %d)" % L.algorithmic_bytes(True),
                     "traffic_source": "profiles/conv_kernel_hbm_traffic.md (rocprofv3 FETCH_SIZE / WRITE_SIZE, L2 misses and "
                                       "write-backs, not measured in this run)",
                     "measured_issue_peak": issue_peak, "frac_vs_measured_issue_peak": achieved / issue_peak,
                     "kernel": "ss::conv_kernel (sparse, fp16)", "flop_per_launch": L.dense_equiv_flop,
                     "kernel_us": kern_ms * 1e3},
    }
    out["measured_issue_peak"] = {"sparse_32x32x32_f16_tflops": issue_peak, "dense_32x32x16_f16_tflops": issue_peak_dense,
                                  "note": "register-only probe, two waves per SIMD on every compute unit, dense-equivalent"}
    out["scaled_batch_full_rounds"]["frac_vs_measured_issue_peak"] = Leven.dense_equiv_flop / te_s / 1e9 / issue_peak
    out["protocol"] = protocol
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(L, wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
