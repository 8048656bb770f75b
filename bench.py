#!/usr/bin/env python3
"""Benchmark of the SegLinear + DualScale hot path on one MI355X.

A "step" is one pass of the whole online path over one batch of synthetic input that is already
resident in HBM:  sq_quantize_act (bf16 -> int8 x+/x-)  followed by  sq_seglinear (dual-path int8 GEMM
with per-K-segment accumulators and the fused dequant epilogue, bf16 out).  Weights are quantized once
before the timed region (the offline step) and reported separately.

Prints ONE JSON line.  `value` = executed int8 ops of the step (both polarity paths counted, skipped
x- work of single-scale segments not counted) / step time.  `roofline` is the GEMM kernel alone, timed
with HIP events on the launch stream inside the timed region.  `cpu_baseline` is the CPU oracle on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5033.2   # 256 CU x 2.4 GHz x 8192 int8 ops/clk/CU (dense)
FP8_MFMA_PEAK_TFLOPS = 5033.2  # the same rate for dense fp8 operands (v_mfma_f32_32x32x64_f8f6f4)
HBM_PEAK_GBS = 8000.0
PREROLL_MS = 80.0              # untimed load before the warm-up steps, so that the device clocks have settled
USE_GRAPHS = True              # --no-graph: time small kernels with plain launches (for runs under rocprofv3)

# Fabric-side traffic per GEMM launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by the
# readings of a plain 256 MiB copy kernel (profiles/bench_all_kernels_rocprofv3.txt), bytes.  None for a
# workload without a committed counter run.
MEASURED_TRAFFIC = {
    "cfg5_outproj": int(294447.2 * 1024 * 2.0 + 54732.0 * 1024 * 1.0),       # 659.1 MB (algorithmic 146.3 MB)
    "cfg4d_qkv_dual": int(69542.1 * 1024 * 2.0 + 76545.7 * 1024 * 1.0),
    "cfg4_qkv": int(69402.0 * 1024 * 2.0 + 76588.6 * 1024 * 1.0),
    "cfg2_dit_fc2": int(19727.0 * 1024 * 2.0 + 4608.0 * 1024 * 1.0),
}
# the same for the skinny weight stream and the activation quantizer (passes of their own in profiles/)
MEASURED_TRAFFIC_SKINNY = {"cfg3": int(4071.5 * 1024 * 2.0 + 216.0 * 1024), "cfg3x28": int(109776.6 * 1024 * 2.0 + 6049.9 * 1024)}
MEASURED_TRAFFIC_QUANT = {"cfg5": int(69204.7 * 1024 * 2.0 + 69120.0 * 1024), "cfg2": int(9252.1 * 1024 * 2.0 + 9216.0 * 1024),
                          "cfg4": int(12786.2 * 1024 * 2.0 + 12750.0 * 1024), "cfg4d": int(12786.2 * 1024 * 2.0 + 12750.0 * 1024)}


def _setup(name):
    import torch

    from paper_2507_14811_amd import workloads as wl
    import paper_2507_14811_amd as sq

    w = wl.make(name)
    dev = "cuda:0"
    layer = sq.Layer.from_workload(w)
    if w.x_dtype == "bf16":
        x = torch.from_numpy(wl.f32_to_bf16_bits(w.x).view(np.int16)).view(torch.bfloat16).to(dev)
    else:
        x = torch.from_numpy(w.x).to(dev)
    wt = torch.from_numpy(w.w).to(dev)
    wq = torch.empty((w.N, w.K), dtype=torch.int8, device=dev)
    wscale = torch.empty((w.S, w.N), dtype=torch.float32, device=dev)
    xq = torch.empty((w.M, w.K), dtype=torch.int8, device=dev)
    y = torch.empty((w.M, w.N), dtype=torch.bfloat16, device=dev)
    return dict(w=w, layer=layer, x=x, wt=wt, wq=wq, wscale=wscale, xq=xq, y=y)


def _time_events(fn, iters):
    import torch

    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in evs]


def _gpu_side_ms(fns, launches=200, replays=5):
    """GPU-side time per launch with the host's launch cost taken out: `launches` launches, cycling over `fns` (one
    callable per buffer set, so that a rotation over distinct buffers defeats the caches), are captured into one HIP
    graph, the graph is replayed, and the time between two events around a replay is divided by the launch count.
    From Python a launch through ctypes costs 6-7 us of host time, more than the small kernels take."""
    import torch

    n = max(len(fns), (launches // len(fns)) * len(fns))
    if not USE_GRAPHS:      # under a profiler: plain launches, one event pair around all of them (host cost included)
        for f in fns:
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fns[i % len(fns)]()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for f in fns:
            f()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        for i in range(n):
            fns[i % len(fns)]()
    g.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / n)
    del g
    return float(np.median(ts))


def measure(name, steps, warmup, rotate_quant=True, hot_only=False):
    """Times one workload.  Returns a dict of per-kernel and per-step figures."""
    import torch

    import paper_2507_14811_amd as sq

    s = _setup(name)
    w, layer = s["w"], s["layer"]

    # offline step: weight quantization (timed on its own)
    sq.sq_quantize_weight(layer, s["wt"], s["wq"], s["wscale"])
    torch.cuda.synchronize()
    t_wq = float(np.median(_time_events(lambda: sq.sq_quantize_weight(layer, s["wt"], s["wq"], s["wscale"]), 5)))

    def quant():
        sq.sq_quantize_act(layer, s["x"], s["xq"])

    def gemm():
        sq.sq_seglinear(layer, s["xq"], s["wq"], s["wscale"], None, s["y"])

    # Clock ramp: the device needs some tens of milliseconds of load before its clocks settle (the first 25 steps
    # of cfg5 run 35 % slower than the steady state, which is reached after ~100 steps).  Untimed pre-roll of
    # about PREROLL_MS, then the W warm-up steps the caller asked for.
    t0 = time.perf_counter()
    quant()
    gemm()
    torch.cuda.synchronize()
    est = max(time.perf_counter() - t0, 1e-5)
    if w.M > 64:
        # large layers: the pre-roll load is the register-only MFMA probe on this layer's own codes (about 10 ms per
        # launch), so that every launch of the layer's kernel in a profiler trace runs at settled clocks and the trace's
        # average duration is the figure this benchmark reports; the W warm-up steps below use the real step
        from paper_2507_14811_amd import probes

        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < PREROLL_MS:
            probes.sqp_mfma(s["xq"].view(-1)[: 16 << 20], 20000)
            torch.cuda.synchronize()
    else:
        preroll = int(min(2000, max(20, PREROLL_MS * 1e-3 / est)))
        for _ in range(preroll):
            quant()
            gemm()
        torch.cuda.synchronize()
    for _ in range(warmup):
        quant()
        gemm()
    torch.cuda.synchronize()

    # ---- the timed region: exactly `steps` steps, HIP events around every GEMM launch ----------------
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        quant()
        a.record()
        gemm()
        b.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / steps
    ms_gemm = float(np.mean([a.elapsed_time(b) for a, b in ev]))

    # the GEMM kernel back to back (one event pair around `steps` launches): for kernels of a few microseconds
    # the per-launch event pairs above mostly measure launch gaps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        gemm()
    e1.record()
    torch.cuda.synchronize()
    ms_gemm_b2b = e0.elapsed_time(e1) / steps

    # quantize pass alone (outside the step timing).  Small inputs would sit in the 256 MB Infinity
    # Cache between calls, so rotate over distinct buffers totalling > 512 MB to measure HBM.
    qbytes = w.quantize_act_bytes()
    nrot = 1
    if rotate_quant and qbytes < 300e6:
        nrot = int(min(64, max(2, np.ceil(600e6 / qbytes))))
    xs = [s["x"]] + [s["x"].clone() for _ in range(nrot - 1)]
    xqs = [s["xq"]] + [torch.empty_like(s["xq"]) for _ in range(nrot - 1)]
    reps = max(2, int(np.ceil(40 / nrot)))

    def quant_rot():
        for i in range(nrot):
            sq.sq_quantize_act(layer, xs[i], xqs[i])

    quant_rot()
    torch.cuda.synchronize()
    ms_quant_stream = float(np.median(_time_events(quant_rot, reps))) / nrot      # launched from Python, one after another
    ms_quant = _gpu_side_ms([(lambda i=i: sq.sq_quantize_act(layer, xs[i], xqs[i])) for i in range(nrot)],
                            launches=max(nrot, 60))
    # restore the canonical buffers for the GEMM
    quant()
    torch.cuda.synchronize()

    ms_calib = ms_quant_fused = ms_quant_fused_lut = ms_quant_dyn = ms_gemm_dyn = ms_calib_pct = ms_wblock = None
    if not hot_only:
        # calibration-side kernels on the same tensors: min/max steps (one read of the activations) and the
        # block-granular weight quantizer
        amax = torch.empty((2, w.S), dtype=torch.float32, device="cuda:0")
        stp = torch.empty((2, w.S), dtype=torch.float32, device="cuda:0")
        sq.sq_calibrate_act(layer, s["x"], amax, stp)
        torch.cuda.synchronize()
        ms_calib = float(np.median(_time_events(lambda: sq.sq_calibrate_act(layer, s["x"], amax, stp), 10)))
        # the activation fused in front of the quantizer: GELU on the dual K-segments (the headline layer's MLP half)
        codes = [sq.SQ_ACT_GELU if d else sq.SQ_ACT_NONE for d in w.dual]
        xq_f = torch.empty_like(s["xq"])
        sq.sq_quantize_act_fused(layer, s["x"], codes, xq_f)
        torch.cuda.synchronize()
        ms_quant_fused = float(np.median(_time_events(lambda: sq.sq_quantize_act_fused(layer, s["x"], codes, xq_f), 20)))
        fws = torch.empty((sq.sq_quantize_act_fused_workspace_bytes(layer),), dtype=torch.uint8, device="cuda:0")
        sq.sq_quantize_act_fused(layer, s["x"], codes, xq_f, workspace=fws)
        torch.cuda.synchronize()
        ms_quant_fused_lut = float(np.median(_time_events(lambda: sq.sq_quantize_act_fused(layer, s["x"], codes, xq_f, workspace=fws), 20)))
        del xq_f
        # dynamic per-token activation steps (the 4-bit settings' activation rule) on the same layer: quantizer that also
        # writes every row's steps, and the GEMM that reads them in its flushes (8-bit weights)
        ms_quant_dyn = ms_gemm_dyn = None
        if w.M > 64:
            tok = torch.empty((2, w.M, w.S), dtype=torch.float32, device="cuda:0")
            xq_d = torch.empty_like(s["xq"])
            y_d = torch.empty_like(s["y"])
            sq.sq_quantize_act_dynamic(layer, s["x"], xq_d, tok)
            sq.sq_seglinear_dynamic(layer, xq_d, tok, s["wq"], 8, s["wscale"], None, y_d)
            torch.cuda.synchronize()
            ms_quant_dyn = float(np.median(_time_events(lambda: sq.sq_quantize_act_dynamic(layer, s["x"], xq_d, tok), 10)))
            ms_gemm_dyn = float(np.median(_time_events(
                lambda: sq.sq_seglinear_dynamic(layer, xq_d, tok, s["wq"], 8, s["wscale"], None, y_d), 10)))
            del xq_d, y_d, tok
        pws = torch.empty((sq.sq_calibrate_workspace_bytes(),), dtype=torch.uint8, device="cuda:0")
        sq.sq_calibrate_act_percentile(layer, s["x"], 0.9999, amax, stp, pws)
        torch.cuda.synchronize()
        ms_calib_pct = float(np.median(_time_events(lambda: sq.sq_calibrate_act_percentile(layer, s["x"], 0.9999, amax, stp, pws), 10)))
        wq2, ws2 = torch.empty_like(s["wq"]), torch.empty_like(s["wscale"])
        sq.sq_quantize_weight_block(layer, s["wt"], wq2, ws2)
        torch.cuda.synchronize()
        ms_wblock = float(np.median(_time_events(lambda: sq.sq_quantize_weight_block(layer, s["wt"], wq2, ws2), 5)))
        del wq2, ws2

    gbytes = w.seglinear_bytes("bf16")

    # Skinny layers are one pass over the weights: with a single weight set the pass is served by the 256 MB
    # Infinity Cache, so also stream over a rotation of distinct (weights, scales) sets totalling > 512 MB.
    ms_gemm_hbm, ms_gemm_hbm_stream, nsets = None, None, 1
    if w.M <= 64:
        wbytes = w.N * w.K
        nsets = int(min(64, max(2, np.ceil(600e6 / wbytes))))
        wqs = [s["wq"]] + [s["wq"].clone() for _ in range(nsets - 1)]
        wss = [s["wscale"]] + [s["wscale"].clone() for _ in range(nsets - 1)]
        reps = max(2, int(np.ceil(2 * steps / nsets)))

        def rot():
            for i in range(nsets):
                sq.sq_seglinear(layer, s["xq"], wqs[i], wss[i], None, s["y"])

        rot()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            rot()
        e1.record()
        torch.cuda.synchronize()
        ms_gemm_hbm_stream = e0.elapsed_time(e1) / (reps * nsets)                # launched from Python
        ms_gemm_hbm = _gpu_side_ms([(lambda i=i: sq.sq_seglinear(layer, s["xq"], wqs[i], wss[i], None, s["y"])) for i in range(nsets)],
                                   launches=max(nsets, 128))
        del wqs, wss
    return dict(
        xq_codes=s["xq"].reshape(-1),
        xq_dual_cols=(s["xq"][:, int(w.kseg_off[int(np.argmax(w.dual))]):int(w.kseg_off[int(np.argmax(w.dual)) + 1])].contiguous()
                      if any(w.dual) else None),
        name=w.name, M=w.M, K=w.K, N=w.N, S=w.S, T=w.T, dual=[int(d) for d in w.dual],
        int8_ops=w.int8_ops, ms_step=ms_step, ms_gemm=ms_gemm, ms_quant=ms_quant, ms_quantize_weight=t_wq,
        gemm_tops=w.int8_ops / (ms_gemm * 1e-3) / 1e12, step_tops=w.int8_ops / (ms_step * 1e-3) / 1e12,
        ms_gemm_b2b=ms_gemm_b2b, gemm_tops_b2b=w.int8_ops / (ms_gemm_b2b * 1e-3) / 1e12,
        gemm_bytes=gbytes, gemm_gbs=gbytes / (ms_gemm * 1e-3) / 1e9, gemm_gbs_b2b=gbytes / (ms_gemm_b2b * 1e-3) / 1e9,
        ms_gemm_hbm=ms_gemm_hbm, ms_gemm_hbm_stream=ms_gemm_hbm_stream, ms_quant_stream=ms_quant_stream, weight_sets=nsets, ms_quant_fused=ms_quant_fused, ms_quant_fused_lut=ms_quant_fused_lut, ms_quant_dyn=ms_quant_dyn, ms_gemm_dyn=ms_gemm_dyn, ms_calibrate=ms_calib, ms_calibrate_percentile=ms_calib_pct, ms_quantize_weight_block=ms_wblock,
        calib_gbs=None if ms_calib is None else (w.M * w.K * (2 if w.x_dtype == "bf16" else 4)) / (ms_calib * 1e-3) / 1e9,
        gemm_gbs_hbm=(gbytes / (ms_gemm_hbm * 1e-3) / 1e9) if ms_gemm_hbm else None,
        quant_bytes=qbytes, quant_gbs=qbytes / (ms_quant * 1e-3) / 1e9, quant_rotation=nrot,
    )


def measure_grouped(layers=28, steps=50):
    """The grouped skinny call: `layers` adaLN-shaped layers (cfg3's shape and weight recipe, separate weight
    buffers) that share one quantized input, in one launch; weight sets rotated so the stream comes from HBM."""
    import torch

    import paper_2507_14811_amd as sq
    from paper_2507_14811_amd import workloads as wl

    dev = "cuda:0"
    w = wl.make("cfg3")
    layer = sq.Layer.from_workload(w)
    x = torch.from_numpy(wl.f32_to_bf16_bits(w.x).view(np.int16)).view(torch.bfloat16).to(dev)
    xq = torch.empty((w.M, w.K), dtype=torch.int8, device=dev)
    sq.sq_quantize_act(layer, x, xq)
    nsets = 3                                   # 3 x 28 x 8 MB = 669 MB of weights > 2 x Infinity Cache... of 256 MB
    sets, sets4 = [], []
    for si in range(nsets):
        items, items4 = [], []
        for l in range(layers):
            wl_l = wl.make("cfg3", seed=1000 + si * layers + l)
            wt = torch.from_numpy(wl_l.w).to(dev)
            wq = torch.empty((w.N, w.K), dtype=torch.int8, device=dev)
            ws = torch.empty((w.S, w.N), dtype=torch.float32, device=dev)
            sq.sq_quantize_weight(layer, wt, wq, ws)
            y = torch.empty((w.M, w.N), dtype=torch.bfloat16, device=dev)
            items.append((wq, ws, None, y))
            wq4 = torch.empty((((w.N + 15) // 16) * 16 * (w.K // 2),), dtype=torch.uint8, device=dev)
            ws4 = torch.empty((w.S, w.N), dtype=torch.float32, device=dev)
            sq.sq_quantize_weight_w4(layer, wt, wq4, ws4)
            items4.append((wq4, ws4, None, y))
        sets.append(sq.GroupItems(items))       # marshalled once: filling 28 items costs more host time than the launch
        sets4.append(sq.GroupItems(items4))
    torch.cuda.synchronize()

    def run_all():
        for items in sets:
            sq.sq_seglinear_grouped(layer, xq, items)

    for _ in range(20):
        run_all()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run_all()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (steps * nsets)
    byt = layers * w.seglinear_bytes("bf16")
    # the same layers one call each, for comparison
    e0.record()
    for _ in range(max(2, steps // 5)):
        for items in sets:
            for (wq, ws, b, y) in items.tensors:
                sq.sq_seglinear(layer, xq, wq, ws, b, y)
    e1.record()
    torch.cuda.synchronize()
    ms_single = e0.elapsed_time(e1) / (max(2, steps // 5) * nsets)

    # Linear(SiLU(c)) from the raw conditioning input: activation + Q_dual inside the weight-stream kernel (one launch)
    # against sq_quantize_act_fused followed by the grouped call (two launches)
    def timed(fn):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (steps * nsets)

    silu = [sq.SQ_ACT_SILU] * w.S

    def one_launch():
        for items in sets:
            sq.sq_seglinear_grouped_fused(layer, x, silu, items)

    def two_launches():
        for items in sets:
            sq.sq_quantize_act_fused(layer, x, silu, xq)
            sq.sq_seglinear_grouped(layer, xq, items)

    ms_one, ms_two = timed(one_launch), timed(two_launches)

    # the same group with packed 4-bit weights, static and per-token steps (3 sets = 334 MB: above the Infinity Cache)
    tok = torch.empty((2, w.M, w.S), dtype=torch.float32, device=dev)
    xq_d = torch.empty_like(xq)
    sq.sq_quantize_act_dynamic(layer, x, xq_d, tok)

    def w4_static():
        for items in sets4:
            sq.sq_seglinear_grouped_w4(layer, xq, items)

    def w4_dynamic():
        for items in sets4:
            sq.sq_seglinear_grouped_w4(layer, xq_d, items, tok_steps=tok)

    ms_w4, ms_w4_dyn = timed(w4_static), timed(w4_dynamic)
    return {"layers": layers, "silu_in_front": {"ms_one_launch_raw_input": round(ms_one, 5),
                                                "ms_quantize_then_grouped": round(ms_two, 5)},
            "w4": {"ms_per_launch": round(ms_w4, 5), "ms_per_launch_dynamic_token_steps": round(ms_w4_dyn, 5)}, "M": w.M, "K": w.K, "N": w.N, "ms_per_launch": round(ms, 5), "bytes": byt,
            "gbs_from_hbm": round(byt / (ms * 1e-3) / 1e9, 1), "frac_hbm_peak": round(byt / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "ms_same_layers_one_call_each": round(ms_single, 5), "weight_sets_rotated": nsets}


def measure_geglu(M=4096, K=5120, steps=20):
    """GEGLU in front of the quantizer at the shape of a GEGLU feed-forward (inner width 4 x 1280, a 64 x 64 latent's
    tokens): h [M][2K] bf16 -> codes [M][K]."""
    import torch

    import paper_2507_14811_amd as sq

    gen = torch.Generator(device="cuda:0").manual_seed(5)
    h = (torch.randn((M, 2 * K), device="cuda:0", generator=gen) * 1.5).to(torch.bfloat16)
    layer = sq.Layer(M, K, 16, [0, K], [0, 16], [1], [4.0 / 127], [0.25 / 127])
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda:0")
    sq.sq_quantize_act_geglu(layer, h, xq)
    torch.cuda.synchronize()
    ms = float(np.median(_time_events(lambda: sq.sq_quantize_act_geglu(layer, h, xq), steps)))
    byt = M * K * 5
    return {"M": M, "K": K, "ms_per_launch": round(ms, 5), "bytes": byt, "achieved": round(byt / (ms * 1e-3) / 1e9, 1),
            "unit": "GB/s", "frac_hbm_peak": round(byt / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "note": "4 B in + 1 B out per output (bf16); two input streams per row and the bit-specified GELU of the gate"}


def measure_w4(steps=40):
    """The stacked modulation layer (cfg3x28) with 4-bit packed weights: one pass over half the weight bytes.  Weight
    sets rotated so the stream comes from HBM."""
    import torch

    import paper_2507_14811_amd as sq

    s = _setup("cfg3x28")
    w, layer = s["w"], s["layer"]
    sq.sq_quantize_act(layer, s["x"], s["xq"])
    nsets = 6                                   # 6 x 111 MB of packed weights > 2 x the 256 MB Infinity Cache
    wq4 = torch.empty((((w.N + 15) // 16) * 16 * (w.K // 2),), dtype=torch.uint8, device="cuda:0")
    sq.sq_quantize_weight_w4(layer, s["wt"], wq4, s["wscale"])
    torch.cuda.synchronize()
    ms_qw = float(np.median(_time_events(lambda: sq.sq_quantize_weight_w4(layer, s["wt"], wq4, s["wscale"]), 5)))
    sets = [wq4] + [wq4.clone() for _ in range(nsets - 1)]

    def rot():
        for t in sets:
            sq.sq_seglinear_w4(layer, s["xq"], t, s["wscale"], None, s["y"])

    for _ in range(5):
        rot()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        rot()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (steps * nsets)
    # the paper's 4-bit setting in full: activations with dynamic per-token steps
    tok = torch.empty((2, w.M, w.S), dtype=torch.float32, device="cuda:0")
    sq.sq_quantize_act_dynamic(layer, s["x"], s["xq"], tok)

    def rot_dyn():
        for t in sets:
            sq.sq_seglinear_dynamic(layer, s["xq"], tok, t, 4, s["wscale"], None, s["y"])

    for _ in range(5):
        rot_dyn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        rot_dyn()
    e1.record()
    torch.cuda.synchronize()
    ms_dyn = e0.elapsed_time(e1) / (steps * nsets)
    ms_qdyn = float(np.median(_time_events(lambda: sq.sq_quantize_act_dynamic(layer, s["x"], s["xq"], tok), 10)))

    # the same from the raw input in ONE launch: SiLU, per-token steps, codes and the W4 stream (s["x"] stands for the
    # pre-activation here: the timing does not depend on the values)
    def rot_fused_dyn():
        for t in sets:
            sq.sq_seglinear_fused_dynamic(layer, s["x"], [sq.SQ_ACT_SILU] * w.S, t, 4, s["wscale"], None, s["y"])

    for _ in range(5):
        rot_fused_dyn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        rot_fused_dyn()
    e1.record()
    torch.cuda.synchronize()
    ms_fused_dyn = e0.elapsed_time(e1) / (steps * nsets)
    # packed codes back to one int8 code per byte (what a layer with many token rows feeds to the int8 tile kernel)
    wq8 = torch.empty((w.N, w.K), dtype=torch.int8, device="cuda:0")
    sq.sq_unpack_w4(layer, sets[0], wq8)
    torch.cuda.synchronize()
    ms_unpack = float(np.median(_time_events(lambda: sq.sq_unpack_w4(layer, sets[0], wq8), 10)))
    del wq8
    byt = int(w.M * w.K + w.N * w.K // 2 + 4 * w.S * w.N + 2 * w.M * w.N)
    return {"workload": "cfg3x28 with 4-bit packed weights", "ms_unpack_w4": round(ms_unpack, 5),
            "unpack_w4_gbs": round(1.5 * w.N * w.K / (ms_unpack * 1e-3) / 1e9, 1), "M": w.M, "K": w.K, "N": w.N, "ms_per_launch": round(ms, 5),
            "bytes": byt, "gbs_from_hbm": round(byt / (ms * 1e-3) / 1e9, 1),
            "frac_hbm_peak": round(byt / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "gemm_tops": round(w.int8_ops / (ms * 1e-3) / 1e12, 1), "ms_quantize_weight_w4": round(ms_qw, 5),
            "ms_per_launch_dynamic_token_steps": round(ms_dyn, 5), "ms_quantize_act_dynamic": round(ms_qdyn, 5),
            "ms_one_launch_raw_input_silu_dynamic": round(ms_fused_dyn, 5),
            "weight_sets_rotated": nsets}


def _timed_launches(fn, reps=200):
    """(ms per launch from one HIP event pair around `reps` back-to-back launches, median ms of single launches each
    bracketed by its own event pair)."""
    import torch

    for _ in range(20):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    b2b = e0.elapsed_time(e1) / reps
    single = float(np.median(_time_events(fn, 50)))
    return b2b, single


def measure_optimizer_side(name="cfg5"):
    """The entry points that serve the paper's optimizers on the headline layer's shape: SmoothQuant factors with one
    alpha per K-segment (per-channel maxima, smoothed quantizers; the factors themselves are a host computation) and the
    rank-64 low-rank side branch of the 4-bit settings."""
    import torch

    import paper_2507_14811_amd as sq

    s = _setup(name)
    w, layer = s["w"], s["layer"]
    dev = "cuda:0"
    ax = torch.empty((w.K,), dtype=torch.float32, device=dev)
    aw = torch.empty((w.K,), dtype=torch.float32, device=dev)
    t_ax = float(np.median(_time_events(lambda: sq.sq_calibrate_channel_amax(layer, s["x"], ax), 10)))
    t_aw = float(np.median(_time_events(lambda: sq.sq_weight_channel_amax(layer, s["wt"], aw), 10)))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    smooth, inv = sq.sq_smooth_factors(layer, ax.cpu().numpy(), aw.cpu().numpy(), [0.5] * w.S)
    t_host = (time.perf_counter() - t0) * 1e3
    sm, iv = torch.from_numpy(smooth).to(dev), torch.from_numpy(inv).to(dev)
    t_qw = float(np.median(_time_events(lambda: sq.sq_quantize_weight_smoothed(layer, s["wt"], sm, s["wq"], s["wscale"]), 5)))
    t_qa = _gpu_side_ms([lambda: sq.sq_quantize_act_smoothed(layer, s["x"], iv, s["xq"])], launches=40)
    ld = torch.randn((64, w.K), device=dev).to(torch.bfloat16)
    lu = torch.randn((w.N, 64), device=dev).to(torch.bfloat16)
    yq = torch.zeros((w.M, w.N), dtype=torch.float32, device=dev)
    ws = torch.empty((sq.sq_lowrank_workspace_bytes(layer, 64),), dtype=torch.uint8, device=dev)
    t_lr = _gpu_side_ms([lambda: sq.sq_lowrank_add(layer, s["x"], ld, lu, yq, s["y"], ws)], launches=20)
    qbytes = w.quantize_act_bytes()
    return {"workload": w.name,
            "smoothing": {"ms_calibrate_channel_amax": round(t_ax, 5), "ms_weight_channel_amax": round(t_aw, 5),
                          "ms_smooth_factors_on_the_host": round(t_host, 3), "ms_quantize_weight_smoothed": round(t_qw, 5),
                          "ms_quantize_act_smoothed": round(t_qa, 5),
                          "quantize_act_smoothed_gbs": round(qbytes / (t_qa * 1e-3) / 1e9, 1),
                          "quantize_act_smoothed_frac_hbm_peak": round(qbytes / (t_qa * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
            "lowrank_rank64": {"ms_per_call": round(t_lr, 5), "launches": 3,
                               "bytes": int(w.M * w.K * 2 + w.M * w.N * 6),
                               "gbs": round((w.M * w.K * 2 + w.M * w.N * 6) / (t_lr * 1e-3) / 1e9, 1),
                               "note": "down projection (bf16 matrix cores, LDS-staged, K slices), slice sum, up projection + add (T as "
                                       "three exact bf16 terms on the bf16 matrix cores): bytes = X once, y_q read as fp32, y written as bf16"}}


def measure_fp8(names=("cfg5", "cfg4", "cfg2")):
    """The 8-bit floating-point variant (E4M3 codes, fp8 matrix cores) on the named layers: activation quantizer and
    product, timed GPU-side like the int8 path, against the fp8 matrix-core peak and the register-only fp8 MFMA probe
    fed with the layer's own codes."""
    import torch

    import paper_2507_14811_amd as sq
    from paper_2507_14811_amd import probes

    out = {}
    for name in names:
        s = _setup(name)
        w = s["w"]
        dev = "cuda:0"
        sp = (w.s_pos * np.float32(127.0 / 448.0)).astype(np.float32)      # the same calibrated ranges over 448
        sn = (w.s_neg * np.float32(127.0 / 448.0)).astype(np.float32)
        layer = sq.Layer(w.M, w.K, w.N, w.kseg_off, w.nseg_off, w.dual, sp, sn, w.seg_scale)
        xq = torch.empty((w.M, w.K), dtype=torch.uint8, device=dev)
        wq = torch.empty((w.N, w.K), dtype=torch.uint8, device=dev)
        sq.sq_quantize_weight_fp8(layer, s["wt"], wq, s["wscale"])
        quant = lambda: sq.sq_quantize_act_fp8(layer, s["x"], xq)
        gemm = lambda: sq.sq_seglinear_fp8(layer, xq, wq, s["wscale"], None, s["y"])
        quant()
        if w.M > 64:          # clock-ramp pre-roll on the fp8 MFMA probe, like measure()
            t0 = time.perf_counter()
            while (time.perf_counter() - t0) * 1e3 < PREROLL_MS:
                probes.sqp_mfma_fp8(xq.view(-1)[: 16 << 20], 10000)
                torch.cuda.synchronize()
        for _ in range(10):
            gemm()
        torch.cuda.synchronize()
        t_q = _gpu_side_ms([quant], launches=50)
        if w.M <= 64:
            # a skinny layer is a weight stream: rotate over distinct weight sets so that the bytes come from HBM
            nsets = max(2, min(64, int(2.5e9 // max(1, w.N * w.K))))
            sets = [wq] + [wq.clone() for _ in range(nsets - 1)]
            t_g = _gpu_side_ms([(lambda q=q: sq.sq_seglinear_fp8(layer, xq, q, s["wscale"], None, s["y"])) for q in sets], launches=64)
            del sets
        else:
            t_g = _gpu_side_ms([gemm], launches=50)
        t_step = _gpu_side_ms([quant, gemm], launches=50) * 2        # per pair
        flops = float(w.int8_ops)                                     # the same multiply-adds, both polarity products
        r = {"M": int(w.M), "K": int(w.K), "N": int(w.N), "ms_quantize_act_fp8": round(t_q, 5), "ms_seglinear_fp8": round(t_g, 5),
             "ms_step": round(t_step, 5), "tflops": round(flops / (t_g * 1e-3) / 1e12, 1),
             "frac_fp8_mfma_peak": round(flops / (t_g * 1e-3) / 1e12 / FP8_MFMA_PEAK_TFLOPS, 4),
             "step_tflops": round(flops / (t_step * 1e-3) / 1e12, 1),
             "quant_gbs": round(w.quantize_act_bytes() / (t_q * 1e-3) / 1e9, 1),
             "quant_frac_hbm_peak": round(w.quantize_act_bytes() / (t_q * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if w.M <= 64:
            gb = w.seglinear_bytes()
            r.update({"bound": "hbm", "bytes": int(gb), "gbs_from_hbm": round(gb / (t_g * 1e-3) / 1e9, 1),
                      "frac_hbm_peak_from_hbm": round(gb / (t_g * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
        if name == names[0]:
            acts = [sq.SQ_ACT_GELU if d else sq.SQ_ACT_NONE for d in w.dual]
            t_qf = _gpu_side_ms([lambda: sq.sq_quantize_act_fp8_fused(layer, s["x"], acts, xq)], launches=30)
            lut_ws = torch.empty((sq.sq_quantize_act_fused_workspace_bytes(layer),), dtype=torch.uint8, device=dev)
            t_qt = _gpu_side_ms([lambda: sq.sq_quantize_act_fp8_fused(layer, s["x"], acts, xq, lut_ws)], launches=30)   # per call (two launches)
            r["ms_quantize_act_fp8_fused_gelu_by_code_table"] = round(t_qt, 5)
            quant()                                               # restore the codes of the plain quantizer
            r["ms_quantize_act_fp8_fused_gelu"] = round(t_qf, 5)
            codes = xq.view(-1)[: 16 << 20]
            for _ in range(3):
                probes.sqp_mfma_fp8(codes, 10000)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ops = probes.sqp_mfma_fp8(codes, 10000)
            e1.record()
            torch.cuda.synchronize()
            ceil = ops / (e0.elapsed_time(e1) * 1e-3) / 1e12
            r["mfma_fp8_tflops_layer_like_operands"] = round(ceil, 1)
            r["frac_of_measured_fp8_mfma_ceiling"] = round(flops / (t_g * 1e-3) / 1e12 / ceil, 4)
        out[name] = r
        del s, xq, wq
    return {"peak_tflops": FP8_MFMA_PEAK_TFLOPS, "workloads": out,
            "note": "OCP E4M3 codes, steps range / 448, products on v_mfma_f32_32x32x64_f8f6f4 with fp32 accumulators; flops count both "
                    "polarity products of the dual K-segments like the int8 figure"}


def measured_ceilings(head_setup_codes, dual_cols=None):
    """Ceilings and floors measured on this device with the probe library, reported next to the datasheet peaks:
    the sustained int8 MFMA rate of a register-only loop (all-zero operands; operands distributed like the headline
    layer's codes; the same with the activation operand split by polarity as the dual path feeds it), a plain device
    copy over 2 x 1 GiB, and what a launch costs: an empty kernel in the launch shapes the library uses, and a kernel
    that makes one dependent trip to memory."""
    import torch

    from paper_2507_14811_amd import probes

    out = {}
    zeros = torch.zeros(16 << 20, dtype=torch.int8, device="cuda:0")
    cases = [("zero_operands", zeros), ("layer_like_operands", head_setup_codes)]
    if dual_cols is not None:   # A operands: X^_+ of the dual K-segment (negatives zeroed), B operands: codes as they are
        n = (min(dual_cols.numel(), 8 << 20) // 64) * 64
        a_op = torch.clamp(dual_cols.reshape(-1)[:n], min=0).view(-1, 64)
        b_op = head_setup_codes.reshape(-1)[:n].view(-1, 64)
        cases.append(("layer_like_operands_positive_polarity", torch.cat([a_op, b_op], dim=1).contiguous().view(-1)))
    for label, codes in cases:
        iters = 20000
        for _ in range(3):   # ~10 ms each: lets the clocks settle at this load
            probes.sqp_mfma(codes, iters)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = probes.sqp_mfma(codes, iters)
        e1.record()
        torch.cuda.synchronize()
        out["mfma_int8_tops_" + label] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    src = torch.empty(1 << 30, dtype=torch.int8, device="cuda:0")
    dst = torch.empty(1 << 30, dtype=torch.int8, device="cuda:0")
    for _ in range(3):
        probes.sqp_copy(src, dst)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        probes.sqp_copy(src, dst)
    e1.record()
    torch.cuda.synchronize()
    out["device_copy_gbs_read_plus_write"] = round(5 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del src, dst
    # launch floors: [back to back, single launch between its own events], microseconds
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    floors = {}
    for label, (grid, block, lds) in {"one_workgroup_64_threads": (1, 64, 0),
                                     "one_workgroup_per_cu_256_threads_144KiB_lds": (cus, 256, 144 * 1024),
                                     "one_workgroup_per_cu_1024_threads_156KiB_lds": (cus, 1024, 156 * 1024),
                                     "2304_workgroups_256_threads": (2304, 256, 0),
                                     "17280_workgroups_256_threads": (17280, 256, 0)}.items():
        fn = lambda: probes.sqp_launch(grid, block, lds)
        b2b, single = _timed_launches(fn)
        floors[label] = {"gpu_side": round(_gpu_side_ms([fn]) * 1e3, 2), "from_python_back_to_back": round(b2b * 1e3, 2),
                         "from_python_single_between_events": round(single * 1e3, 2)}
    buf_a = torch.zeros(cus * 1024, dtype=torch.int32, device="cuda:0")
    buf_b = torch.zeros(cus * 1024, dtype=torch.int32, device="cuda:0")
    fn = lambda: probes.sqp_roundtrip(buf_a, buf_b, cus, 1024)
    b2b, single = _timed_launches(fn)
    floors["one_memory_round_trip_1024_threads_per_cu"] = {"gpu_side": round(_gpu_side_ms([fn]) * 1e3, 2),
                                                           "from_python_back_to_back": round(b2b * 1e3, 2),
                                                           "from_python_single_between_events": round(single * 1e3, 2)}
    out["launch_floor_us"] = floors
    return out


def cpu_baseline(name, budget_s=15.0):
    """The CPU oracle, as it stands, on a bounded sample of the workload's token rows."""
    import oracle
    from paper_2507_14811_amd import workloads as wl

    oracle.build()
    w = wl.make(name)
    wq, ws = oracle.quantize_weight(w.w, w.kseg_off)
    probe = min(w.M, 8)
    xp, xn = oracle.quantize_act(w.x[:probe], w.kseg_off, w.dual, w.s_pos, w.s_neg)
    t0 = time.perf_counter()
    oracle.int_gemm(xp, xn, wq, w.kseg_off, w.dual)
    per_row = max((time.perf_counter() - t0) / probe, 1e-6)
    rows = int(max(probe, min(w.M, budget_s / per_row)))
    xs = np.ascontiguousarray(w.x[:rows])
    t0 = time.perf_counter()
    xp, xn = oracle.quantize_act(xs, w.kseg_off, w.dual, w.s_pos, w.s_neg)
    ap, an = oracle.int_gemm(xp, xn, wq, w.kseg_off, w.dual)
    y32, _ = oracle.dequant(ap, an, w.nseg_off, w.dual, w.s_pos, w.s_neg, ws, w.seg_scale, w.bias, want64=False)
    oracle.cast_bf16(y32)
    dt = time.perf_counter() - t0
    ops = 2.0 * rows * w.N * w.keff
    return {"value": ops / dt / 1e12, "unit": "int8 TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {w.M} token rows of {w.name}: quantize_act + integer GEMM + dequant + bf16 cast, "
                      f"{dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="cfg5", help="headline workload (cfg2 | cfg4 | cfg4d | cfg5)")
    ap.add_argument("--others", default="cfg2,cfg3,cfg3x28,cfg4,cfg4d", help="extra workloads summarised in the same line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", type=int, default=-1, help="force an MFMA tile variant (diagnostics)")
    ap.add_argument("--no-graph", action="store_true", help="no HIP graphs: small kernels are timed with plain launches "
                    "(host launch cost included); for runs under rocprofv3")
    ap.add_argument("--fp8-only", action="store_true", help="time only the 8-bit floating-point variant and print its JSON object "
                    "(the command of the fp8 profile passes)")
    ap.add_argument("--only", default="", help="time this one workload (hot path only) and print a short JSON line: "
                    "one workload per profiler pass")
    args = ap.parse_args()
    global USE_GRAPHS
    USE_GRAPHS = not args.no_graph
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(token rows are independent: a second GPU would take its own share of M, with no exchange)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2507_14811_amd as sq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    sq.load_library()
    if args.variant >= 0:
        sq.sq_tuning_set("gemm_variant", args.variant)

    # One plain device copy of known size (256 MiB read + 256 MiB written): under rocprofv3 --pmc it gives
    # the reading of FETCH_SIZE / WRITE_SIZE for a known traffic, which scales the kernels' readings.
    from paper_2507_14811_amd import probes

    if args.fp8_only:
        probes.sqp_copy(torch.zeros(256 << 20, dtype=torch.int8, device="cuda:0"), torch.empty(256 << 20, dtype=torch.int8, device="cuda:0"))
        print(json.dumps(measure_fp8((args.config,) + tuple(n for n in ("cfg4", "cfg2", "cfg3x28") if n in args.others.split(",") and n != args.config))))
        return
    if args.only:
        r = measure(args.only, args.steps, args.warmup, hot_only=True)
        print(json.dumps({"workload": r["name"], "ms_quantize_act": round(r["ms_quant"], 5), "ms_seglinear": round(r["ms_gemm_b2b"], 5),
                          "ms_seglinear_from_hbm": None if r["ms_gemm_hbm"] is None else round(r["ms_gemm_hbm"], 5)}))
        return

    cal_src = torch.zeros(256 << 20, dtype=torch.int8, device="cuda:0")
    cal_dst = torch.empty_like(cal_src)
    probes.sqp_copy(cal_src, cal_dst)      # probe_copy_kernel: 256 MiB fetched, 256 MiB written
    torch.cuda.synchronize()
    del cal_src, cal_dst

    head = measure(args.config, args.steps, args.warmup)
    dual_cols = head.pop("xq_dual_cols")
    ceilings = measured_ceilings(head.pop("xq_codes"), dual_cols)
    del dual_cols
    grouped = measure_grouped() if "cfg3" in args.others.split(",") else None
    w4 = measure_w4() if "cfg3x28" in args.others.split(",") else None
    geglu = measure_geglu()
    optimizer_side = measure_optimizer_side(args.config)
    fp8 = measure_fp8((args.config,) + tuple(n for n in ("cfg4", "cfg2", "cfg3x28") if n in args.others.split(",") and n != args.config))
    others = {}
    for name in [n for n in args.others.split(",") if n and n != args.config]:
        sq.sq_tuning_set("gemm_variant", -1)
        r = measure(name, max(10, args.steps // 2), max(3, args.warmup // 2), hot_only=True)
        skinny = r["M"] <= 64
        others[name] = {
            "M": r["M"], "K": r["K"], "N": r["N"], "ms_gemm_in_step": round(r["ms_gemm"], 5),
            "ms_gemm": round(r["ms_gemm_b2b"], 5), "ms_quant": round(r["ms_quant"], 5),
            "gemm_tops": round(r["gemm_tops_b2b"], 2), "gemm_frac_mfma_peak": round(r["gemm_tops_b2b"] / INT8_MFMA_PEAK_TOPS, 4),
            "gemm_gbs": round(r["gemm_gbs_b2b"], 1), "gemm_frac_hbm_peak": round(r["gemm_gbs_b2b"] / HBM_PEAK_GBS, 4),
            "gemm_bound": "hbm" if skinny else "mfma",
            "quant_gbs": round(r["quant_gbs"], 1), "quant_frac_hbm_peak": round(r["quant_gbs"] / HBM_PEAK_GBS, 4),
            "quant_bytes": r["quant_bytes"], "ms_quant_launched_from_python": round(r["ms_quant_stream"], 5),
            "ms_quantize_weight": round(r["ms_quantize_weight"], 5),
        }
        if skinny:   # the stream from HBM (rotation over distinct weight sets) is the figure for the HBM roofline
            others[name].update({
                "weight_sets_rotated": r["weight_sets"], "ms_gemm_from_hbm": round(r["ms_gemm_hbm"], 5),
                "ms_gemm_from_hbm_launched_from_python": round(r["ms_gemm_hbm_stream"], 5), "gemm_bytes": r["gemm_bytes"],
                "gemm_gbs_from_hbm": round(r["gemm_gbs_hbm"], 1),
                "gemm_frac_hbm_peak_from_hbm": round(r["gemm_gbs_hbm"] / HBM_PEAK_GBS, 4),
                "gemm_gbs_cache_resident": round(r["gemm_gbs_b2b"], 1)})

    for name, o in others.items():
        o["quant_traffic"] = MEASURED_TRAFFIC_QUANT.get(name)
        if o["gemm_bound"] == "hbm":
            o["gemm_traffic"] = MEASURED_TRAFFIC_SKINNY.get(name)
    floors = ceilings["launch_floor_us"]
    for name, o in others.items():
        if o["gemm_bound"] == "hbm":
            # a skinny layer is one launch of one workgroup per compute unit (1024 threads, the whole LDS): what that
            # launch costs empty, and with one trip to memory, next to what the layer takes (all GPU-side)
            o["launch_floor_us"] = floors["one_workgroup_per_cu_1024_threads_156KiB_lds"]["gpu_side"]
            o["one_round_trip_floor_us"] = floors["one_memory_round_trip_1024_threads_per_cu"]["gpu_side"]
            o["gemm_us_over_round_trip_floor"] = round(o["ms_gemm_from_hbm"] * 1e3 / max(o["one_round_trip_floor_us"], 1e-3), 2)
            # the most a single launch of this layer can reach: its bytes at the HBM peak behind one round trip
            best_us = o["one_round_trip_floor_us"] + o["gemm_bytes"] / (HBM_PEAK_GBS * 1e3)
            o["frac_hbm_peak_reachable_by_one_launch"] = round(o["gemm_bytes"] / (best_us * 1e3) / HBM_PEAK_GBS, 4)
    line = {
        "metric": "int8 TOPS (both dual paths) of SegLinear+DualScale GEMM; % int8 MFMA peak",
        "value": round(head["step_tops"], 3),
        "unit": "int8 TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(head["ms_step"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": head["name"], "M": head["M"], "K": head["K"], "N": head["N"],
                   "k_segments": head["S"], "n_segments": head["T"], "dual": head["dual"],
                   "step": "sq_quantize_act + sq_seglinear (bf16 in, bf16 out); weights pre-quantized",
                   "preroll_ms": PREROLL_MS},
        "roofline": {
            "kernel": "seglinear_mfma_kernel",
            "bound": "mfma",
            "achieved": round(head["gemm_tops"], 2),
            "peak": INT8_MFMA_PEAK_TOPS,
            "unit": "TOP/s",
            "frac": round(head["gemm_tops"] / INT8_MFMA_PEAK_TOPS, 4),
            "ms_per_launch": round(head["ms_gemm"], 5),
            "ms_per_launch_back_to_back": round(head["ms_gemm_b2b"], 5),
            "traffic": MEASURED_TRAFFIC.get(head["name"]),
            "frac_of_measured_mfma_ceiling": round(head["gemm_tops"] / max(ceilings["mfma_int8_tops_layer_like_operands"], 1e-9), 4),
        },
        "quantize_act": {"bound": "hbm", "achieved": round(head["quant_gbs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(head["quant_gbs"] / HBM_PEAK_GBS, 4), "ms_per_launch": round(head["ms_quant"], 5),
                         "bytes": head["quant_bytes"], "traffic": MEASURED_TRAFFIC_QUANT.get(args.config)},
        "quantize_act_fused": {"bound": "hbm", "activation": "GELU (tanh form) on the dual K-segments",
                               "path": "code tables in LDS (bf16 input, two launches: table fill + stream)",
                               "ms_per_call": round(head["ms_quant_fused_lut"], 5),
                               "achieved": round(head["quant_bytes"] / (head["ms_quant_fused_lut"] * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": round(head["quant_bytes"] / (head["ms_quant_fused_lut"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                               "bytes": head["quant_bytes"],
                               "ms_per_launch_arithmetic_path": round(head["ms_quant_fused"], 5)},
        "quantize_act_geglu": geglu,
        "dynamic_token_steps": {"workload": head["name"], "ms_quantize_act_dynamic": None if head["ms_quant_dyn"] is None else round(head["ms_quant_dyn"], 5),
                                "ms_seglinear_dynamic": None if head["ms_gemm_dyn"] is None else round(head["ms_gemm_dyn"], 5),
                                "note": "per-token steps written by the quantizer and read by the GEMM's flushes; 8-bit weights"},
        "quantize_weight_ms": round(head["ms_quantize_weight"], 5),
        "quantize_weight_block_ms": round(head["ms_quantize_weight_block"], 5),
        "calibrate_act": {"bound": "hbm", "ms_per_call": round(head["ms_calibrate"], 5), "achieved": round(head["calib_gbs"], 1),
                          "unit": "GB/s", "frac": round(head["calib_gbs"] / HBM_PEAK_GBS, 4),
                          "note": "three launches (init, max-reduce, steps); cfg5's activations fit the Infinity Cache"},
        "calibrate_act_percentile": {"p": 0.9999, "ms_per_call": round(head["ms_calibrate_percentile"], 5),
                                     "note": "exact radix select: one histogram pass over the activations per 8 bits "
                                             "(two for bf16 input), each followed by a bin-select kernel"},
        "other_workloads": others,
        "grouped_skinny": grouped,
        "w4_skinny": w4,
        "optimizer_side": optimizer_side,
        "fp8_variant": fp8,
        "measured_ceilings": ceilings,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(args.config)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
