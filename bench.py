#!/usr/bin/env python3
"""Benchmark of the BRA forward hot path on one MI355X.

A "step" is one bra_forward call (every step of the path: routing, projections,
routed attention, LCE, output projection) over one batch of the stage-1 BiFormer
shape (B=64, 56x56 map, C=64, 2 heads, S=7, k=1, bf16), inputs resident in HBM.
Prints ONE JSON line.  The line also carries: the roofline figures of the kernel
that takes the most time (timed live with events on the launch stream), the CPU
oracle's rate on a bounded sample of the same workload, and the throughput of the
other named workloads.
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

METRIC = "BRA fwd images/sec per stage shape + achieved TFLOP/s and HBM GB/s"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
VALU_F32_PEAK_TFLOPS = 157.3
CALIBRATION_BYTES = 64 << 20
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 counter
    summary (profiles/hbm_traffic.txt, written by traffic_summary.py),
    or None if there is no entry."""
    try:
        with open(TRAFFIC_FILE) as f:
            for ln in f:
                parts = ln.split()
                if len(parts) >= 4 and parts[0] == "traffic" and parts[1] == workload and parts[2] == kernel:
                    return int(float(parts[3]))
    except OSError:
        pass
    return None


def flops_per_image(cfg):
    """Algorithmic flops of one image (2 per multiply-add): projections (Eq. 3),
    region pooling + routing (Eq. 4), attention (Eq. 7), LCE, W^o (Eq. 2)."""
    N, C, R, n, kn = cfg.H * cfg.W, cfg.C, cfg.R, cfg.n, cfg.kn
    proj = 6 * N * C * C
    pool = N * C + 4 * R * C * C
    aff = 2 * R * R * C
    attn = 4 * N * kn * C
    lce = 50 * N * C
    wo = 2 * N * C * C
    return dict(proj=proj, pool=pool, aff=aff, attn=attn, lce=lce, wo=wo,
                total=proj + pool + aff + attn + lce + wo)


def kernel_model(name, cfg):
    """(bound, work per launch, unit of `achieved`, peak) of one library kernel.

    HBM-bound kernels are priced on their ALGORITHMIC bytes: unit = N*C*eb bytes
    per image (one pass over a token tensor in the storage type)."""
    eb = 2 if cfg.dtype == "bf16" else 4
    unit = cfg.H * cfg.W * cfg.C * eb * cfg.B
    f = flops_per_image(cfg)
    B = cfg.B
    # the attention kernels: priced on bytes where the routed keys are few (HBM / L2 gather bound),
    # on matrix-core flops where the arithmetic intensity of their share of the layer lies beyond
    # the ridge of the chip (many keys per query: the 128x128 and the S = 16 shapes)
    attn_flops = B * (f["attn"] + f["lce"] + f["wo"])
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    attn = ("mfma", attn_flops, MFMA_BF16_PEAK_TFLOPS) if attn_flops / (4.0 * unit) > ridge else ("hbm", 4 * unit, HBM_PEAK_GBS)
    table = {
        # generic (VALU float32) family
        "gen_pool": ("hbm", unit, HBM_PEAK_GBS),
        "gen_region_qk": ("alu", B * 4 * cfg.R * cfg.C * cfg.C, VALU_F32_PEAK_TFLOPS),
        "gen_affinity_topk": ("alu", B * f["aff"], VALU_F32_PEAK_TFLOPS),
        "gen_gemm_qkv": ("alu", B * f["proj"], VALU_F32_PEAK_TFLOPS),
        "gen_attention": ("alu", B * f["attn"], VALU_F32_PEAK_TFLOPS),
        "gen_lce_add": ("alu", B * f["lce"], VALU_F32_PEAK_TFLOPS),
        "gen_gemm_wo": ("alu", B * f["wo"], VALU_F32_PEAK_TFLOPS),
        # matrix-core family
        "mfma_prep": ("hbm", 2 * 4 * cfg.C * cfg.C * eb, HBM_PEAK_GBS),    # weights in and out
        "mfma_pool_qk": ("hbm", unit, HBM_PEAK_GBS),                   # reads X once
        "mfma_route_rows": ("alu", B * f["aff"], VALU_F32_PEAK_TFLOPS),
        "mfma_route": ("alu", B * (4 * cfg.R * cfg.C * cfg.C + f["aff"]), VALU_F32_PEAK_TFLOPS),
        "mfma_qkv": ("hbm", 4 * unit, HBM_PEAK_GBS),                   # X in, Q K V out
        "mfma_attention": attn,                                        # Q K V in, Y out
        "mfma_fused_k1": ("hbm", 2 * unit, HBM_PEAK_GBS),              # X in, Y out
        "mfma_attn_small": ("hbm", 4 * unit, HBM_PEAK_GBS),            # Q K V in, O out
        "mfma_lce_add": ("hbm", 3 * unit, HBM_PEAK_GBS),               # O V in, O out
        "mfma_wo": ("hbm", 2 * unit, HBM_PEAK_GBS),                    # O in, Y out
    }
    return table[name]


def device_inputs(cfg, sets, smooth=False):
    import numpy as np
    import torch

    from synthetic_inputs import bf16_bits, make_config_inputs

    X, Wqkv, Wo, Wlce = make_config_inputs(cfg, smooth=smooth)

    def dev(a):
        if cfg.dtype == "bf16":
            return torch.from_numpy(bf16_bits(a).view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    Xd = dev(X)
    # rotating input/output sets so that the footprint exceeds the 256 MB last-level cache
    Xs = [Xd] + [torch.roll(Xd, shifts=i, dims=0).contiguous() for i in range(1, sets)]
    Ys = [torch.empty_like(Xd) for _ in range(sets)]
    return (X, Wqkv, Wo, Wlce), Xs, Ys, dev(Wqkv), dev(Wo), dev(Wlce)


_RAMP = {}


def ramp_clocks(ms=60.0):
    """Keeps the GPU busy for about `ms` milliseconds with the library's probe kernels (a streaming copy
    and a register-only matrix-core loop; none of the workload's kernels), so that a measurement with
    few warm-up steps does not start on the idle clocks: with 5 warm-up steps alone, 20 timed steps of
    workload 2 read 51 us per step; after 500 warm-up steps, 45."""
    import torch

    import paper_2303_08810_amd as bra

    if not _RAMP:
        _RAMP["src"] = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").random_()
        _RAMP["dst"] = torch.empty_like(_RAMP["src"])
        _RAMP["scratch"] = torch.zeros(4, dtype=torch.float32, device="cuda")
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(8):
            bra.util_copy(_RAMP["dst"], _RAMP["src"])
            bra.util_mfma32(256 * 4, 200, _RAMP["scratch"])
        torch.cuda.synchronize()


def time_config(cfg, steps, warmup, profile=True):
    import torch

    import paper_2303_08810_amd as bra

    unit_mb = cfg.B * cfg.H * cfg.W * cfg.C * (2 if cfg.dtype == "bf16" else 4) / 1e6
    sets = max(2, min(24, int(600 / (2 * unit_mb)) + 1))
    host, Xs, Ys, Wqkv, Wo, Wlce = device_inputs(cfg, sets)
    shape = bra.make_shape(cfg.B, cfg.H, cfg.W, cfg.C, cfg.heads, cfg.S, cfg.k, Xs[0].dtype)
    ws = bra.alloc_workspace(shape, Xs[0].device)

    def step(i):
        bra.bra_forward(Xs[i % sets], Wqkv, Wo, Wlce, cfg.S, cfg.k, cfg.heads, ws=ws, out=Ys[i % sets])

    if warmup < 200:
        ramp_clocks()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = max(wall_ms, ev_ms) / steps

    kernels = {}
    if profile:
        # the same K steps again, every kernel launch bracketed by two events on the stream
        per_step = 16
        bra.profile_begin(steps * per_step)
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        for name, ms in bra.profile_end(steps * per_step):
            k = kernels.setdefault(name, [0, 0.0])
            k[0] += 1
            k[1] += ms
    return dict(ms_per_step=ms_per_step, wall_ms=wall_ms, event_ms=ev_ms, kernels=kernels,
                host=host, sets=sets)


def time_block(cfg, steps, warmup, expansion=3):
    """One whole block (position encoding, LayerNorm, BRA, LayerNorm, MLP with e = 3) at a named
    workload's shape: context beside the headline figure, never `value`."""
    import numpy as np
    import torch

    import paper_2303_08810_amd as bra
    from synthetic_inputs import bf16_bits, make_block_inputs

    X, P = make_block_inputs(cfg, expansion=expansion)
    if cfg.dtype == "bf16":
        bf = lambda a: torch.from_numpy(bf16_bits(a).view(np.int16)).view(torch.bfloat16).cuda()
    else:
        bf = lambda a: torch.from_numpy(a).cuda()
    dP = {n: (bf(P[n]) if n in bra.BraBlockParams.MATRICES else torch.from_numpy(P[n]).cuda())
          for n in bra.BraBlockParams.FIELDS}
    Xd = bf(X)
    unit_mb = Xd.numel() * Xd.element_size() / 1e6
    sets = max(2, min(24, int(600 / (2 * unit_mb)) + 1))
    Xs = [Xd] + [torch.roll(Xd, shifts=i, dims=0).contiguous() for i in range(1, sets)]
    Ys = [torch.empty_like(Xd) for _ in range(sets)]
    shape = bra.make_shape(cfg.B, cfg.H, cfg.W, cfg.C, cfg.heads, cfg.S, cfg.k, Xd.dtype)
    hidden = expansion * cfg.C
    ws = torch.empty(bra.block_workspace_bytes(shape, hidden), dtype=torch.uint8, device="cuda")

    def step(i):
        bra.bra_block_forward(Xs[i % sets], dP, cfg.S, cfg.k, cfg.heads, ws=ws, out=Ys[i % sets])

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    ms = max((time.perf_counter() - t0) * 1e3, e0.elapsed_time(e1)) / steps
    bra.profile_begin(steps * 24)
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    kernels = {}
    for name, t in bra.profile_end(steps * 24):
        kernels[name] = kernels.get(name, 0.0) + t
    tokens = cfg.B * cfg.H * cfg.W
    mlp_flops = 4.0 * tokens * cfg.C * hidden
    bra_flops = cfg.B * flops_per_image(cfg)["total"]
    # algorithmic traffic: X in, Xout out; everything between them could stay on the chip
    return {
        "images_per_s": round(cfg.B / (ms / 1e3), 1), "ms_per_step": round(ms, 5), "expansion": expansion,
        "achieved_tflops": round((mlp_flops + bra_flops) / (ms / 1e3) / 1e12, 3),
        "min_traffic_gbs": round(2 * Xd.numel() * Xd.element_size() / (ms / 1e3) / 1e9, 1),
        "kernels_avg_us": {k: round(1e3 * v / steps, 2) for k, v in kernels.items()},
    }


def time_padded(steps, warmup):
    """bra_forward_padded on a detection-like first-stage map that S = 16 does not divide
    (B = 2, 200 x 300, C = 64, k = 4; padded to 208 x 304 inside): context, never `value`."""
    import numpy as np
    import torch

    import paper_2303_08810_amd as bra
    from synthetic_inputs import BASE_SEED, bf16_bits, make_inputs

    B, H, W, C, heads, S, k = 2, 200, 300, 64, 2, 16, 4
    arrs = make_inputs(B, H, W, C, seed=BASE_SEED + 100, dtype="bf16")
    X, Wqkv, Wo, Wlce = (torch.from_numpy(bf16_bits(a).view(np.int16)).view(torch.bfloat16).cuda() for a in arrs)

    def step():
        bra.bra_forward_padded(X, Wqkv, Wo, Wlce, S, k, heads)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return {"workload": f"B={B} H={H} W={W} C={C} heads={heads} S={S} k={k} bf16, padded to 208x304",
            "images_per_s": round(B / (ms / 1e3), 1), "ms_per_step": round(ms, 5),
            "note": "includes the binding's workspace and output allocation per call"}


def time_backward(cfg, steps, warmup):
    """bra_backward (fixed routing) at a named workload's shape, with the workspace allocated once
    and HIP events around the timed calls: context, never `value`.  bf16 workloads with heads of 32
    or 64 channels, C a multiple of 64 and at most 4096 routing entries per image run on the
    matrix-core kernels, the others on the scalar float32 ones."""
    import ctypes

    import torch

    import paper_2303_08810_amd as bra

    host, Xs, Ys, Wqkv, Wo, Wlce = device_inputs(cfg, 2)
    X = Xs[0]
    Y, Ir = bra.bra_forward(X, Wqkv, Wo, Wlce, cfg.S, cfg.k, cfg.heads, want_Ir=True)
    dY = torch.randn_like(Y.float()).to(Y.dtype)
    shape = bra.make_shape(cfg.B, cfg.H, cfg.W, cfg.C, cfg.heads, cfg.S, cfg.k, X.dtype)
    need = ctypes.c_size_t(0)
    bra._check(bra.lib().bra_backward_workspace_bytes(ctypes.byref(shape), ctypes.byref(need)))
    ws = torch.empty(need.value, dtype=torch.uint8, device="cuda")
    for _ in range(warmup):
        bra.bra_backward(X, Wqkv, Wo, Wlce, Ir, dY, cfg.S, cfg.heads, ws=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        bra.bra_backward(X, Wqkv, Wo, Wlce, Ir, dY, cfg.S, cfg.heads, ws=ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    f = flops_per_image(cfg)
    mfma = (cfg.dtype == "bf16" and cfg.C % 64 == 0 and cfg.C // cfg.heads in (32, 64)
            and cfg.S * cfg.S * cfg.k <= 4096)
    # the backward pass recomputes the forward (1x) and does about twice its arithmetic again
    return {"images_per_s": round(cfg.B / (ms / 1e3), 1), "ms_per_step": round(ms, 4),
            "achieved_tflops": round(3 * cfg.B * f["total"] / (ms / 1e3) / 1e12, 3),
            "kernels": "matrix-core (bf16 operands, float32 sums)" if mfma
                       else "scalar float32 with atomic scatter-add",
            "note": "includes the binding's output allocations"}


def time_variants(cfg, steps, warmup):
    """Further timings of the same workload, for context (none of them is `value`): repeats of
    the K-step measurement, spatially smooth inputs (concentrated routing), a single input
    set (everything stays in the last-level cache), replay of a HIP graph that holds one
    pass over the rotating input sets, and independent forwards alternating between two streams."""
    import statistics

    import torch

    import paper_2303_08810_amd as bra

    def measure(sets, smooth=False, graph=False):
        host, Xs, Ys, Wqkv, Wo, Wlce = device_inputs(cfg, sets, smooth=smooth)
        shape = bra.make_shape(cfg.B, cfg.H, cfg.W, cfg.C, cfg.heads, cfg.S, cfg.k, Xs[0].dtype)
        ws = bra.alloc_workspace(shape, Xs[0].device)

        def step(i):
            bra.bra_forward(Xs[i % sets], Wqkv, Wo, Wlce, cfg.S, cfg.k, cfg.heads, ws=ws, out=Ys[i % sets])

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        launch, per_launch = step, 1
        if graph:
            side = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for i in range(sets):
                        step(i)
            torch.cuda.synchronize()
            launch, per_launch = (lambda i: g.replay()), sets
        times = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n = max(1, steps // per_launch)
            e0.record()
            for i in range(n):
                launch(i)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) / (n * per_launch))
        return times

    def measure_two_streams(sets):
        """Independent forwards alternate between two streams, each with a workspace of its own:
        one call's drain overlaps the next call's fill (what a serving loop with two requests in
        flight would see).  Wall-clock over all steps, both streams drained at both ends."""
        host, Xs, Ys, Wqkv, Wo, Wlce = device_inputs(cfg, sets)
        shape = bra.make_shape(cfg.B, cfg.H, cfg.W, cfg.C, cfg.heads, cfg.S, cfg.k, Xs[0].dtype)
        wss = [bra.alloc_workspace(shape, Xs[0].device) for _ in range(2)]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]       # default priority

        def run(n):
            for i in range(n):
                with torch.cuda.stream(streams[i % 2]):
                    bra.bra_forward(Xs[i % sets], Wqkv, Wo, Wlce, cfg.S, cfg.k, cfg.heads, ws=wss[i % 2],
                                    out=Ys[i % sets])

        torch.cuda.synchronize()
        run(warmup)
        torch.cuda.synchronize()
        times = []
        for _ in range(5):
            t0 = time.perf_counter()
            run(steps)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) * 1e3 / steps)
        return times

    unit_mb = cfg.B * cfg.H * cfg.W * cfg.C * (2 if cfg.dtype == "bf16" else 4) / 1e6
    sets = max(2, min(24, int(600 / (2 * unit_mb)) + 1))
    rot = measure(sets)
    out = {"repeats_ms_per_step": [round(t, 5) for t in rot],
           "median_ms_per_step": round(statistics.median(rot), 5), "min_ms_per_step": round(min(rot), 5),
           "smooth_inputs_median_ms_per_step": round(statistics.median(measure(sets, smooth=True)), 5),
           "hot_cache_median_ms_per_step": round(statistics.median(measure(1)), 5),
           "graph_replay_median_ms_per_step": round(statistics.median(measure(sets, graph=True)), 5),
           "two_streams_median_ms_per_step": round(statistics.median(measure_two_streams(sets)), 5)}
    return out


def measured_peaks():
    """What plain streaming kernels reach on this GPU, beside the published HBM peak the roofline
    uses: a copy and a read of 512 MiB (twice the last-level cache); and what the matrix cores reach
    on register operands with each of the two dense bf16 instruction shapes, beside the published
    2.5 PFLOP/s."""
    import torch

    import paper_2303_08810_amd as bra

    nbytes = 512 << 20
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_()
    dst = torch.empty_like(src)
    scratch = torch.zeros(4, dtype=torch.float32, device="cuda")

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps / 1e3

    t_copy = timed(lambda: bra.util_copy(dst, src), 20)
    t_read = timed(lambda: bra.util_read(src, scratch), 20)
    # matrix cores: 8 workgroups of 4 wavefronts per compute unit, register operands only
    wgs, iters = 256 * 8, 4000
    t16 = timed(lambda: bra.util_mfma(wgs, iters, scratch), 3)
    t32 = timed(lambda: bra.util_mfma32(wgs, iters, scratch), 3)
    return {"hbm_copy_GBs": round(2 * nbytes / t_copy / 1e9, 1), "hbm_read_GBs": round(nbytes / t_read / 1e9, 1),
            "mfma_bf16_16x16x32_TFLOPs": round(wgs * 4 * 8 * iters * 16384 / t16 / 1e12, 1),
            "mfma_bf16_32x32x16_TFLOPs": round(wgs * 4 * 4 * iters * 32768 / t32 / 1e12, 1)}


def roofline_of(cfg, kernels):
    if not kernels:
        return None, {}
    summary = {n: dict(launches=c, avg_us=1e3 * t / c) for n, (c, t) in kernels.items()}
    name = max(kernels, key=lambda n: kernels[n][1])
    bound, work, peak = kernel_model(name, cfg)
    avg_s = kernels[name][1] / kernels[name][0] / 1e3
    if bound == "hbm":
        achieved, unit = work / avg_s / 1e9, "GB/s"
    else:
        achieved, unit = work / avg_s / 1e12, "TFLOP/s"
    roof = dict(kernel=name, bound=bound, achieved=round(achieved, 2), peak=peak, unit=unit,
                frac=round(achieved / peak, 4), traffic=measured_traffic(name, cfg.name),
                avg_us=round(avg_s * 1e6, 2), work_per_launch=work)
    return roof, summary


def step_roofline(cfg, ms_per_step):
    """The whole step against both roofs: the bytes a perfectly fused layer has to move (X in, Y
    out) and the layer's flops, over the measured time of one step."""
    eb = 2 if cfg.dtype == "bf16" else 4
    nbytes = 2 * cfg.B * cfg.H * cfg.W * cfg.C * eb
    flops = cfg.B * flops_per_image(cfg)["total"]
    t = ms_per_step / 1e3
    peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else VALU_F32_PEAK_TFLOPS
    return {"min_bytes": nbytes, "hbm_frac": round(nbytes / t / 1e9 / HBM_PEAK_GBS, 4), "flops": flops,
            "flops_frac": round(flops / t / 1e12 / peak, 4),
            "flops_peak": "bf16 mfma" if cfg.dtype == "bf16" else "fp32 vector"}


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, host, budget_s=12.0):
    """The oracle (float32 instance, as it stands) on the host cores, on whole
    images taken from the same batch; OpenMP over images."""
    import numpy as np

    import oracle

    X, Wqkv, Wo, Wlce = host
    threads = max(1, min(16, os.cpu_count() or 1))
    kw = dict(S=cfg.S, k=cfg.k, heads=cfg.heads, precision="f32", threads=threads)
    n0 = min(threads, X.shape[0])
    t0 = time.perf_counter()
    oracle.bra_forward(X[:n0], Wqkv, Wo, Wlce, **kw)
    t_probe = time.perf_counter() - t0
    # whole images per call: bounded by memory (about 1 GiB of float32 inputs), then repeated
    per_call = max(n0, min(X.shape[0], int((1 << 30) // (X[0].size * 4))) // n0 * n0)
    idx = np.arange(per_call) % X.shape[0]
    Xs = np.ascontiguousarray(X[idx])
    reps = int(max(1, min(200, round(budget_s / max(t_probe * per_call / n0, 1e-3)))))
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.bra_forward(Xs, Wqkv, Wo, Wlce, **kw)
    dt = time.perf_counter() - t0
    n_img = per_call * reps
    # the same oracle on one thread, on a few images (about 3 s)
    n1 = max(1, min(X.shape[0], int(3.0 / max(t_probe * threads / n0, 1e-3))))
    t0 = time.perf_counter()
    oracle.bra_forward(X[:n1], Wqkv, Wo, Wlce, S=cfg.S, k=cfg.k, heads=cfg.heads, precision="f32", threads=1)
    dt1 = time.perf_counter() - t0
    return dict(value=round(n_img / dt, 3), unit="images/s", cores=threads, kind="oracle",
                sample=f"{n_img} whole images of the same workload ({reps} passes over {per_call} images, "
                       f"float32 oracle, OpenMP over images), {dt:.1f} s",
                cpu_model=cpu_model(), host_cpus=os.cpu_count(),
                single_thread={"value": round(n1 / dt1, 3), "unit": "images/s", "cores": 1,
                               "sample": f"{n1} whole images, {dt1:.1f} s"})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=500)     # about 25 ms: the clocks have settled
    ap.add_argument("--workload", type=int, default=2, help="named workload index 1..5 (default 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other named workloads")
    ap.add_argument("--no-block", action="store_true",
                    help="skip the whole-block timings (position encoding, LayerNorm, BRA, MLP)")
    ap.add_argument("--block-same", action="store_true",
                    help="whole-block and backward timings for the chosen workload only (for counter runs)")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the context timings (repeats, smooth inputs, hot cache, graph replay)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the plain copy kernel (64 MiB, 10 times): the reference against "
                         "which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (images are independent; data "
              "parallelism over several GPUs needs no exchange and is not part of this build)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2303_08810_amd as bra
    from synthetic_inputs import CONFIGS, NEXT_CONFIGS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = CONFIGS[args.workload]
    res = time_config(cfg, args.steps, args.warmup)
    f = flops_per_image(cfg)
    ms = res["ms_per_step"]
    value = cfg.B / (ms / 1e3)
    roof, summary = roofline_of(cfg, res["kernels"])
    eb = 2 if cfg.dtype == "bf16" else 4
    line = {
        "metric": METRIC, "value": round(value, 1), "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} H=W={cfg.H} C={cfg.C} heads={cfg.heads} "
                               f"S={cfg.S} k={cfg.k} {cfg.dtype}", "rotating_input_sets": res["sets"]},
        "achieved_tflops": round(cfg.B * f["total"] / (ms / 1e3) / 1e12, 3),
        "min_traffic_gbs": round(2 * cfg.B * cfg.H * cfg.W * cfg.C * eb / (ms / 1e3) / 1e9, 1),
        "roofline": roof, "step_roofline": step_roofline(cfg, ms), "kernels": {k: {"launches": v["launches"], "avg_us": round(v["avg_us"], 2)}
                                      for k, v in summary.items()},
    }
    if not args.no_variants:
        line["variants"] = time_variants(cfg, args.steps, args.warmup)
        line["measured_peaks"] = measured_peaks()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, res["host"])
    if not args.no_others:
        others = {}
        for idx, c in {**CONFIGS, **NEXT_CONFIGS}.items():
            if idx == args.workload:
                continue
            r = time_config(c, max(20, args.steps // 4), max(5, args.warmup // 2), profile=True)
            fo = flops_per_image(c)
            rf, sm = roofline_of(c, r["kernels"])
            others[c.name] = {
                "images_per_s": round(c.B / (r["ms_per_step"] / 1e3), 1),
                "ms_per_step": round(r["ms_per_step"], 5),
                "achieved_tflops": round(c.B * fo["total"] / (r["ms_per_step"] / 1e3) / 1e12, 3),
                "step_roofline": step_roofline(c, r["ms_per_step"]),
                "dominant": rf,
                "kernels_avg_us": {k: round(v["avg_us"], 2) for k, v in sm.items()},
            }
        line["other_workloads"] = others
    if not args.no_block:
        # one whole block around BRA at every workload's shape (context, never `value`)
        blocks = {}
        for idx, c in {**CONFIGS, **NEXT_CONFIGS}.items():
            if args.block_same and idx != args.workload:
                continue
            n = args.steps if idx == args.workload else max(20, args.steps // 4)
            blocks[c.name] = time_block(c, n, n)
        line["block_forward"] = blocks
        if not args.block_same:
            line["padded_forward"] = time_padded(max(20, args.steps // 4), max(20, args.steps // 4))
        line["backward"] = {CONFIGS[i].name: time_backward(CONFIGS[i], 30, 10)
                            for i in ((args.workload,) if args.block_same else (1, 2, 3, 4, 5))}
    if args.calibrate:
        src = torch.empty(CALIBRATION_BYTES, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        for _ in range(10):
            bra.util_copy(dst, src)
        torch.cuda.synchronize()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
