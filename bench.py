#!/usr/bin/env python3
"""Benchmark of the OCS-expanded quantized layer on one MI355X.

A step is one pass of the whole hot path over one batch of the ResNet-style 3x3 convolution
(batch 64, 256->256 channels, 14x14, lowered by im2col: M=12544, K=2304, N=256, r=0.02,
8-bit weights and activations):

    ocs_split_weights   channel maxima of W, greedy selection, halve + quantize     (W1-W3)
    ocs_split_act       max|X| for the per-batch activation grid, then duplicate
                        the chosen channels, quantize, pack                         (X1, X2)
    ocs_qgemm           int8 MFMA GEMM over the expanded K, dequantizing epilogue   (G1, G2)

Inputs are resident in HBM before the timed region.  The activations rotate through several
copies so that no step finds its input in the 256 MB Infinity Cache.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
METRIC = "expanded int8 GEMM TOPS (% MFMA peak); split+quantize GB/s (% HBM)"

# HBM bytes per launch of the split+quantize kernel on this workload, from two rocprofv3 --pmc
# runs (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for the plain
# copy kernel of known size launched after the timed region (profiles/x2_config2_hbm_traffic.md).
# Valid only for the kernel source it was measured on: reported as null once that file changes.
X2_TRAFFIC = {"quantize_hip_sha256": "45a57b8aea8a8f6f2679f9a34efae37e9dacd2c5f5f7534957576038a29265f9",
              "bytes_per_launch": 146916747}


def x2_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_1901_09504_amd", "csrc", "quantize.hip")
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    return X2_TRAFFIC["bytes_per_launch"] if digest == X2_TRAFFIC["quantize_hip_sha256"] else None


def cpu_baseline(layer, W, X, budget_s=12.0, max_reps=100):
    """The CPU oracle, as it stands, on the same workload on this machine's host cores: whole
    steps on all rows, repeated for about budget_s seconds of CPU work."""
    from oracle import ref

    s = ref.num_splits(layer.C, layer.r)
    Ke = (layer.C + s) * layer.g
    ldq = (Ke + 63) // 64 * 64
    times = []
    t_all = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_all < budget_s and len(times) < max_reps):
        t0 = time.perf_counter()
        sp = ref.split_weights(W, layer.C, layer.g, s)
        Wq, sw = ref.quantize(sp["T_out"], layer.bits_w, ldq=ldq)
        Xq, sx, _ = ref.split_act(X, layer.C, layer.g, sp["chan_src"], None, s, layer.bits_x, ldq=ldq)
        ref.qgemm(Xq, Wq, Ke, sx[1], sw[1], want_acc=False)
        times.append(time.perf_counter() - t0)
    best, med = min(times), float(np.median(times))
    tops = 2.0 * X.shape[0] * layer.N * Ke / best / 1e12
    return {"value": tops, "unit": "TOPS", "cores": ref.get_threads(), "kind": "oracle",
            "sample": f"whole step on all {X.shape[0]} rows of the workload, best of {len(times)} "
                      f"({time.perf_counter() - t_all:.1f} s of CPU work)",
            "seconds_per_step": best, "seconds_per_step_median": med}


def mfma_bound_gemm(torch, B, wl, ExpandedLayer, launches, copies=5):
    """The GEMM alone on the one MFMA-bound layer shape of the paper's networks (ResNet-50's
    512->512 3x3 convolutions at batch 256, configs[4]): the workload's own GEMM sits on the
    HBM side of the ridge, so this is the launch that the "% of MFMA peak" figure can be read
    on.  Codes come from the library's own weight and activation passes on synthetic data; the
    activation codes rotate through several copies.  Every launch is timed by its own events."""
    layer = next(l for l in wl.config(5) if l.name == "s4b0_3x3")
    M, N = layer.M, layer.N
    Wd = torch.from_numpy(wl.weights(layer)).cuda()
    Xd = torch.from_numpy(wl.activations(layer)).cuda()
    L = ExpandedLayer(N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, max_rows=M)
    L.prepare_weights(Wd)
    L.split_act(Xd)
    torch.cuda.synchronize()
    del Xd
    Xq = [L.Xq.clone() for _ in range(copies)]
    stream = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in ev:
        e.record(stream)
    us = []
    for i in range(launches + 4):
        B.ocs_time_next(B.TIME_GEMM, ev[0], ev[1])
        B.ocs_qgemm(Xq[i % copies], L.ldq, L.Wq, L.ldq, M, N, L.Ke, L.bits_x, L.bits_w, L.scale_x,
                    L.scale_w, None, 0, L.Y, N, None, None)
        torch.cuda.synchronize()
        if i >= 4:
            us.append(ev[0].elapsed_time(ev[1]) * 1e3)
    avg = float(np.mean(us))
    ops = 2.0 * M * N * L.Ke
    return {"workload": f"configs[4] layer 512->512 3x3 at batch 256 as im2col GEMM: M={M} K'={L.Ke} "
                        f"(padded {L.ldq}) N={N}, {layer.bits_w}-bit weights, {layer.bits_x}-bit activations",
            "avg_launch_us": avg, "min_launch_us": float(np.min(us)), "launches_timed": len(us),
            "tops": ops / avg / 1e6, "pct_mfma_peak": 100.0 * ops / avg / 1e6 / INT8_PEAK_TOPS,
            "arithmetic_intensity_op_per_byte": ops / (M * L.Ke + N * L.Ke + 4.0 * M * N)}


def conv_unlowered(torch, B, wl, layer, steps, copies=24):
    """The workload's convolution given un-lowered (activation [64, 14, 14, 256] fp32, 12.8 MB,
    instead of its 115.6 MB im2col image): weight path + tap-major weights, split+quantize of the
    activation with a per-batch grid, convolution with the lowering inside the GEMM kernel's
    loader.  Reported beside the headline, which is defined on the lowered GEMM."""
    from paper_1901_09504_amd.layer import ExpandedConv

    Bn, H, W = 64, 14, 14
    Wd = torch.from_numpy(wl.weights(layer)).cuda()
    gen = torch.Generator(device="cuda").manual_seed(layer.seed)
    As = [torch.randn(Bn, H, W, layer.C, device="cuda", generator=gen).abs_() for _ in range(copies)]
    L = ExpandedConv(layer.N, layer.C, 3, 3, 1, 1, layer.r, layer.bits_w, layer.bits_x)

    def step(i):
        L.prepare_weights(Wd)
        L.forward(As[i % copies])

    for i in range(10):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    ops = 2.0 * Bn * H * W * layer.N * L.E * 9
    return {"workload": f"the same layer un-lowered: A [{Bn},{H},{W},{layer.C}] fp32 x {copies} rotating copies, "
                        f"3x3 stride 1 pad 1, K walked as 9 taps x {L.ldc} bytes",
            "us_per_step": us, "tops_whole_step": ops / us / 1e6, "steps": steps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--copies", type=int, default=6, help="rotating copies of X (6 x 115.6 MB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sample-every", type=int, default=8,
                    help="every n-th timed step carries the per-phase and per-kernel events")
    ap.add_argument("--mfma-gemm-launches", type=int, default=24,
                    help="launches of the GEMM on the MFMA-bound layer shape after the timed region (0: skip)")
    ap.add_argument("--graph-steps", type=int, default=200,
                    help="steps replayed from HIP graphs after the timed region (0: skip)")
    ap.add_argument("--conv-steps", type=int, default=100,
                    help="steps of the same layer given un-lowered, after the timed region (0: skip)")
    ap.add_argument("--calib-copies", type=int, default=6,
                    help="plain copies of X launched after the timed region (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1901_09504_amd import binding as B
    from paper_1901_09504_amd import workloads as wl
    from paper_1901_09504_amd.layer import ExpandedLayer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()  # fails loudly when libocs.so is missing

    (layer,) = wl.config(2)
    M, N, K = layer.M, layer.N, layer.K
    W = wl.weights(layer)
    X = wl.activations(layer)
    Wd = torch.from_numpy(W).cuda()
    Xd = [torch.from_numpy(X).cuda() for _ in range(max(1, args.copies))]
    L = ExpandedLayer(N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, max_rows=M)
    Ke, ldq = L.Ke, L.ldq
    stream = torch.cuda.current_stream()

    def step(i, ev=None, kev=None):
        x = Xd[i % len(Xd)]
        if ev: ev[0].record(stream)
        L.prepare_weights(Wd)
        if ev: ev[1].record(stream)
        if kev:
            B.ocs_time_next(B.TIME_ABSMAX, kev[4], kev[5])
            B.ocs_time_next(B.TIME_SPLIT_QUANTIZE, kev[0], kev[1])
        # per-batch grid: max|X| pass, then the split+quantize pass (one call, two kernels)
        B.ocs_split_act(x, M, L.C, L.g, K, L.chan_src, None, L.s, L.bits_x, None, 1.0, L.Xq, ldq,
                        L.scale_x, L.ws_x)
        if ev: ev[2].record(stream)
        if kev: B.ocs_time_next(B.TIME_GEMM, kev[2], kev[3])
        L.qgemm(M)
        if ev:
            ev[3].record(stream)
            ev[4].record(stream)   # ev[3] -> ev[4] brackets nothing: the cost of a bracket itself

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    # kernel events: stamped by the launch itself with the dispatch's begin and end (the two
    # dominant kernels only).  Recording them once creates their handles.
    kevents = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    for ke in kevents:
        for e in ke:
            e.record(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % args.sample_every == 0:
            step(i, events[i], kevents[i])
        else:
            step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3

    # after the timed region: plain copies of known size, so that a counter run of this same
    # command also holds the reference the HBM byte counters are scaled by
    dst = torch.empty_like(Xd[0])
    if args.calib_copies > 0:
        for i in range(args.calib_copies):
            B.ocs_calib_copy(Xd[i % len(Xd)], dst, Xd[0].numel() * 4)
        torch.cuda.synchronize()
    # the dominant kernel once more, cache-cold: inside a step it runs right after the pass that
    # takes max|X| over the same X, so part of its input comes from the 256 MB memory-side cache;
    # here nothing has touched the copy it reads for the last len(Xd) - 1 launches (static grid)
    cold_us = []
    cev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in cev:
        e.record(stream)
    for i in range(3 * len(Xd)):
        B.ocs_time_next(B.TIME_SPLIT_QUANTIZE, cev[0], cev[1])
        B.ocs_split_act(Xd[i % len(Xd)], M, L.C, L.g, K, L.chan_src, None, L.s, L.bits_x, L.scale_x, 1.0,
                        L.Xq, ldq, L.scale_x, L.ws_x)
        torch.cuda.synchronize()
        if i >= len(Xd):
            cold_us.append(cev[0].elapsed_time(cev[1]) * 1e3)
    sampled = list(range(0, args.steps, args.sample_every))
    phase = np.array([[events[i][k].elapsed_time(events[i][k + 1]) for k in range(4)] for i in sampled])  # ms
    raw = phase.mean(axis=0)
    bracket_ms = float(raw[3])       # an empty event pair, measured in the same timed region
    avg = np.maximum(raw[:3] - bracket_ms, 1e-6)
    names = ["split_weights", "split_act", "qgemm"]
    x2_kernel_ms = float(np.mean([kevents[i][0].elapsed_time(kevents[i][1]) for i in sampled]))
    gemm_kernel_ms = float(np.mean([kevents[i][2].elapsed_time(kevents[i][3]) for i in sampled]))
    x1_kernel_ms = float(np.mean([kevents[i][4].elapsed_time(kevents[i][5]) for i in sampled]))

    ops = 2.0 * M * N * Ke
    x2_bytes = 4.0 * M * K + 1.0 * M * Ke                       # X2: read fp32 X, write codes
    x1_bytes = 4.0 * M * K
    w_bytes = 8.0 * N * K + 1.0 * N * Ke                        # W1 + W3
    gemm_bytes = 1.0 * M * Ke + 1.0 * N * Ke + 4.0 * M * N
    x2_gbs = x2_bytes / (x2_kernel_ms * 1e-3) / 1e9
    gemm_tops = ops / (gemm_kernel_ms * 1e-3) / 1e12
    gemm_ai = ops / gemm_bytes
    gemm_roof_tops = min(INT8_PEAK_TOPS, gemm_ai * HBM_PEAK_GBS / 1e3)

    out = {
        "metric": METRIC,
        "value": ops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TOPS (2*M*N*K' of the expanded layer per second of whole-step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "dtype_detail": "int8 codes x int8 codes -> int32 accumulators; fp32 in, fp32 out",
        "data": "synthetic",
        "config": {"workload": "configs[1]: 3x3 conv 256->256, 14x14, batch 64 as im2col GEMM "
                               f"M={M} K={K} N={N}, r={layer.r} (s={L.s}, K'={Ke}, padded {ldq}), "
                               "8-bit weights and activations, weight OCS, per-batch activation grid",
                   "x_copies_rotated": len(Xd), "steps_carrying_events": len(sampled)},
        "gemm_tops": gemm_tops, "gemm_pct_mfma_peak": 100.0 * gemm_tops / INT8_PEAK_TOPS,
        "split_quant_gbps": x2_gbs, "split_quant_pct_hbm": 100.0 * x2_gbs / HBM_PEAK_GBS,
        "roofline": {"kernel": "expand_quantize_kernel (ocs_split_act, X2)", "bound": "hbm",
                     "achieved": x2_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": x2_gbs / HBM_PEAK_GBS, "traffic": x2_traffic(),
                     "algorithmic_bytes_per_launch": x2_bytes, "avg_launch_us": x2_kernel_ms * 1e3,
                     "timing": "HIP events stamped by the launch itself (hipExtLaunchKernel) on its "
                               "stream: the dispatch's own begin and end",
                     "launches_timed": len(sampled),
                     "cache_cold": {"avg_launch_us": float(np.mean(cold_us)),
                                    "achieved": x2_bytes / float(np.mean(cold_us)) / 1e3,
                                    "frac": x2_bytes / float(np.mean(cold_us)) / 1e3 / HBM_PEAK_GBS,
                                    "launches_timed": len(cold_us),
                                    "note": "same kernel after the timed region on copies of X that "
                                            "no launch has touched since 5 other copies were streamed "
                                            "(in the step it follows the max|X| pass over the same X, "
                                            "which leaves part of X in the 256 MB memory-side cache)"}},
        "phases": {n: {"avg_us": float(avg[k] * 1e3)} for k, n in enumerate(names)},
    }
    out["phases"]["split_weights"]["algorithmic_GBps"] = w_bytes / (avg[0] * 1e-3) / 1e9
    out["phases"]["split_act"].update({
        "what": "ocs_split_act with a per-batch grid: the max|X| pass, then the split+quantize pass",
        "absmax_kernel_us": x1_kernel_ms * 1e3,
        "absmax_algorithmic_GBps": x1_bytes / (x1_kernel_ms * 1e-3) / 1e9,
        "kernel_us": x2_kernel_ms * 1e3, "algorithmic_GBps": x2_gbs})
    out["phases"]["qgemm"]["kernel_us"] = gemm_kernel_ms * 1e3
    out["phase_timing"] = ("avg_us: HIP event brackets around each call minus an empty bracket "
                           f"({bracket_ms * 1e3:.2f} us here), includes dispatch gaps; kernel_us: the "
                           "kernel's own begin/end")
    out["phases"]["qgemm"].update({
        "tops": gemm_tops, "algorithmic_GBps": gemm_bytes / (gemm_kernel_ms * 1e-3) / 1e9,
        "arithmetic_intensity_op_per_byte": gemm_ai,
        "regime": "hbm" if gemm_ai < INT8_PEAK_TOPS * 1e3 / HBM_PEAK_GBS else "mfma",
        "roof_tops_min_mfma_hbm": gemm_roof_tops, "frac_of_that_roof": gemm_tops / gemm_roof_tops})
    if args.mfma_gemm_launches > 0:
        out["gemm_mfma_bound"] = mfma_bound_gemm(torch, B, wl, ExpandedLayer, args.mfma_gemm_launches)
    if args.graph_steps > 0:
        # the same step replayed from HIP graphs (one per rotating copy of X): what the dispatch
        # gaps between the step's seven launches cost
        graphs = []
        for x in Xd:
            g_ = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_):
                L.prepare_weights(Wd)
                B.ocs_split_act(x, M, L.C, L.g, K, L.chan_src, None, L.s, L.bits_x, None, 1.0, L.Xq, ldq,
                                L.scale_x, L.ws_x)
                L.qgemm(M)
            graphs.append(g_)
        for i in range(10):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for i in range(args.graph_steps):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - tg) / args.graph_steps * 1e6
        out["graph_replay"] = {"us_per_step": us, "tops_whole_step": ops / us / 1e6, "steps": args.graph_steps}
    if args.conv_steps > 0:
        out["conv_unlowered"] = conv_unlowered(torch, B, wl, layer, args.conv_steps)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layer, W, X)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
