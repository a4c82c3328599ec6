#!/usr/bin/env python3
"""Benchmark of the OCS-expanded quantized layer on one MI355X.

The workload is the ResNet-50-shaped sweep: all 53 convolution layers as im2col GEMMs at batch
256, OCS at r = 0.05, 4-bit weights, 8-bit activations (2.22 tera-ops of expanded GEMM work per
pass).  A step is one pass of the hot path over that batch, layer after layer:

    ocs_split_weights   channel maxima of W, greedy selection, halve + clip + quantize   (W1-W3)
    ocs_split_act       duplicate the chosen channels, quantize on the static grid, pack  (X2)
    ocs_qgemm           int8 MFMA GEMM over the expanded K, dequantizing epilogue         (G1, G2)

The activation grid is static (Sec. 5 of the paper fixes it from profiling), so the pass that
takes max|X| (X1) is not in the step; `dynamic_grid` reports the step with it.  The weight path
depends on nothing the activation path produces and is queued on a second stream (`single_stream`
reports the step with everything in order on one stream).  Every layer owns
its activation tensor (22.3 GB in all, resident in HBM before the timed region), so between two
reads of a tensor 22 GB stream through the chip and nothing is served by the 256 MB memory-side
cache.  `value` is whole-pass throughput from the wall clock around the timed steps.  Kernel
durations come from a second, untimed run of the same steps in which every split+quantize and
GEMM launch stamps its own begin and end (HIP events on the launch stream).  Prints ONE JSON line.
"""
import argparse
import hashlib
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
RIDGE = INT8_PEAK_TOPS * 1e3 / HBM_PEAK_GBS   # op per byte
METRIC = "expanded int8 GEMM TOPS (% MFMA peak); split+quantize GB/s (% HBM)"
STATIC_T = 5.0               # the static activation grid's range (inputs are |N(0,1)|)

# HBM bytes per step moved by the split+quantize launches of this workload, from two rocprofv3
# --pmc runs of this command (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter
# reads for the plain copy kernel of known size that runs after the timed region
# (profiles/bench_config5_headline.md).  Valid only for the kernel source it was measured on:
# reported as null once that file changes.
X2_TRAFFIC = {"quantize_hip_sha256": "af4bb4e0e029d50a5d0fd005ad943fb80f02f0f7054c896d3ab774679a02eb2c",
              "bytes_per_step": 28940640069}


# The same for the launches of the one-launch pass (`--extras fused`), keyed on the GEMM source.
FUSED_TRAFFIC = {"qgemm_hip_sha256": "e877844785df958f9fab9f298e8557ced25473f8f65d32942d078a62d6984872",
                 "bytes_per_step": 22973502667}


def fused_traffic():
    src = os.path.join(ROOT, "paper_1901_09504_amd", "csrc", "qgemm.hip")
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    return FUSED_TRAFFIC["bytes_per_step"] if digest == FUSED_TRAFFIC["qgemm_hip_sha256"] else None


def x2_traffic():
    src = os.path.join(ROOT, "paper_1901_09504_amd", "csrc", "quantize.hip")
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    return X2_TRAFFIC["bytes_per_step"] if digest == X2_TRAFFIC["quantize_hip_sha256"] else None


class Net:
    """The 53 layers with their device buffers: weights, activations, one ExpandedLayer each."""

    def __init__(self, torch, wl, ExpandedLayer, layers, clip):
        self.layers = layers
        self.torch = torch
        self.wev = [torch.cuda.Event() for _ in layers]
        self.L, self.W, self.X = [], [], []
        gen = torch.Generator(device="cuda")
        for l in layers:
            self.W.append(torch.from_numpy(wl.weights(l)).cuda())
            # post-ReLU-like half-normal values drawn on the device (the passes' times do not
            # depend on the values; the parity tests use the host generators)
            gen.manual_seed(l.seed)
            x = torch.empty((l.M, l.K), dtype=torch.float32, device="cuda")
            x.normal_(generator=gen).abs_()
            self.X.append(x)
            self.L.append(ExpandedLayer(l.N, l.C, l.g, l.r, l.bits_w, l.bits_x, clip_ratio_w=clip,
                                        max_rows=l.M))
        self.thr = torch.tensor([STATIC_T], dtype=torch.float32, device="cuda")

    def step(self, B=None, ev=None, dynamic=False, weights=True, side=None, fused=None):
        """One pass.  ev: per-layer event lists [x2 a, x2 b, gemm a, gemm b, absmax a, absmax b]
        that the launches stamp themselves (B = the binding).  side: a second stream for the weight
        path, which depends on nothing the activation path produces: every layer's weight
        preparation is queued there, and the activation path waits, layer by layer, for the event
        behind it."""
        thr = None if dynamic else self.thr
        torch = self.torch
        if side is not None and weights:
            main = torch.cuda.current_stream()
            side.wait_stream(main)             # the previous pass no longer reads the weight codes
            with torch.cuda.stream(side):
                for i, L in enumerate(self.L):
                    L.prepare_weights(self.W[i])
                    self.wev[i].record(side)
        for i, (l, L) in enumerate(zip(self.layers, self.L)):
            if weights and side is None:
                L.prepare_weights(self.W[i])
            elif weights:
                torch.cuda.current_stream().wait_event(self.wev[i])
            if fused is not None and not dynamic and fused[i]:
                if ev is not None:
                    B.ocs_time_next(B.TIME_GEMM, ev[i][2], ev[i][3])
                L.forward_fused(self.X[i], thr)
                continue
            if ev is not None:
                if dynamic:
                    B.ocs_time_next(B.TIME_ABSMAX, ev[i][4], ev[i][5])
                B.ocs_time_next(B.TIME_SPLIT_QUANTIZE, ev[i][0], ev[i][1])
            L.split_act(self.X[i], thr)
            if ev is not None:
                B.ocs_time_next(B.TIME_GEMM, ev[i][2], ev[i][3])
            L.qgemm(l.M)


def stamped_steps(torch, B, net, n, dynamic=False, side=None, fused=None):
    """n passes whose split+quantize, GEMM (and max|X|) launches carry their own events.
    Returns arrays [n, layers] of kernel microseconds."""
    nl = len(net.layers)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(nl)]
    for row in ev:
        for e in row:
            e.record()
    torch.cuda.synchronize()
    x2 = np.zeros((n, nl))
    gm = np.zeros((n, nl))
    x1 = np.zeros((n, nl))
    for s in range(n):
        net.step(B, ev, dynamic=dynamic, side=side, fused=fused)
        torch.cuda.synchronize()
        for i in range(nl):
            if fused is None or not fused[i]:     # (a fused layer has no split+quantize launch)
                x2[s, i] = ev[i][0].elapsed_time(ev[i][1]) * 1e3
            gm[s, i] = ev[i][2].elapsed_time(ev[i][3]) * 1e3
            if dynamic:
                x1[s, i] = ev[i][4].elapsed_time(ev[i][5]) * 1e3
    return x2, gm, x1


def per_layer_report(net, x2, gm):
    rows = []
    for i, (l, L) in enumerate(zip(net.layers, net.L)):
        x2_bytes = 4.0 * l.M * l.K + 1.0 * l.M * L.Ke
        ops = 2.0 * l.M * l.N * L.Ke
        g_bytes = 1.0 * l.M * L.Ke + 1.0 * l.N * L.Ke + 4.0 * l.M * l.N
        ai = ops / g_bytes
        x2_us, g_us = float(np.median(x2[:, i])), float(np.median(gm[:, i]))
        roof = min(INT8_PEAK_TOPS, ai * HBM_PEAK_GBS / 1e3)
        rows.append({"layer": l.name, "M": l.M, "K": l.K, "N": l.N, "s": L.s, "Kexp": L.Ke, "ld": L.ldq,
                     "split_quant_us": round(x2_us, 2), "split_quant_GBps": round(x2_bytes / x2_us / 1e3, 1),
                     "split_quant_frac_hbm": round(x2_bytes / x2_us / 1e3 / HBM_PEAK_GBS, 4),
                     "gemm_us": round(g_us, 2), "gemm_tops": round(ops / g_us / 1e6, 1),
                     "gemm_GBps": round(g_bytes / g_us / 1e3, 1), "gemm_ai": round(ai, 1),
                     "gemm_regime": "mfma" if ai >= RIDGE else "hbm",
                     "gemm_frac_of_min_roof": round(ops / g_us / 1e6 / roof, 4)})
    return rows


def config2_step(torch, B, wl, ExpandedLayer, steps=100, stamped=24, copies=6):
    """The single 3x3 convolution of the second workload (batch 64, M=12544 K=2304 N=256,
    r=0.02, 8/8 bit) with a per-batch activation grid: weight path, max|X|, split+quantize, GEMM.
    X rotates through `copies` tensors (694 MB); inside a step the split+quantize pass still
    follows the max|X| pass over the same X, so its in-step time is cache-assisted and labelled so."""
    (layer,) = wl.config(2)
    M, N, K = layer.M, layer.N, layer.K
    Wd = torch.from_numpy(wl.weights(layer)).cuda()
    X = torch.from_numpy(wl.activations(layer)).cuda()
    Xd = [X] + [X.clone() for _ in range(copies - 1)]
    L = ExpandedLayer(N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, max_rows=M)

    def step(i, ev=None):
        L.prepare_weights(Wd)
        if ev:
            B.ocs_time_next(B.TIME_ABSMAX, ev[4], ev[5])
            B.ocs_time_next(B.TIME_SPLIT_QUANTIZE, ev[0], ev[1])
        L.split_act(Xd[i % copies], None)
        if ev:
            B.ocs_time_next(B.TIME_GEMM, ev[2], ev[3])
        L.qgemm(M)

    for i in range(10):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    for e in ev:
        e.record()
    k = np.zeros((stamped, 3))
    for i in range(stamped):
        step(i, ev)
        torch.cuda.synchronize()
        k[i] = [ev[0].elapsed_time(ev[1]) * 1e3, ev[2].elapsed_time(ev[3]) * 1e3, ev[4].elapsed_time(ev[5]) * 1e3]
    # the split+quantize pass alone on a static grid: nothing has touched the copy it reads since
    # the other copies were streamed (cache-cold)
    cold = []
    for i in range(copies + stamped):
        B.ocs_time_next(B.TIME_SPLIT_QUANTIZE, ev[0], ev[1])
        L.split_act(Xd[i % copies], L.scale_x)
        torch.cuda.synchronize()
        if i >= copies:
            cold.append(ev[0].elapsed_time(ev[1]) * 1e3)
    ops = 2.0 * M * N * L.Ke
    x2_bytes = 4.0 * M * K + 1.0 * M * L.Ke
    x2_us, g_us, x1_us, cold_us = (float(np.median(k[:, 0])), float(np.median(k[:, 1])),
                                   float(np.median(k[:, 2])), float(np.median(cold)))

    # the calibration-time and variant entry points on the same layer (wall clock per call)
    def per_call(fn, n=50):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n * 1e6

    hist = torch.empty(2048, dtype=torch.int64, device="cuda")
    mse = torch.empty(512, dtype=torch.float64, device="cuda")
    thr2 = torch.empty(2, dtype=torch.float32, device="cuda")
    variants = {
        "weights_plain_halves_us": per_call(lambda i: L.prepare_weights(Wd)),
        "weights_qa_members_us (Sec. 3.3)": per_call(lambda i: L.prepare_weights(Wd, qa=True)),
        "mse_clip_search_on_X_us (Sec. 4.1, 2048 bins, 512 candidates)":
            per_call(lambda i: B.ocs_mse_clip_threshold(Xd[i % copies], M, K, K, 8, 2048, 512, thr2, hist, mse, L.ws_x)),
        "mse_clip_search_on_W_us": per_call(lambda i: B.ocs_mse_clip_threshold(Wd, N, K, K, 8, 2048, 512, thr2, hist,
                                                                              mse, L.ws_w)),
        "forward_per_batch_activation_ocs_us (Sec. 5.3, Eq. 4)": per_call(lambda i: L.forward_act_ocs(Wd, Xd[i % copies])),
        "forward_per_batch_activation_ocs_qa_us": per_call(lambda i: L.forward_act_ocs(Wd, Xd[i % copies], qa=True)),
    }
    L.prepare_weights(Wd)
    return {"workload": f"configs[1]: M={M} K={K} N={N} r={layer.r} (K'={L.Ke}, padded {L.ldq}), 8/8 bit, "
                        "weight path + per-batch grid + split+quantize + GEMM per step",
            "us_per_step": us, "tops_whole_step": ops / us / 1e6, "steps": steps,
            "absmax_kernel_us": x1_us, "gemm_kernel_us": g_us, "gemm_tops": ops / g_us / 1e6,
            "gemm_pct_mfma_peak": 100.0 * ops / g_us / 1e6 / INT8_PEAK_TOPS,
            "variants": variants,
            "split_quant_cache_cold": {"kernel_us": cold_us, "GBps": x2_bytes / cold_us / 1e3,
                                       "frac_hbm": x2_bytes / cold_us / 1e3 / HBM_PEAK_GBS,
                                       "launches_timed": len(cold)},
            "split_quant_in_step_cache_assisted": {"kernel_us": x2_us, "GBps": x2_bytes / x2_us / 1e3,
                                                   "frac_hbm": x2_bytes / x2_us / 1e3 / HBM_PEAK_GBS,
                                                   "launches_timed": stamped,
                                                   "note": "follows the max|X| pass over the same 115.6 MB X, "
                                                           "part of which the memory-side cache still holds"}}


class ChainedNet:
    """The same 53 layers with the convolutions given un-lowered and, inside every bottleneck, the
    activations handed from layer to layer as codes (1x1 -> ReLU -> 3x3 -> ReLU -> 1x1; the block's
    last layer and its projection write fp32, since the residual sum follows them).  Weight OCS on
    every layer, static grids.  Per block: one split+quantize pass over the block's fp32 input
    [B, H, W, C] (not over its im2col image), then the three convolutions."""

    def __init__(self, torch, wl, layers, clip, batch=256):
        from paper_1901_09504_amd.layer import ConvChain, ExpandedConv
        by = {l.name: l for l in layers}
        gen = torch.Generator(device="cuda")
        self.torch, self.batch = torch, batch

        def dev_w(l):
            return torch.from_numpy(wl.weights(l)).cuda()

        def dev_x(l, size, seed):
            gen.manual_seed(seed)
            x = torch.empty((batch, size, size, l.C), dtype=torch.float32, device="cuda")
            return x.normal_(generator=gen).abs_()

        stem = by["stem_7x7"]
        self.stem = ExpandedConv(stem.N, stem.C, 7, 7, 2, 3, stem.r, stem.bits_w, stem.bits_x, clip_ratio_w=clip)
        self.stem_w, self.stem_x = dev_w(stem), dev_x(stem, 224, stem.seed)
        self.blocks = []
        for stage, nblocks in zip((1, 2, 3, 4), (3, 4, 6, 3)):
            for b in range(nblocks):
                la, lb, lc = (by[f"s{stage}b{b}_{t}"] for t in ("1x1a", "3x3", "1x1b"))
                size = int(round((la.M / batch) ** 0.5))
                stride = 2 if lb.M * 4 == la.M else 1
                chain = ConvChain(la.C, [(la.N, 1, 1, 0), (lb.N, 3, stride, 1), (lc.N, 1, 1, 0)], la.r,
                                  la.bits_w, la.bits_x, clip_ratio_w=clip)
                proj = pw = None
                if b == 0:
                    lp = by[f"s{stage}b{b}_proj"]
                    proj = ExpandedConv(lp.N, lp.C, 1, 1, stride, 0, lp.r, lp.bits_w, lp.bits_x, clip_ratio_w=clip)
                    pw = dev_w(lp)
                self.blocks.append((chain, [dev_w(la), dev_w(lb), dev_w(lc)], dev_x(la, size, la.seed), proj, pw))
        self.thr_in = torch.tensor([STATIC_T], dtype=torch.float32, device="cuda")
        self.thr_mid = torch.tensor([4.0], dtype=torch.float32, device="cuda")

    def step(self):
        self.stem.prepare_weights(self.stem_w)
        self.stem.forward(self.stem_x, self.thr_in)
        thr = [self.thr_in, self.thr_mid, self.thr_mid]
        for chain, ws, x, proj, pw in self.blocks:
            chain.prepare_weights(ws)
            chain.forward(x, thr)
            if proj is not None:
                proj.prepare_weights(pw)
                proj.forward(x, self.thr_in)


def chained_pass(torch, wl, layers, clip, ops, steps=10):
    net = ChainedNet(torch, wl, layers, clip)
    for _ in range(2):
        net.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    return {"what": "the same 53 layers, convolutions un-lowered (the lowering happens in the GEMM kernel's operand "
                    "loader), codes handed from layer to layer inside each bottleneck (re-quantizing epilogue), "
                    "fp32 only at block outputs; weight path included; same 2.22 tera-ops",
            "ms_per_step": ms, "tops_whole_step": ops / ms / 1e9, "steps": steps}


def split_k_compare(torch, B, wl, ExpandedLayer, launches=24, copies=5):
    """The one layer shape above the MFMA ridge (512 -> 512 3x3 at batch 256: 196 tiles of 256 x 128 for
    256 compute units) through ocs_qgemm and through ocs_qgemm_split_k (98 tiles of 256 x 256, K shared
    by 2 or 3 workgroups each); the activation codes rotate through several copies."""
    layer = next(l for l in wl.config(5) if l.name == "s4b0_3x3")
    M, N = layer.M, layer.N
    L = ExpandedLayer(N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, max_rows=M)
    L.prepare_weights(torch.from_numpy(wl.weights(layer)).cuda())
    L.split_act(torch.from_numpy(wl.activations(layer)).cuda())
    torch.cuda.synchronize()
    Xq = [L.Xq.clone() for _ in range(copies)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in ev:
        e.record()
    ops = 2.0 * M * N * L.Ke
    out = {"workload": f"M={M} N={N} K'={L.Ke} (padded {L.ldq}), {copies} rotating copies of the activation codes"}
    Y_ref = None
    for parts in (1, 2, 3):
        ws = torch.empty(max(256, B.ocs_qgemm_split_k_workspace_bytes(M, N, L.Ke, parts)), dtype=torch.uint8,
                         device="cuda")
        us = []
        for i in range(launches + 4):
            B.ocs_time_next(B.TIME_GEMM, ev[0], ev[1])
            if parts == 1:
                B.ocs_qgemm(Xq[i % copies], L.ldq, L.Wq, L.ldq, M, N, L.Ke, L.bits_x, L.bits_w, L.scale_x,
                            L.scale_w, None, 0, L.Y, N, None)
            else:
                B.ocs_qgemm_split_k(Xq[i % copies], L.ldq, L.Wq, L.ldq, M, N, L.Ke, L.bits_x, L.bits_w, L.scale_x,
                                    L.scale_w, None, 0, L.Y, N, parts, ws)
            torch.cuda.synchronize()
            if i >= 4:
                us.append(ev[0].elapsed_time(ev[1]) * 1e3)
        if Y_ref is None:
            Y_ref = L.Y.clone()
        med = float(np.median(us))
        out["un-split" if parts == 1 else f"{parts} parts"] = {
            "median_us": med, "tops": ops / med / 1e6, "pct_mfma_peak": 100.0 * ops / med / 1e6 / INT8_PEAK_TOPS,
            "same_output_bits": bool(torch.equal(Y_ref, L.Y)), "launches_timed": len(us)}
    return out


def calib_copy(torch, B, net, reps=4):
    """The library's plain 16-byte copy kernel on the largest activation tensor (1.89 GB each way)."""
    src = max(net.X, key=lambda x: x.numel())
    dst = torch.empty_like(src)
    n = src.numel() * 4 // 16 * 16
    us = _timed(torch, lambda: B.ocs_calib_copy(src, dst, n, 1024), reps)
    us1 = _timed(torch, lambda: B.ocs_calib_copy(src, dst, n, 0), reps)
    return {"kernel": "calib_copy_kernel (16-byte loads and stores, grid-stride loop of 1024 workgroups: the launches the "
                      "HBM byte counters are scaled against)", "bytes_each_way": int(n),
            "median_us": us, "read_plus_write_GBps": 2.0 * n / us / 1e3,
            "frac_hbm": 2.0 * n / us / 1e3 / HBM_PEAK_GBS, "launches": reps + 1,
            "one_shot_form": {"kernel": "calib_copy_shot_kernel (one 16-byte group per lane, a workgroup per 4 KB, no loop)",
                              "median_us": us1, "read_plus_write_GBps": 2.0 * n / us1 / 1e3,
                              "frac_hbm": 2.0 * n / us1 / 1e3 / HBM_PEAK_GBS, "launches": reps + 1}}


def _timed(torch, fn, reps):
    """Median microseconds of fn() over reps launches (event brackets; the launches here run for
    hundreds of microseconds to milliseconds, so the bracket's own few microseconds do not matter)."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    us = []
    for r in range(reps + 1):
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        if r >= 1:
            us.append(a.elapsed_time(b) * 1e3)
    return float(np.median(us))


def ceilings(torch, B, reps=5):
    """What this chip gives plain kernels of known work (the library's measurement helpers):
    copy, read-only sweep and fill of 2 GiB; the same read over 2 MiB that stays in every L2; a
    bare loop of the GEMM's matrix instruction on zero, constant and random operand bytes."""
    n = 2 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    a.random_(0, 256)
    sink = torch.zeros(65536 * 4, dtype=torch.int32, device="cuda")
    out = {"bytes": n}
    def best_of(fn, grids):
        best = None
        for wgs in grids:
            us = _timed(torch, lambda: fn(wgs), reps)
            if best is None or us < best[0]:
                best = (us, wgs)
        return best

    # each kernel in its one-shot form (one 16-byte group per lane, a workgroup per 4 KB, no loop:
    # "workgroups": 0) and as a grid-stride loop with the best of several grid sizes
    grids = (256, 512, 1024, 2048, 4096)
    def both(fn, nbytes, key, rate_key):
        us0 = _timed(torch, lambda: fn(0), reps)
        usl, wgs = best_of(fn, grids)
        out[key] = {"us": us0, "workgroups": 0, rate_key: nbytes / us0 / 1e3, "frac_hbm": nbytes / us0 / 1e3 / HBM_PEAK_GBS,
                    "grid_stride_loop": {"us": usl, "workgroups": wgs, rate_key: nbytes / usl / 1e3,
                                         "frac_hbm": nbytes / usl / 1e3 / HBM_PEAK_GBS}}
    both(lambda w: B.ocs_calib_copy(a, b, n, w), 2.0 * n, "copy", "read_plus_write_GBps")
    both(lambda w: B.ocs_calib_pack(a, b, n, w), 1.25 * n, "pack_16B_in_4B_out", "read_plus_write_GBps")
    both(lambda w: B.ocs_calib_read(a, n, 1, w, sink), 1.0 * n, "read", "GBps")
    for key, nt in (("fill", 0), ("fill_nontemporal", 1)):
        both(lambda w: B.ocs_calib_fill(b, n, 7, nt, w), 1.0 * n, key, "GBps")
    small, passes = 2 << 20, 4096
    l2 = {}
    for wgs in (250, 500, 1000, 2000):
        us = _timed(torch, lambda: B.ocs_calib_read(a, small, passes, wgs, sink), reps)
        l2[str(wgs)] = small * passes / us / 1e3
    out["read_l2_resident"] = {"buffer_bytes": small, "passes": passes, "GBps_by_workgroups": l2,
                               "note": "the stream wraps around 2 MiB, which each of the 8 L2s keeps (a lane's own "
                                       "addresses are 4 KB and more apart, beyond what the 32 KB L1 holds); "
                                       "workgroups of 256 lanes, two 16-byte loads in flight per lane"}
    iters, wgs = 20000, 1024
    ops = wgs * 4.0 * iters * 4 * 65536
    mf = {}
    for name, fill in (("zeros", lambda t: t.zero_()), ("constant_0x01", lambda t: t.fill_(1)),
                       ("random_int8", lambda t: t.random_(0, 256))):
        opnd = torch.empty(16384, dtype=torch.uint8, device="cuda")
        fill(opnd)
        us = _timed(torch, lambda: B.ocs_calib_mfma(opnd, iters, wgs, sink), reps)
        mf[name] = {"us": us, "tops": ops / us / 1e6, "frac_int8_peak": ops / us / 1e6 / INT8_PEAK_TOPS}
    out["mfma_i32_32x32x32_i8"] = {"workgroups": wgs, "waves_per_cu": 16, "iters": iters, "by_operand_data": mf}
    return out


def cpu_baseline(wl, layers, clip, row_fraction=4):
    """The CPU oracle, as it stands, on this machine's host cores: the whole step (weight path in
    full, activation pass and GEMM on the first 1/row_fraction of every layer's rows)."""
    from oracle import ref

    t_total, ops = 0.0, 0.0
    for l in layers:
        rows = max(1, l.M // row_fraction)
        W = wl.weights(l)
        X = wl.activations(l, 0, rows)
        s = ref.num_splits(l.C, l.r)
        Ke = (l.C + s) * l.g
        ldq = (Ke + 63) // 64 * 64
        t0 = time.perf_counter()
        sp = ref.split_weights(W, l.C, l.g, s)
        Wq, sw = ref.quantize(sp["T_out"], l.bits_w, clip_ratio=clip, ldq=ldq)
        Xq, sx, _ = ref.split_act(X, l.C, l.g, sp["chan_src"], None, s, l.bits_x, threshold=STATIC_T, ldq=ldq)
        ref.qgemm(Xq, Wq, Ke, sx[1], sw[1], want_acc=False)
        t_total += time.perf_counter() - t0
        ops += 2.0 * rows * l.N * Ke
    return {"value": ops / t_total / 1e12, "unit": "TOPS", "cores": ref.get_threads(), "kind": "oracle",
            "sample": f"whole step over the 53 layers with the first 1/{row_fraction} of every layer's rows "
                      f"(batch {256 // row_fraction} of 256; the weight path in full), one pass, "
                      f"{t_total:.1f} s of CPU work, {ops / 1e12:.3f} tera-ops",
            "seconds": t_total}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--clip", type=float, default=0.9, help="weight clip ratio used in the timed step")
    ap.add_argument("--stamped-steps", type=int, default=20,
                    help="untimed passes whose launches carry their own events (at least 20 samples per layer)")
    ap.add_argument("--single-stream", action="store_true",
                    help="queue the weight path in order on the activation path's stream instead of on a second one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", default="", help="key=value[,key=value]: launch-shape overrides (ocs_tune) for experiments")
    ap.add_argument("--fused-layers", default="", help="with the `fused` extra: only these layers take the one-launch path")
    ap.add_argument("--extras", default="steps,fused,chained,ceilings,config2,splitk",
                    help="secondary measurements to run: steps (per-batch grid, single stream, off-line weights, "
                         "weight path by clip), chained, ceilings, config2, splitk")
    ap.add_argument("--only", choices=["chained", "ceilings", "config2", "splitk"], default=None,
                    help="run one secondary measurement alone and print it (no headline)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the secondary measurements (dynamic grid, weight path, ceilings, config 2)")
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

    layers = wl.config(5)
    if args.only:
        # one secondary measurement by itself (for profiler runs that should see only its kernels)
        ops5 = sum(2.0 * l.M * l.N * (l.C + B.ocs_num_splits(l.C, l.r)) * l.g for l in layers)
        res = {"chained": lambda: chained_pass(torch, wl, layers, args.clip, ops5),
               "ceilings": lambda: ceilings(torch, B),
               "config2": lambda: config2_step(torch, B, wl, ExpandedLayer),
               "splitk": lambda: split_k_compare(torch, B, wl, ExpandedLayer)}[args.only]()
        print(json.dumps({"only": args.only, args.only: res}))
        return
    net = Net(torch, wl, ExpandedLayer, layers, args.clip)
    torch.cuda.synchronize()
    for kv in filter(None, args.tune.split(",")):
        B.ocs_tune(kv.split("=")[0], int(kv.split("=")[1]))

    # the weight path depends on nothing the activation path produces: it is queued on a second
    # stream (default priority), and each layer's activation pass waits for the event behind its
    # weights; --single-stream keeps everything in order on one stream
    side = None if args.single_stream else torch.cuda.Stream()

    def timed(n, **kw):
        for _ in range(max(1, args.warmup) if n == args.steps else 2):
            net.step(**kw)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            net.step(**kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3

    ms_per_step = timed(args.steps, side=side)

    n_stamp = max(20, args.stamped_steps)
    x2, gm, _ = stamped_steps(torch, B, net, n_stamp, side=side)
    # a plain copy of known size right behind the measured passes: the reference that the HBM byte
    # counters of a profiled run of this same command are scaled by, and this chip's own copy rate
    copy_ref = calib_copy(torch, B, net)
    rows = per_layer_report(net, x2, gm)
    ops = sum(2.0 * l.M * l.N * L.Ke for l, L in zip(layers, net.L))
    x2_bytes = sum(4.0 * l.M * l.K + 1.0 * l.M * L.Ke for l, L in zip(layers, net.L))
    x2_us_step = float(np.mean(x2.sum(axis=1)))          # all 53 launches of one pass, mean over passes
    gemm_us_step = float(np.mean(gm.sum(axis=1)))
    x2_gbs = x2_bytes / x2_us_step / 1e3
    gemm_tops = ops / gemm_us_step / 1e6
    mfma = [r for r in rows if r["gemm_regime"] == "mfma"]

    out = {
        "metric": METRIC,
        "value": ops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TOPS (2*M*N*K' of the 53 expanded layers per second of whole-pass wall time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "dtype_detail": "int8 codes x int8 codes -> int32 accumulators; fp32 in, fp32 out",
        "data": "synthetic",
        "config": {"workload": "configs[4]: ResNet-50-shaped sweep, all 53 conv layers as im2col GEMMs at batch "
                               f"256, r=0.05, 4-bit weights (clip {args.clip} x max|W'|), 8-bit activations on a "
                               "static grid; per layer: weight path, split+quantize, expanded GEMM; weight path "
                               + ("in order on the same stream" if side is None else "queued on a second stream"),
                   "tera_ops_per_step": ops / 1e12, "layers": len(layers),
                   "activation_bytes_resident": int(sum(x.numel() * 4 for x in net.X)),
                   "stamped_steps": n_stamp},
        "gemm_tops": gemm_tops, "gemm_pct_mfma_peak": 100.0 * gemm_tops / INT8_PEAK_TOPS,
        "split_quant_gbps": x2_gbs, "split_quant_pct_hbm": 100.0 * x2_gbs / HBM_PEAK_GBS,
        "roofline": {"kernel": "expand_quantize_shot_kernel (expand_quantize_tile_kernel on the stem) (ocs_split_act, X2): the 53 "
                               "launches of one pass", "bound": "hbm",
                     "achieved": x2_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": x2_gbs / HBM_PEAK_GBS,
                     "traffic": None if x2_traffic() is None else x2_traffic() / len(layers),
                     "traffic_bytes_per_step": x2_traffic(),
                     "algorithmic_bytes_per_step": x2_bytes, "kernel_us_per_step": x2_us_step,
                     "avg_launch_us": x2_us_step / len(layers), "launches_per_step": len(layers),
                     "launches_timed": int(x2.size), "cache": "cold: every launch reads a tensor that 22 GB of "
                                                              "other traffic have passed since its last use",
                     "timing": "HIP events stamped by the launch itself (hipExtLaunchKernel) on its stream: the "
                               "dispatch's own begin and end; mean over the stamped passes of the per-pass sum"},
        "step_breakdown_ms": {"split_quant_kernels": x2_us_step / 1e3, "gemm_kernels": gemm_us_step / 1e3,
                              "rest (weight path not hidden behind them, dispatch gaps)":
                                  ms_per_step - (x2_us_step + gemm_us_step) / 1e3},
        "gemm_mfma_bound": [{k: r[k] for k in ("layer", "M", "N", "Kexp", "gemm_us", "gemm_tops", "gemm_ai")} |
                            {"pct_mfma_peak": round(100.0 * r["gemm_tops"] / INT8_PEAK_TOPS, 2)} for r in mfma],
        "calib_copy": copy_ref,
        "layers": rows,
    }
    extras = set() if args.no_extras else set(args.extras.split(","))
    if "fused" in extras:
        # split+quantize and GEMM as one launch wherever that entry point serves the layer
        fmap = [L.fused_pays(x) for L, x in zip(net.L, net.X)]
        if args.fused_layers:
            names = set(args.fused_layers.split(","))
            fmap = [f and l.name in names for f, l in zip(fmap, layers)]
        f_ms = timed(10, side=side, fused=fmap)
        x2f, gmf, _ = stamped_steps(torch, B, net, 10, side=side, fused=fmap)
        frows = []
        for i, (l, L) in enumerate(zip(layers, net.L)):
            if fmap[i]:
                us = float(np.median(gmf[:, i]))
                byt = 4.0 * l.M * l.K + 1.0 * l.N * L.Ke + 4.0 * l.M * l.N
                frows.append({"layer": l.name, "M": l.M, "K": l.K, "N": l.N, "fused_us": round(us, 2),
                              "two_launch_us": round(rows[i]["split_quant_us"] + rows[i]["gemm_us"], 2),
                              "GBps": round(byt / us / 1e3, 1), "frac_hbm": round(byt / us / 1e3 / HBM_PEAK_GBS, 4)})
        f_bytes = sum(4.0 * l.M * l.K + 1.0 * l.N * L.Ke + 4.0 * l.M * l.N
                      for l, L, f in zip(layers, net.L, fmap) if f)
        f_us = float(np.mean(gmf[:, np.array(fmap)].sum(axis=1)))
        out["fused_split_gemm"] = {
            "what": "the same pass with ocs_split_act_qgemm (split+quantize and GEMM as one launch, no code tensor "
                    "in memory) on every layer where the library expects it to be ahead; the other layers as above",
            "ms_per_step": f_ms, "tops_whole_step": ops / f_ms / 1e9, "steps": 10, "layers_fused": int(sum(fmap)),
            "roofline": {"kernel": "split_act_qgemm_kernel: its launches of one pass", "bound": "hbm",
                         "achieved": f_bytes / f_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": f_bytes / f_us / 1e3 / HBM_PEAK_GBS,
                         "traffic": None if fused_traffic() is None else fused_traffic() / int(sum(fmap)),
                         "traffic_bytes_per_step": fused_traffic(),
                         "algorithmic_bytes_per_step": f_bytes, "bytes_per_unit": "4*M*K + N*K' + 4*M*N per layer",
                         "kernel_us_per_step": f_us, "avg_launch_us": f_us / int(sum(fmap)),
                         "launches_per_step": int(sum(fmap)), "launches_timed": int(gmf[:, np.array(fmap)].size)},
            "layers": frows}
    if "steps" in extras:
        # the pass with a per-batch activation grid: X1 (max|X|) in front of every split+quantize
        dyn_ms = timed(5, dynamic=True, side=side)
        _, _, x1 = stamped_steps(torch, B, net, 5, dynamic=True, side=side)
        x1_us_step = float(np.mean(x1.sum(axis=1)))
        x1_bytes = sum(4.0 * l.M * l.K for l in layers)
        out["dynamic_grid"] = {"ms_per_step": dyn_ms, "tops_whole_step": ops / dyn_ms / 1e9,
                               "absmax_kernels_ms_per_step": x1_us_step / 1e3,
                               "absmax_GBps": x1_bytes / x1_us_step / 1e3,
                               "absmax_frac_hbm": x1_bytes / x1_us_step / 1e3 / HBM_PEAK_GBS, "steps": 5}
        # the same pass with everything in order on one stream
        if side is not None:
            ss_ms = timed(10)
            out["single_stream"] = {"ms_per_step": ss_ms, "tops_whole_step": ops / ss_ms / 1e9, "steps": 10}
        # the pass without the weight path (weights prepared once, off-line, as in Sec. 3.5)
        nw_ms = timed(10, weights=False)
        out["weights_prepared_off_line"] = {"ms_per_step": nw_ms, "tops_whole_step": ops / nw_ms / 1e9, "steps": 10}
        # the weight path alone, per clip ratio (the ratio changes only the grid and the codes)
        wp = {}
        for clip in (1.0, 0.9, 0.8):
            for L in net.L:
                L.clip_ratio_w = clip
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                for i, L in enumerate(net.L):
                    L.prepare_weights(net.W[i])
            torch.cuda.synchronize()
            wp[str(clip)] = (time.perf_counter() - t0) / 5 * 1e3
        for L in net.L:
            L.clip_ratio_w = args.clip
        out["weight_path_ms_per_pass_by_clip"] = wp
    del net
    torch.cuda.empty_cache()
    if "chained" in extras:
        out["chained_unlowered"] = chained_pass(torch, wl, layers, args.clip, ops)
        torch.cuda.empty_cache()
    if "ceilings" in extras:
        out["ceilings"] = ceilings(torch, B)
    if "config2" in extras:
        out["config2_step"] = config2_step(torch, B, wl, ExpandedLayer)
    if "splitk" in extras:
        out["gemm_split_k"] = split_k_compare(torch, B, wl, ExpandedLayer)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, layers, args.clip)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
