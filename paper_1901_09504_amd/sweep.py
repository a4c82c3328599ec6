"""Per-layer and aggregate throughput of the expanded quantized layer over a whole config.

    python -m paper_1901_09504_amd.sweep --config 5 --batch 256 [--json]

For every distinct layer shape of the config: the weights are prepared once (weight OCS), then
the split+quantize pass on a static activation grid (the paper's deployment: Sec. 5 fixes the
activation grid from profiling) and the GEMM are timed, each by events that the launch itself
stamps with the kernel's begin and end.  The activations are synthetic (device-generated
half-normal values; these passes' times do not depend on the values) and rotate through enough
copies to keep the memory-side cache from serving them.  The aggregate weighs every shape by
the number of times it occurs in the network.  Arithmetic runs in libocs.so only; there is no
fallback."""
import argparse
import json
import sys

import numpy as np


def run(config, batch, reps=6, static_threshold=5.0):
    import torch

    from . import binding as B
    from . import workloads as wl
    from .layer import ExpandedLayer

    if not torch.cuda.is_available():
        raise RuntimeError("sweep: no GPU visible")
    B.lib()
    layers = wl.config(config, batch=batch) if config == 5 else wl.config(config)
    seen = {}
    for l in layers:
        key = (l.M, l.C, l.g, l.N, l.r, l.bits_w, l.bits_x)
        seen.setdefault(key, [l, 0])
        seen[key][1] += 1
    thr = torch.tensor([static_threshold], device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    rows = []
    for (M, C, g, N, _r, _bw, _bx), (l, count) in seen.items():
        K = C * g
        L = ExpandedLayer(N, C, g, l.r, l.bits_w, l.bits_x, max_rows=M)
        L.prepare_weights(torch.from_numpy(wl.weights(l)).cuda())
        copies = 1 if 4.0 * M * K > 600e6 else int(700e6 // (4.0 * M * K)) + 1
        Xs = [torch.empty((M, K), dtype=torch.float32, device="cuda").normal_().abs_() for _ in range(copies)]
        tx, tg = [], []
        for it in range(max(reps, copies + 2)):
            B.ocs_time_next(B.TIME_SPLIT_QUANTIZE, ev[0], ev[1])
            L.split_act(Xs[it % copies], thr)
            B.ocs_time_next(B.TIME_GEMM, ev[2], ev[3])
            L.qgemm(M)
            torch.cuda.synchronize()
            tx.append(ev[0].elapsed_time(ev[1]) * 1e3)
            tg.append(ev[2].elapsed_time(ev[3]) * 1e3)
        x_us, g_us = float(np.median(tx[1:])), float(np.median(tg[1:]))
        rows.append({"layer": l.name, "M": M, "K": K, "N": N, "r": l.r, "count": count, "Kexp": L.Ke, "ld": L.ldq,
                     "split_quant_us": x_us, "split_quant_GBps": (4.0 * M * K + M * L.Ke) / x_us / 1e3,
                     "gemm_us": g_us, "gemm_tops": 2.0 * M * N * L.Ke / g_us / 1e6,
                     "gemm_GBps": (M * L.Ke + N * L.Ke + 4.0 * M * N) / g_us / 1e3})
        del L, Xs
        torch.cuda.empty_cache()
    ops = sum(2.0 * r["M"] * r["N"] * r["Kexp"] * r["count"] for r in rows)
    us = sum((r["split_quant_us"] + r["gemm_us"]) * r["count"] for r in rows)
    return {"config": config, "batch": batch if config == 5 else None, "layers": rows,
            "aggregate": {"tera_ops": ops / 1e12, "ms": us / 1e3, "tops": ops / us / 1e6,
                          "split_quant_ms": sum(r["split_quant_us"] * r["count"] for r in rows) / 1e3,
                          "gemm_ms": sum(r["gemm_us"] * r["count"] for r in rows) / 1e3}}


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", type=int, default=5, choices=[2, 3, 4, 5])
    ap.add_argument("--batch", type=int, default=256, help="batch size of config 5's layers")
    ap.add_argument("--json", action="store_true", help="one JSON object instead of the table")
    args = ap.parse_args()
    out = run(args.config, args.batch)
    if args.json:
        print(json.dumps(out))
        return
    print(f"{'layer':30s} {'M':>8s} {'K':>5s} {'N':>5s} {'r':>5s} cnt | split+quantize us  GB/s %HBM | GEMM us   TOPS   GB/s")
    for r in out["layers"]:
        print(f"{r['layer']:30s} {r['M']:8d} {r['K']:5d} {r['N']:5d} {r['r']:5.2f} {r['count']:3d} | {r['split_quant_us']:9.1f} "
              f"{r['split_quant_GBps']:9.0f} {r['split_quant_GBps'] / 80:4.0f}% | {r['gemm_us']:7.1f} "
              f"{r['gemm_tops']:6.0f} {r['gemm_GBps']:6.0f}")
    a = out["aggregate"]
    print(f"aggregate: {a['tera_ops']:.2f} TOP in {a['ms']:.2f} ms (split+quantize {a['split_quant_ms']:.2f} ms, "
          f"GEMM {a['gemm_ms']:.2f} ms) = {a['tops']:.0f} TOPS")


if __name__ == "__main__":
    sys.exit(main())
