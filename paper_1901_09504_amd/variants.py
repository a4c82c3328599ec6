"""Times of the calibration-time and variant entry points on one config's first layer.

    python -m paper_1901_09504_amd.variants --config 2 [--reps 30] [--json]

Weight preparation with plain halves (Eq. 3) and with quantization-aware members (Sec. 3.3), the
MSE clip-threshold search (Sec. 4.1) on the weights and on a batch of activations, the forward
pass with weight OCS and a per-batch activation grid, and the forward pass with the channels
chosen on the batch itself (Eq. 4, Sec. 5.3), with plain halves and with quantization-aware
members.  Each figure is the mean over `reps` calls between two events on the stream, after a
few untimed calls; the activations rotate through enough device copies to keep the memory-side
cache from serving them.  Inputs are the seeded synthetic tensors of the config.  Arithmetic
runs in libocs.so only; there is no fallback.  (Under rocprofv3 --kernel-trace the same run
gives every kernel's own time.)"""
import argparse
import json
import sys


def run(config, reps=30):
    import torch

    from . import binding as B
    from . import workloads as wl
    from .layer import ExpandedLayer

    if not torch.cuda.is_available():
        raise RuntimeError("variants: no GPU visible")
    B.lib()
    layer = wl.config(config)[0]
    W = torch.from_numpy(wl.weights(layer)).cuda()
    X0 = torch.from_numpy(wl.activations(layer)).cuda()
    copies = max(2, int(700e6 // (4.0 * layer.M * layer.K)) + 1)
    Xs = [X0] + [X0.clone() for _ in range(copies - 1)]
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, max_rows=layer.M)

    def timed(fn):
        for i in range(4):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    out = torch.zeros(2, device="cuda")
    hist = torch.zeros(2048, dtype=torch.int64, device="cuda")
    mse = torch.zeros(512, dtype=torch.float64, device="cuda")
    res = {"config": config, "layer": layer.name, "M": layer.M, "K": layer.K, "N": layer.N, "splits": L.s,
           "x_copies": copies, "reps": reps, "us": {}}
    us = res["us"]
    us["weights_plain_halves"] = timed(lambda i: L.prepare_weights(W))
    us["weights_qa_members"] = timed(lambda i: L.prepare_weights(W, qa=True))
    us["mse_clip_on_weights"] = timed(lambda i: B.ocs_mse_clip_threshold(
        W, layer.N, layer.K, W.stride(0), layer.bits_w, 2048, 512, out, hist, mse, L.ws_w))
    us["mse_clip_on_activations"] = timed(lambda i: B.ocs_mse_clip_threshold(
        Xs[i % copies], layer.M, layer.K, layer.K, layer.bits_x, 2048, 512, out, hist, mse, L.ws_x))
    L.prepare_weights(W)
    us["forward_weight_ocs_per_batch_grid"] = timed(lambda i: L.forward(Xs[i % copies]))
    us["forward_activation_ocs_plain_halves"] = timed(lambda i: L.forward_act_ocs(W, Xs[i % copies]))
    us["forward_activation_ocs_qa_members"] = timed(lambda i: L.forward_act_ocs(W, Xs[i % copies], qa=True))
    return res


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4])
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--json", action="store_true", help="one JSON object instead of the table")
    args = ap.parse_args()
    res = run(args.config, args.reps)
    if args.json:
        print(json.dumps(res))
        return
    print(f"config {res['config']} layer {res['layer']}: M={res['M']} K={res['K']} N={res['N']} "
          f"splits={res['splits']} ({res['x_copies']} rotating copies of X, mean of {res['reps']} calls)")
    for k, v in res["us"].items():
        print(f"  {k:40s} {v:9.1f} us")


if __name__ == "__main__":
    sys.exit(main())
