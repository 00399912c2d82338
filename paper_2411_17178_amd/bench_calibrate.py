"""Times the window calibration (paper Section 2: metric R_w, threshold R_0) on one GPU:
post-softmax attention maps of N reference samples -> one radius per (head, query scale, key
scale).  Run as

    python -m paper_2411_17178_amd.bench_calibrate [--samples 8] [--heads 30] [--r0 0.95] [--band]

Prints one JSON line.  The maps are seeded synthetic rows (a noisy bump around each query's
position, block-causal across scales, rows summing to one), resident in HBM; the algorithmic
bytes are the map's block-causal entries, read once (4 bytes each).
"""
import argparse
import json
import sys

VAR_SCALES = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--samples", type=int, default=8)
    ap.add_argument("--heads", type=int, default=30)
    ap.add_argument("--r0", type=float, default=0.95)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--band", action="store_true",
                    help="the band mask mode's parts (Section 2, step (2) read literally)")
    args = ap.parse_args()

    import torch

    import paper_2411_17178_amd as lv
    import workloads

    lv.load_library()
    if not torch.cuda.is_available():
        print("bench_calibrate: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    scales = VAR_SCALES
    L = sum(s * s for s in scales)
    # one seeded sample from the CPU recipe per head, the other samples: the same rows with
    # fresh multiplicative noise drawn on the device, renormalised
    base = workloads.make_attn_map(scales, 1, args.heads, 2024).to(dev)
    g = torch.Generator(device=dev).manual_seed(7)
    maps = torch.empty((args.samples, args.heads, L, L), dtype=torch.float32, device=dev)
    for n in range(args.samples):
        w = base[0] * torch.exp(0.3 * torch.randn(base[0].shape, generator=g, device=dev))
        maps[n] = w / w.sum(dim=-1, keepdim=True)
    calibrate = lv.litevar_window_calibrate_band if args.band else lv.litevar_window_calibrate
    for _ in range(args.warmup):
        radius = calibrate(scales, maps, args.r0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.iters):
        radius = calibrate(scales, maps, args.r0)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / args.iters
    off, causal = 0, 0
    for s in scales:
        off += s * s
        causal += s * s * off
    nbytes = 4 * causal * args.samples * args.heads
    r = radius.cpu()
    print(json.dumps({
        "metric": ("band" if args.band else "window") + " calibration, microseconds per call",
        "value": round(us, 2), "unit": "us",
        "higher_is_better": False, "dtype": "f64 sums over f32 maps",
        "data": "synthetic (seeded noisy bumps, block-causal rows summing to one)",
        "config": {"workload": "VAR 10-scale attention maps", "scales": list(scales),
                   "samples": args.samples, "heads": args.heads, "r0": args.r0},
        "roofline": {"bound": "hbm", "achieved": round(nbytes / (us * 1e-6) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "bytes_per_call": nbytes, "traffic": None},
        "radius_last_scale_head0": r[0, len(scales) - 1].tolist()}))


if __name__ == "__main__":
    main()
