"""Times all KV-cache generation steps of the attention layers of a VAR model (paper
Section 2: scale-by-scale generation) on one GPU: per layer, one library call per scale, the
queries being that scale's tokens and the keys the cache rows of the scales so far; with
--asc the unconditional half of the batch reuses the conditional half's attention output
everywhere (paper Section 3).  Run as

    python -m paper_2411_17178_amd.bench_generation [--workload var_d30_kvstep] [--asc] [--graph]

Prints one JSON line: microseconds per layer (all steps of one layer), per step, and the
effective TFLOP/s over the retained (query, key) pairs that were computed.  Inputs are
seeded synthetic N(0,1) tensors resident in HBM, each layer with its own Q, K, V and O.
"""
import argparse
import json
import sys
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="var_d30_kvstep", help="gives scales, radius, batch, heads")
    ap.add_argument("--layers", type=int, default=30)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--asc", action="store_true", help="share the conditional output everywhere")
    ap.add_argument("--graph", action="store_true", help="replay each layer's steps as one HIP graph")
    ap.add_argument("--batch", type=int, default=0, help="batch size (0 = the workload's)")
    ap.add_argument("--no-hint", action="store_true", help="do not tell the plans the batch size")
    args = ap.parse_args()

    import torch

    import paper_2411_17178_amd as lv
    import workloads
    from paper_2411_17178_amd.generation import GenerationLayer

    lv.load_library()
    if not torch.cuda.is_available():
        print("bench_generation: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    w = workloads.get(args.workload)
    B, H = args.batch or w.batch, w.heads
    working = B * H // 2 if args.asc else B * H          # (batch, head) pairs that compute
    gen = GenerationLayer(w.scales, w.radius, n_sink_scales=w.n_sink, device=dev,
                          batch_heads=0 if args.no_hint else working)
    L = gen.kv_len
    g = torch.Generator(device=dev).manual_seed(w.seed + 999)

    def draw():
        return (torch.randn((B, H, L, 64), generator=g, device=dev) * w.input_scale).to(torch.bfloat16)

    calls = []
    keep = []
    for _ in range(args.layers):
        q, k, v = draw(), draw(), draw()
        o = torch.empty_like(q)
        rows = [gen.rows(s) for s in range(gen.n_steps)]
        q_steps = [q[:, :, lo:hi] for lo, hi in rows]
        o_steps = [o[:, :, lo:hi] for lo, hi in rows]
        keep.append((q, k, v, o))
        calls.append((q_steps, k, v, o_steps))

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        layer_calls = [gen.prepare(qs, k, v, w.sm_scale, os_, share_all=args.asc, stream=stream)
                       for qs, k, v, os_ in calls]
        if args.graph:
            graphs = []
            for lc in layer_calls:
                for c in lc:        # one eager pass first
                    c()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=stream):
                    for c in lc:
                        c()
                graphs.append(gr)

            def run_all():
                for gr in graphs:
                    gr.replay()
        else:
            def run_all():
                for lc in layer_calls:
                    for c in lc:
                        c()

        for _ in range(args.warmup):
            run_all()
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.iters):
            run_all()
        stream.synchronize()
        t1 = time.perf_counter()

    us_layer = (t1 - t0) / (args.iters * args.layers) * 1e6
    pairs = gen.retained_pairs() * H * (B // 2 if args.asc else B)
    print(json.dumps({
        "metric": "windowed-attn effective TFLOP/s (retained pairs), all generation steps of a layer",
        "value": round(256.0 * pairs / (us_layer * 1e-6) / 1e12, 3), "unit": "TFLOP/s",
        "us_per_layer": round(us_layer, 2), "us_per_step": round(us_layer / gen.n_steps, 2),
        "steps_per_layer": gen.n_steps, "layers": args.layers, "iters": args.iters,
        "dtype": "bf16", "data": "synthetic (seeded N(0,1), drawn on the device)",
        "config": {"workload": w.name + " (all steps)", "scales": list(w.scales), "batch": B,
                   "heads": H, "radius": w.radius, "asc_everywhere": bool(args.asc),
                   "patches_per_group": [int(p.waves_per_group) for p in gen.plans],
                   "hip_graph": bool(args.graph)}}))


if __name__ == "__main__":
    main()
