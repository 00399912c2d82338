#!/usr/bin/env python3
"""Benchmark of the windowed-attention hot path on one MI355X.

One step = one generation step's attention for a whole model: the plan build
(scale table, window tables, work-list) followed by one windowed-attention forward per
transformer layer, each layer with its own Q/K/V/O tensors resident in HBM (so
consecutive launches never re-read the same inputs from cache).  The headline workload is
the VAR-d30 KV-cache step (256 queries of the 16x16 scale against all 680 keys, batch 16,
30 heads, radius 3, 30 layers).

Prints ONE JSON line: effective TFLOP/s on window-retained pairs, ms per step, the
attention kernel's HIP-event duration and roofline fraction, and the fp64 oracle's
throughput on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
LAYERS = {"tiny_f32": 1, "var_d16": 16, "var_d30_kvstep": 30, "var_d36_512": 36, "var_2k_cfg": 4}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="var_d30_kvstep")
    ap.add_argument("--layers", type=int, default=0, help="0 = the model's depth")
    ap.add_argument("--waves", type=int, default=0, help="compute waves per workgroup (0 = library default)")
    ap.add_argument("--chunk", type=int, default=0, help="keys per LDS chunk (0 = library default)")
    ap.add_argument("--depth", type=int, default=0, help="chunks in flight (0 = library default)")
    ap.add_argument("--spare", type=int, default=-1, help="spare ring chunks (-1 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--dense", action="store_true", help="dense block-causal path (radius -1)")
    return ap.parse_args()


def measured_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE runs, each scaled by a known-size copy kernel); None when
    no summary exists for this kernel instance."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        f"{kernel.split(chr(60))[0]}_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if " = " in line:
            a, b = line.split(" = ", 1)
            kv[a.strip()] = b.strip()
    if kv.get("kernel") != kernel or kv.get("workload") != workload:
        return None
    return int(kv["traffic_bytes_per_launch"])


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2411_17178_amd as lv
    import workloads
    from paper_2411_17178_amd.binding import prepare_attn_call

    lv.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    w = workloads.get(args.workload)
    tiling = (args.waves, args.chunk, args.depth, args.spare)
    layers = args.layers or LAYERS[w.name]
    radius = -1 if args.dense else w.radius
    tdtype = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    esize = 2 if w.dtype == "bf16" else 4

    # layer 0: the canonical seeded CPU recipe; other layers: same distribution drawn on the device
    q0, k0, v0 = workloads.make_workload_qkv(w)
    share = workloads.make_cfg_share(w.heads, len(w.scales), w.seed).to(dev) if w.cfg_share else None
    qs, ks, vs, os_ = [q0.to(dev)], [k0.to(dev)], [v0.to(dev)], []
    g = torch.Generator(device=dev).manual_seed(w.seed + 12345)
    for _ in range(1, layers):
        for lst, ref in ((qs, q0), (ks, k0), (vs, v0)):
            t = torch.randn(ref.shape, generator=g, device=dev, dtype=torch.float32) * w.input_scale
            lst.append(t.to(tdtype))
    for l in range(layers):
        os_.append(torch.empty_like(qs[l]))

    nbytes = lv.litevar_mask_plan_bytes(w.scales, radius, None, w.n_sink, w.q_scales, tiling)
    blob = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def build_plan():
        return lv.litevar_mask_build(w.scales, radius, None, w.n_sink, w.q_scales,
                                     waves_per_group=tiling, blob=blob)

    plan = build_plan()
    lv.litevar_plan_check(plan)
    calls = [prepare_attn_call(plan, qs[l], ks[l], vs[l], w.sm_scale, os_[l], share)
             for l in range(layers)]

    def step(ev0=None, ev1=None):
        p = build_plan()                      # a1-a3: tables and work-list, on the device
        assert p.n_steps == plan.n_steps
        if ev0 is not None:
            ev0.record()
        for c in calls:                       # a5-a10: one fused attention launch per layer
            c()
        if ev1 is not None:
            ev1.record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(*ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) / args.steps * 1e3
    attn_ms = sum(a.elapsed_time(b) for a, b in ev)            # all attention launches
    kernel_us = attn_ms * 1e3 / (args.steps * layers)          # average per launch

    BH = w.batch * w.heads
    pairs = plan.retained_pairs * BH
    if share is not None:   # shared uncond (head, query scale) rows are not computed
        qb, qe = w.q_range
        per_scale = np.zeros(len(w.scales), dtype=np.int64)
        for k in range(qb, qe):
            per_scale[k] = lv.litevar_mask_plan_stats(w.scales, radius, None, w.n_sink, (k, k + 1),
                                                      tiling).retained_pairs
        sh = share.cpu().numpy().astype(np.int64)
        pairs -= int((sh * per_scale[None, :]).sum()) * (w.batch // 2)
    flops_layer = 256.0 * pairs
    value = flops_layer * layers / (ms_per_step * 1e-3) / 1e12
    kernel_tflops = flops_layer / (kernel_us * 1e-6) / 1e12

    # algorithmic HBM bytes of one launch: Q read + O written (128 B per row each) and
    # K + V read once per (batch, head) (256 B per token)
    bytes_layer = BH * (2 * plan.q_len * 64 * esize + 2 * plan.kv_len * 64 * esize)
    achieved = bytes_layer / (kernel_us * 1e-6) / 1e9

    if w.dtype == "bf16" and plan.waves_per_group == 16:
        # the library's rule: one patch per wave when the working workgroups fit the CUs
        working = BH * plan.n_groups
        if share is not None:
            working = (working + 1) // 2
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        pw = plan.patches_per_wave or (1 if working <= cus else 2)
        kname = f"k_attn_bf16_pair<{pw}>"
    elif w.dtype == "bf16":
        kname = (f"k_attn_bf16<{plan.waves_per_group}, {plan.chunk_keys}, 1, {plan.prefetch_chunks}, "
                 f"{plan.ring_chunks - plan.prefetch_chunks - 2}>")
    else:
        kname = "k_attn_f32"
    traffic = None if args.dense else measured_traffic(w.name, kname)

    out = {
        "metric": "windowed-attn effective TFLOP/s (retained pairs)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic (seeded N(0,1); layer 0 from the CPU recipe, other layers drawn on the device)",
        "config": {"workload": w.name + ("_dense" if args.dense else ""), "scales": list(w.scales),
                   "batch": w.batch, "heads": w.heads, "head_dim": w.head_dim, "radius": radius,
                   "q_len": plan.q_len, "kv_len": plan.kv_len, "layers_per_step": layers,
                   "cfg_share": bool(w.cfg_share), "waves_per_group": plan.waves_per_group,
                   "chunk_keys": plan.chunk_keys, "ring_chunks": plan.ring_chunks,
                   "prefetch_chunks": plan.prefetch_chunks,
                   "step": "plan build + one attention forward per layer"},
        "us_per_layer": round(kernel_us, 3),
        "kernel_tflops_retained": round(kernel_tflops, 2),
        "mfma_frac_retained": round(kernel_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "tile_density": round(plan.retained_pairs / plan.computed_pairs, 4),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "kernel": kname,
                     "bytes_per_launch": bytes_layer, "kernel_us": round(kernel_us, 3)},
    }

    if not args.no_cpu_baseline:
        import oracle
        radii = [radius] * len(w.scales)
        arrs = [workloads.to_oracle_array(t) for t in (q0, k0, v0)]
        # bounded sample: time a few (batch, head) pairs, then as many as fit the budget
        n0 = min(BH, oracle.num_threads())
        ta = time.perf_counter()
        oracle.attn(w.scales, radii, *arrs, w.sm_scale, w.n_sink, w.q_scales, bh_range=(0, n0))
        dt0 = time.perf_counter() - ta
        n = int(max(n0, min(BH, n0 * args.cpu_seconds / max(dt0, 1e-3))))
        # repeat the sample until about cpu_seconds of oracle time have been spent
        reps, dt = 0, 0.0
        while reps == 0 or (dt < args.cpu_seconds and n == BH):
            ta = time.perf_counter()
            ref = oracle.attn(w.scales, radii, *arrs, w.sm_scale, w.n_sink, w.q_scales, bh_range=(0, n))
            dt += time.perf_counter() - ta
            reps += 1
        got = os_[0].float().cpu().numpy().reshape(BH, plan.q_len, 64)[:n]
        if share is not None:
            got, ref_c = got[: min(n, BH // 2)], ref.reshape(BH, plan.q_len, 64)[: min(n, BH // 2)]
        else:
            ref_c = ref.reshape(BH, plan.q_len, 64)[:n]
        err = float(np.abs(got - ref_c).max())
        out["cpu_baseline"] = {
            "value": round(256.0 * plan.retained_pairs * n * reps / dt / 1e12, 6), "unit": "TFLOP/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of {BH} (batch, head) pairs of one layer, {reps} time(s), {dt:.2f} s",
            "gpu_vs_oracle_max_abs_err": err}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
