#!/usr/bin/env python3
"""Benchmark of the windowed-attention hot path on one MI355X.

One step = one generation step's attention for a whole model: the plan build
(scale table, window tables, work-list) followed by one windowed-attention forward per
transformer layer, each layer with its own Q/K/V/O tensors resident in HBM (so
consecutive launches never re-read the same inputs from cache).  The headline workload is
the VAR-d30 KV-cache step (256 queries of the 16x16 scale against all 680 keys, batch 16,
30 heads, radius 3, 30 layers).

Prints ONE JSON line: effective TFLOP/s on window-retained pairs, ms per step, the
attention kernel's HIP-event duration and roofline fraction, the fp64 oracle's throughput
on the host cores as a reported baseline, what this GPU delivers on a streaming copy and a
register-only MFMA loop (`measured_peaks`), and -- unless --no-extra -- a shorter
measurement of the other workloads (`workloads`: VAR-d16, VAR-d36 windowed and dense
block-causal, the 2K sequence with output sharing).
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
EXTRA = [("var_d16", False), ("var_d36_512", False), ("var_d36_512", True), ("var_2k_cfg", False)]


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
    ap.add_argument("--ppw", type=int, default=0, help="16 patches per group: patches per wave (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--dense", action="store_true", help="dense block-causal path (radius -1)")
    ap.add_argument("--no-extra", action="store_true", help="headline workload only")
    return ap.parse_args()


def measured_traffic(workload, kernel, kernel_us):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE runs, each scaled by a known-size copy kernel).  None when no
    summary exists for this kernel instance, or when the kernel time recorded with the
    counters differs from this run's by more than 8 % (the summary then describes another
    version of the kernel; short runs under the profiler are a few per cent slower than a
    long run without it)."""
    path = os.path.join(ROOT, "profiles", f"{kernel.split(chr(60))[0]}_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if " = " in line:
            a, b = line.split(" = ", 1)
            kv[a.strip()] = b.strip()
    if kv.get("kernel") != kernel or kv.get("workload") != workload or "kernel_us" not in kv:
        return None
    if abs(float(kv["kernel_us"]) - kernel_us) > 0.08 * kernel_us:
        return None
    return int(kv["traffic_bytes_per_launch"])


def kernel_name(plan, w, working, cus):
    if w.dtype == "bf16" and plan.waves_per_group == 16:
        # the library's rule: one patch per wave when the working workgroups fit the CUs
        pw = plan.patches_per_wave or (1 if working <= cus else 2)
        return f"k_attn_bf16_pair<{pw}, false>"
    if w.dtype == "bf16":
        return (f"k_attn_bf16<{plan.waves_per_group}, {plan.chunk_keys}, 1, {plan.prefetch_chunks}, "
                f"{plan.ring_chunks - plan.prefetch_chunks - 2}>")
    return "k_attn_f32"


def run_workload(name, dense, steps, warmup, layers, tiling, keep_layer0=False):
    """Times `steps` steps (plan build + one attention launch per layer) of one workload;
    returns (result dict, context for the oracle leg)."""
    import numpy as np
    import torch

    import paper_2411_17178_amd as lv
    import workloads
    from paper_2411_17178_amd.binding import prepare_attn_call

    dev = torch.device("cuda:0")
    w = workloads.get(name)
    radius = -1 if dense else w.radius
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

    # (the plan is told the B * H of its launches: small batches get smaller groups)
    BH = w.batch * w.heads
    nbytes = lv.litevar_mask_plan_bytes(w.scales, radius, None, w.n_sink, w.q_scales, tiling, batch_heads=BH)
    blob = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def build_plan():
        return lv.litevar_mask_build(w.scales, radius, None, w.n_sink, w.q_scales,
                                     waves_per_group=tiling, blob=blob, batch_heads=BH)

    plan = build_plan()
    lv.litevar_plan_check(plan)
    calls = [prepare_attn_call(plan, qs[l], ks[l], vs[l], w.sm_scale, os_[l], share)
             for l in range(layers)]

    def step(ev0=None, ev1=None):
        p = build_plan()                      # scale table, window tables and work-list, on the device
        assert p.n_steps == plan.n_steps
        if ev0 is not None:
            ev0.record()
        for c in calls:                       # one fused attention launch per layer
            c()
        if ev1 is not None:
            ev1.record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(*ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) / steps * 1e3
    attn_ms = sum(a.elapsed_time(b) for a, b in ev)       # all attention launches
    kernel_us = attn_ms * 1e3 / (steps * layers)          # average per launch

    pairs = plan.retained_pairs * BH
    if share is not None:   # shared uncond (head, query scale) rows are not computed
        qb, qe = w.q_range
        per_scale = np.zeros(len(w.scales), dtype=np.int64)
        for k in range(qb, qe):
            per_scale[k] = lv.litevar_mask_plan_stats(w.scales, radius, None, w.n_sink, (k, k + 1),
                                                      tiling, batch_heads=BH).retained_pairs
        sh = share.cpu().numpy().astype(np.int64)
        pairs -= int((sh * per_scale[None, :]).sum()) * (w.batch // 2)
    flops_layer = 256.0 * pairs
    value = flops_layer * layers / (ms_per_step * 1e-3) / 1e12
    kernel_tflops = flops_layer / (kernel_us * 1e-6) / 1e12

    # algorithmic HBM bytes of one launch: Q read + O written (128 B per row each) and
    # K + V read once per (batch, head) (256 B per token)
    bytes_layer = BH * (2 * plan.q_len * 64 * esize + 2 * plan.kv_len * 64 * esize)
    achieved = bytes_layer / (kernel_us * 1e-6) / 1e9
    t_mfma_us = flops_layer / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6
    t_hbm_us = bytes_layer / (HBM_PEAK_GBS * 1e9) * 1e6

    working = BH * plan.n_groups
    if share is not None:
        working = (working + 1) // 2
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    kname = kernel_name(plan, w, working, cus)
    res = {
        "workload": w.name + ("_dense" if dense else ""), "kernel": kname,
        "us_per_layer": round(kernel_us, 3), "ms_per_step": round(ms_per_step, 4),
        "step_tflops_retained": round(value, 3),
        "kernel_tflops_retained": round(kernel_tflops, 2),
        "mfma_frac_retained": round(kernel_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "hbm_gbs": round(achieved, 1), "hbm_frac": round(achieved / HBM_PEAK_GBS, 4),
        # the roofline that binds: the larger of the two floors against the measured time
        "bound": "hbm" if t_hbm_us >= t_mfma_us else "mfma",
        "floor_us": round(max(t_hbm_us, t_mfma_us), 2),
        "binding_roofline_frac": round(max(t_hbm_us, t_mfma_us) / kernel_us, 4),
        "tile_density": round(plan.retained_pairs / plan.computed_pairs, 4),
        "retained_pairs_per_bh": int(plan.retained_pairs), "layers": layers, "steps": steps,
        "bytes_per_launch": bytes_layer,
    }
    ctx = dict(w=w, plan=plan, radius=radius, q0=q0, k0=k0, v0=v0, o0=os_[0], share=share, BH=BH)
    if not keep_layer0:
        ctx = None
    return res, ctx


def run_variants(steps=8, layers=8):
    """The rows built beyond the bf16 window path, on the headline shape (VAR-d30 KV step):
    8-bit Q/K/V (paper Section 4), the band reading of the window, one radius table per head."""
    import numpy as np
    import torch

    import paper_2411_17178_amd as lv
    import workloads

    dev = torch.device("cuda:0")
    w = workloads.get("var_d30_kvstep")
    BH, K = w.batch * w.heads, len(w.scales)
    g = torch.Generator(device=dev).manual_seed(99)
    qs = [torch.randn((w.batch, w.heads, 256, 64), generator=g, device=dev).to(torch.bfloat16) for _ in range(layers)]
    ks = [torch.randn((w.batch, w.heads, 680, 64), generator=g, device=dev).to(torch.bfloat16) for _ in range(layers)]
    vs = [torch.randn((w.batch, w.heads, 680, 64), generator=g, device=dev).to(torch.bfloat16) for _ in range(layers)]
    outs = [torch.empty_like(q) for q in qs]

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps          # us

    def attn_us(plan):
        def layer_pass():
            for l in range(layers):
                lv.litevar_windowed_attn_fwd(plan, qs[l], ks[l], vs[l], w.sm_scale, out=outs[l])
        return timed(layer_pass, steps) / layers

    out = []
    base = lv.litevar_mask_build(w.scales, w.radius, None, w.n_sink, w.q_scales, batch_heads=BH)
    t_base = attn_us(base)

    # ---- QKV8: quantiser (HBM-bound: 128 B read, 64 + 8 B written per row) and attention on 8-bit operands
    t_quant = timed(lambda: [lv.litevar_qkv8_quantize(k) for k in ks], steps) / layers
    rows = BH * 680
    q8 = [lv.litevar_qkv8_quantize(t) for t in qs]
    k8 = [lv.litevar_qkv8_quantize(t) for t in ks]
    v8 = [lv.litevar_qkv8_quantize(t) for t in vs]
    work = torch.empty(lv.litevar_windowed_attn_qkv8_workspace_bytes(base, w.batch, w.heads), dtype=torch.uint8,
                       device=dev)      # (empty: the KV-step plan converts in the attention kernel)

    def qkv8_pass():
        for l in range(layers):
            lv.litevar_windowed_attn_qkv8_fwd(base, *q8[l], *k8[l], *v8[l], w.sm_scale, out=outs[l], workspace=work)
    t_q8 = timed(qkv8_pass, steps) / layers

    def copy_pass():                     # the other route: one dequantising pass, then the bf16 kernel
        for l in range(layers):
            lv.litevar_windowed_attn_fwd(base, *(lv.litevar_qkv8_dequantize(*t[l]) for t in (q8, k8, v8)),
                                         w.sm_scale, out=outs[l])
    t_copy = timed(copy_pass, steps) / layers
    bytes_q8 = BH * (256 * (72 + 128) + 2 * 680 * 72)
    out.append({"variant": "qkv8", "section": "Section 4",
                "quantize_us_per_tensor": round(t_quant, 2),
                "quantize_gbs": round(rows * (128 + 72) / (t_quant * 1e-6) / 1e9, 1),
                "quantize_frac_of_hbm_spec": round(rows * (128 + 72) / (t_quant * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                "attn_us_per_layer": round(t_q8, 2), "bf16_attn_us_per_layer": round(t_base, 2),
                "algorithmic_bytes": bytes_q8,
                "hbm_frac_of_spec_on_8bit_bytes": round(bytes_q8 / (t_q8 * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                "dequantise_pass_then_bf16_us_per_layer": round(t_copy, 2),
                "note": "codes and (scale, zero point) go straight into the attention kernel, which converts "
                        "them on their way into LDS (registers instead of LDS-DMA); the conversion costs "
                        "vector instructions that the bf16 kernel does not have"})
    del q8, k8, v8, work

    # ---- band reading of the window (Section 2, step (2)): bands as wide as the window's footprint
    band = lv.litevar_mask_build(w.scales, 24, None, w.n_sink, w.q_scales, batch_heads=BH, mask_mode=1)
    t_band = attn_us(band)
    out.append({"variant": "band_1d_radius_24", "section": "Section 2 step (2)",
                "attn_us_per_layer": round(t_band, 2), "retained_pairs_per_bh": int(band.retained_pairs),
                "kernel_tflops_retained": round(256.0 * band.retained_pairs * BH / (t_band * 1e-6) / 1e12, 1),
                "tile_density": round(band.retained_pairs / band.computed_pairs, 4)})

    # ---- one radius table per head (Section 2, step (3)): thirty heads, radii 2..4 per part
    rng = np.random.default_rng(7)
    tabs = rng.integers(2, 5, size=(w.heads, K, K))
    ph = lv.litevar_mask_build(w.scales, 0, tabs.tolist(), w.n_sink, w.q_scales, batch_heads=BH)
    t_ph = attn_us(ph)
    pairs = sum(int(ph.retained_pairs_of_group[ph.head_group[h]]) for h in range(w.heads)) * w.batch
    out.append({"variant": "radius_table_per_head", "section": "Section 2 step (3)",
                "attn_us_per_layer": round(t_ph, 2), "heads": w.heads, "head_groups": int(ph.n_head_groups),
                "kernel_tflops_retained": round(256.0 * pairs / (t_ph * 1e-6) / 1e12, 1),
                "plan_bytes": int(ph.blob_bytes)})
    return out


def measure_peaks():
    """Streaming-copy GB/s (read + write) and register-only bf16 MFMA TFLOP/s of this GPU."""
    import torch

    import paper_2411_17178_amd as lv
    dev = torch.device("cuda:0")
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    out = torch.zeros(1, dtype=torch.float32, device=dev)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    t_copy = timed(lambda: lv.litevar_peak_copy(src, dst), 10)
    t_read = timed(lambda: lv.litevar_peak_read(src, out), 10)
    flops = [0.0]

    def mfma():
        flops[0] = lv.litevar_peak_mfma_bf16(2048, out)
    t_mfma = timed(mfma, 5)
    del src, dst
    return {"copy_gbs": round(2 * n / t_copy / 1e9, 1), "copy_bytes": 2 * n,
            "copy_frac_of_spec": round(2 * n / t_copy / 1e9 / HBM_PEAK_GBS, 4),
            "read_gbs": round(n / t_read / 1e9, 1),
            "read_frac_of_spec": round(n / t_read / 1e9 / HBM_PEAK_GBS, 4),
            "mfma_bf16_tflops": round(flops[0] / t_mfma / 1e12, 1),
            "mfma_frac_of_spec": round(flops[0] / t_mfma / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "spec": {"hbm_gbs": HBM_PEAK_GBS, "mfma_bf16_tflops": MFMA_BF16_PEAK_TFLOPS}}


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

    lv.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    tiling = (args.waves, args.chunk, args.depth, args.spare, args.ppw)
    w = workloads.get(args.workload)
    layers = args.layers or LAYERS[w.name]
    res, ctx = run_workload(args.workload, args.dense, args.steps, args.warmup, layers, tiling,
                            keep_layer0=True)
    plan, radius = ctx["plan"], ctx["radius"]
    traffic = None if args.dense else measured_traffic(w.name, res["kernel"], res["us_per_layer"])

    out = {
        "metric": "windowed-attn effective TFLOP/s (retained pairs)",
        "value": res["step_tflops_retained"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic (seeded N(0,1); layer 0 from the CPU recipe, other layers drawn on the device)",
        "config": {"workload": res["workload"], "scales": list(w.scales),
                   "batch": w.batch, "heads": w.heads, "head_dim": w.head_dim, "radius": radius,
                   "q_len": plan.q_len, "kv_len": plan.kv_len, "layers_per_step": layers,
                   "cfg_share": bool(w.cfg_share), "waves_per_group": plan.waves_per_group,
                   "chunk_keys": plan.chunk_keys, "ring_chunks": plan.ring_chunks,
                   "prefetch_chunks": plan.prefetch_chunks,
                   "step": "plan build + one attention forward per layer"},
        "us_per_layer": res["us_per_layer"],
        "kernel_tflops_retained": res["kernel_tflops_retained"],
        "mfma_frac_retained": res["mfma_frac_retained"],
        "binding_roofline_frac": res["binding_roofline_frac"],
        "tile_density": res["tile_density"],
        "roofline": {"bound": "hbm", "achieved": res["hbm_gbs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": res["hbm_frac"], "traffic": traffic,
                     "traffic_source": ("committed rocprofv3 --pmc summary under profiles/ (not measured by "
                                        "this run); dropped when its kernel time is not this run's"),
                     "kernel": res["kernel"],
                     "bytes_per_launch": res["bytes_per_launch"], "kernel_us": res["us_per_layer"]},
    }

    if not args.no_cpu_baseline:
        import oracle
        BH, q0, k0, v0, share = ctx["BH"], ctx["q0"], ctx["k0"], ctx["v0"], ctx["share"]
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
        got = ctx["o0"].float().cpu().numpy().reshape(BH, plan.q_len, 64)[:n]
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
    del ctx
    torch.cuda.empty_cache()

    out["measured_peaks"] = measure_peaks()
    if not args.no_extra and not args.dense and args.workload == "var_d30_kvstep":
        extra = []
        for name, dense in EXTRA:
            torch.cuda.empty_cache()
            r, _ = run_workload(name, dense, 4 if dense else 8, 2, min(LAYERS[name], 8), (0, 0, 0, -1, 0))
            extra.append(r)
        win = next(r for r in extra if r["workload"] == "var_d36_512")
        den = next(r for r in extra if r["workload"] == "var_d36_512_dense")
        out["workloads"] = extra
        torch.cuda.empty_cache()
        out["variants"] = run_variants()
        out["d36_windowed_vs_dense"] = {
            "speedup": round(den["us_per_layer"] / win["us_per_layer"], 3),
            "flop_ratio": round(den["retained_pairs_per_bh"] / win["retained_pairs_per_bh"], 3)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
