"""Where the time of one launch of the 16-patch attention kernel goes, wave by wave.

Uses the profiling build of the library (`python -m paper_2411_17178_amd.build --timeline`,
-DLITEVAR_TIMELINE): every wave of k_attn_bf16_pair<2> records wall-clock stamps (start,
tokens in, loads issued and landed, first barrier, end of the phase loop, stored) and cycle
sums (in steps, issuing loads, waiting for memory, at barriers) into a buffer whose address
the library reads from the environment.  Run on a GPU as

    python -m paper_2411_17178_amd.timeline [workload]

Each of six layers gets its own inputs, so that no launch finds its data in a cache; the
last launch of the second pass is the one that is recorded.
"""
import collections
import os
import sys

import numpy as np


def main():
    import torch

    from . import binding, build
    if not os.path.exists(build.LIB_TIMELINE):
        raise SystemExit(f"{build.LIB_TIMELINE} is missing: run `python -m paper_2411_17178_amd.build --timeline`")
    binding._LIB_PATH = build.LIB_TIMELINE
    import paper_2411_17178_amd as lv
    import workloads

    w = workloads.get(sys.argv[1] if len(sys.argv) > 1 else "var_d30_kvstep")
    plan = lv.litevar_mask_build(w.scales, w.radius, None, w.n_sink, w.q_scales,
                                 waves_per_group=(16, 0, 0, -1, 2))
    BH = w.batch * w.heads
    nblk = (BH + 7) // 8 * 8 * plan.n_groups
    dev = torch.device("cuda")
    q0, k0, v0 = workloads.make_workload_qkv(w)
    L = 6
    qs = [torch.randn_like(q0.float()).to(q0.dtype).to(dev) for _ in range(L)]
    ks = [torch.randn_like(k0.float()).to(k0.dtype).to(dev) for _ in range(L)]
    vs = [torch.randn_like(v0.float()).to(v0.dtype).to(dev) for _ in range(L)]
    outs = [torch.empty_like(q) for q in qs]
    tl = torch.zeros(nblk * 8 * 16, dtype=torch.int64, device=dev)
    for rep in range(2):
        for l in range(L):
            if rep == 1 and l == L - 1:
                os.environ["LITEVAR_TIMELINE_PTR"] = hex(tl.data_ptr())
            lv.litevar_windowed_attn_fwd(plan, qs[l], ks[l], vs[l], w.sm_scale, out=outs[l])
    torch.cuda.synchronize()
    os.environ.pop("LITEVAR_TIMELINE_PTR", None)

    d = tl.cpu().numpy().reshape(nblk, 8, 16).astype(np.float64)
    d = d[d[:, 0, 0] > 0]                                  # workgroups that ran
    t0 = d[:, :, 0].min()
    us = lambda x: (x - t0) / 100.0                        # the wall clock runs at 100 MHz
    start, end = us(d[:, :, 0].min(axis=1)), us(d[:, :, 6].max(axis=1))
    loop_us = (d[:, :, 5] - d[:, :, 4]) / 100.0
    mhz = float(np.median(d[:, :, 11] / np.maximum(loop_us, 1e-9)))
    med = lambda x: float(np.median(x))
    cyc = lambda i: med(d[:, :, i]) / mhz
    print(f"{w.name}: {len(d)} workgroups, launch {end.max():.2f} us, shader clock in the loop {mhz:.0f} MHz")
    print("workgroup duration, percentiles 0/25/50/75/100: ",
          np.percentile(end - start, [0, 25, 50, 75, 100]).round(2))
    print("start-up (us after the workgroup's start, median wave): tokens and plan words in %.2f, "
          "loads and chunks issued %.2f, landed %.2f, first barrier passed %.2f"
          % tuple(med(us(d[:, :, i]) - us(d[:, :, 0])) for i in (1, 2, 3, 4)))
    rest = med(loop_us - (d[:, :, 8] + d[:, :, 9] + d[:, :, 10] + d[:, :, 13]) / mhz)
    print("phase loop %.2f us = steps %.2f + issuing loads %.2f + waiting for memory %.2f + barriers %.2f + rest %.2f; "
          "store %.2f us" % (med(loop_us), cyc(8), cyc(9), cyc(13), cyc(10), rest,
                             med((d[:, :, 6] - d[:, :, 5]) / 100.0)))
    for wv in range(8):
        print("   wave %d: steps %.2f, issuing %.2f, waiting %.2f, barriers %.2f"
              % tuple([wv] + [med(d[:, wv, i]) / mhz for i in (8, 9, 13, 10)]))
    # workgroups per CU, from the hardware id (XCC, SE, CU)
    hw = d[:, 0, 12].astype(np.int64)
    cu = ((hw >> 32) & 0xf) * 1000 + ((hw >> 13) & 7) * 100 + ((hw >> 12) & 1) * 10 + ((hw >> 8) & 0xf)
    count = collections.Counter(cu.tolist())
    for n in sorted(set(count.values())):
        sel = np.array([count[c] == n for c in cu.tolist()])
        print(f"   CUs with {n} workgroup(s): {sel.sum()} workgroups, duration median "
              f"{np.median((end - start)[sel]):.2f} us, last end {end[sel].max():.2f} us")


if __name__ == "__main__":
    main()
