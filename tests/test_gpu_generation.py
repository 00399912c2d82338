"""All KV-cache generation steps of one layer (paper Section 2: scale-by-scale generation;
Section 3: the unconditional half reuses the conditional half's attention output) through
the C ABI, against the oracle's full-sequence result: block-causal attention makes the rows
of scale k depend on the keys of scales <= k only, so the per-step outputs concatenate to the
full-sequence output."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
VAR_SCALES = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    m.load_library()
    return m


def _full_reference(scales, radius, q, k, v, n_sink, share_all):
    arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
    ref = oracle.attn(scales, [radius] * len(scales), *arrs, 0.125, n_sink, None, None, None)
    if share_all:
        H = q.shape[1]
        oracle.cfg_share(scales, ref, np.ones((H, len(scales)), dtype=np.uint8), None)
    return ref


def _run_steps(gen, q, k, v, dtype, share_all):
    """Scale-by-scale generation: the caches hold NaN beyond the scales appended so far, so a
    step that read a future key would poison its output."""
    from paper_2411_17178_amd.generation import GenerationLayer  # noqa: F401
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    k_cache = torch.full_like(kd, float("nan"))
    v_cache = torch.full_like(vd, float("nan"))
    out = torch.empty_like(qd)
    for s in range(gen.n_steps):
        lo, hi = gen.rows(s)
        k_cache[:, :, lo:hi] = kd[:, :, lo:hi]         # in-place append of scale s
        v_cache[:, :, lo:hi] = vd[:, :, lo:hi]
        print(f"  generation step {s}: queries [{lo}, {hi}) {dtype} share_all={share_all}", flush=True)
        q_s = qd[:, :, lo:hi]                           # strided views: no copies
        gen.step(s, q_s, k_cache, v_cache, 0.125, out_k=out[:, :, lo:hi], share_all=share_all)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("share_all", [False, True])
def test_generation_steps_concatenate_to_the_full_sequence(lv, dtype, share_all):
    from paper_2411_17178_amd.generation import GenerationLayer
    radius, n_sink, B, H = 2, 3, 2, 3
    q, k, v = workloads.make_qkv(VAR_SCALES, B, H, 64, dtype, 77, 1.0, None)
    gen = GenerationLayer(VAR_SCALES, radius, n_sink_scales=n_sink)
    assert gen.kv_len == 680 and gen.n_steps == 10
    out = _run_steps(gen, q, k, v, dtype, share_all)
    assert bool(torch.isfinite(out.float()).all()), "a step read a key of a later scale"
    ref = _full_reference(VAR_SCALES, radius, q, k, v, n_sink, share_all)
    err = float(np.abs(out.float().cpu().numpy().astype(np.float64) - ref).max())
    assert err <= TOL[dtype], err
    if share_all:      # the unconditional rows are copies of the conditional ones
        assert torch.equal(out[B // 2:], out[:B // 2])
    # the steps' retained pairs add up to the full sequence's
    full = lv.litevar_mask_plan_stats(VAR_SCALES, radius, None, n_sink)
    assert gen.retained_pairs() == int(full.retained_pairs)


def test_generation_layer_in_a_graph(lv):
    """The ten calls of a layer captured in one HIP graph: every replay, with eager work and
    synchronisations of the program's own between the replays, equals the eager result."""
    from paper_2411_17178_amd.generation import GenerationLayer
    radius, B, H = 3, 2, 4
    gen = GenerationLayer(VAR_SCALES, radius)
    q, k, v = workloads.make_qkv(VAR_SCALES, B, H, 64, "bf16", 5, 1.0, None)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    q_steps = [qd[:, :, lo:hi] for lo, hi in map(gen.rows, range(gen.n_steps))]
    eager = torch.empty_like(qd)
    for s in range(gen.n_steps):
        lo, hi = gen.rows(s)
        gen.step(s, q_steps[s], kd, vd, 0.125, out_k=eager[:, :, lo:hi], share_all=True)
    torch.cuda.synchronize()

    out = torch.zeros_like(qd)
    out_steps = [out[:, :, lo:hi] for lo, hi in map(gen.rows, range(gen.n_steps))]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        calls = gen.prepare(q_steps, kd, vd, 0.125, out_steps, share_all=True, stream=side)
        print("  capturing the ten steps", flush=True)
        with torch.cuda.graph(graph, stream=side):
            for call in calls:
                call()
    for rep in range(4):
        out.fill_(float(rep))                     # eager work between the replays
        torch.cuda.synchronize()
        print(f"  replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
        scratch = (out.float() * 2).sum().item()  # more eager work, a library reduction included
        assert np.isfinite(scratch)


@pytest.mark.parametrize("share_all", [False, True])
def test_generation_steps_on_an_8_bit_cache(lv, share_all):
    """Section 4 on the generation path: K and V live in the cache as 8-bit codes with one
    (scale, zero point) per token; rows of later scales carry NaN parameters, so a step that
    read one would poison its output.  Quantisation is per token, so the steps concatenate to
    the oracle's full-sequence result on quantised operands."""
    from paper_2411_17178_amd.generation import GenerationLayer
    radius, n_sink, B, H = 2, 0, 2, 3
    q, k, v = workloads.make_qkv(VAR_SCALES, B, H, 64, "bf16", 78, 1.0, None)
    gen = GenerationLayer(VAR_SCALES, radius, n_sink_scales=n_sink)
    (k8, kz), (v8, vz) = lv.litevar_qkv8_quantize(k.cuda()), lv.litevar_qkv8_quantize(v.cuda())
    k_cache, v_cache = torch.zeros_like(k8), torch.zeros_like(v8)
    kz_cache, vz_cache = torch.full_like(kz, float("nan")), torch.full_like(vz, float("nan"))
    work = torch.empty(gen.qkv8_workspace_bytes(B, H), dtype=torch.uint8, device="cuda")
    out = torch.empty(q.shape, dtype=torch.bfloat16, device="cuda")
    for s in range(gen.n_steps):
        lo, hi = gen.rows(s)
        for cache, src in ((k_cache, k8), (v_cache, v8), (kz_cache, kz), (vz_cache, vz)):
            cache[:, :, lo:hi] = src[:, :, lo:hi]      # in-place append of scale s
        q8, qz = lv.litevar_qkv8_quantize(q[:, :, lo:hi].contiguous().cuda())
        print(f"  8-bit generation step {s}: queries [{lo}, {hi}) share_all={share_all}", flush=True)
        out[:, :, lo:hi] = gen.step_qkv8(s, q8, qz, k_cache, kz_cache, v_cache, vz_cache, 0.125,
                                         share_all=share_all, workspace=work)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all()), "a step read a key of a later scale"
    arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
    ref = oracle.attn_qkv8(VAR_SCALES, [radius] * len(VAR_SCALES), *arrs, 0.125, n_sink, None)
    if share_all:
        oracle.cfg_share(VAR_SCALES, ref, np.ones((H, len(VAR_SCALES)), dtype=np.uint8), None)
    err = float(np.abs(out.float().cpu().numpy().astype(np.float64) - ref).max())
    print(f"  8-bit cache generation: max-abs err {err:.3e}")
    assert err <= 3e-2, err
