"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle.

Integer outputs (window tables, masks, index sets) must match bit-exactly; attention
outputs within 1e-5 (fp32) / 2e-2 (bf16 inputs, fp32 accumulation) max-abs.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    m.load_library()
    return m


def _plan(lv, w, waves=0, **over):
    scales = over.get("scales", w.scales)
    return lv.litevar_mask_build(scales, over.get("radius", w.radius), over.get("radii"),
                                 over.get("n_sink", w.n_sink), over.get("q_scales", w.q_scales),
                                 waves_per_group=waves)


def _gpu_attn(lv, plan, q, k, v, sm_scale, share=None):
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    sd = share.cuda() if share is not None else None
    print(f"  attn fwd: q{tuple(q.shape)} kv{tuple(k.shape)} {q.dtype} waves={plan.waves_per_group}",
          flush=True)
    o = lv.litevar_windowed_attn_fwd(plan, qd, kd, vd, sm_scale, cfg_share=sd)
    torch.cuda.synchronize()
    return o


def _oracle_attn(scales, radii, q, k, v, sm_scale, n_sink=0, q_scales=None, rows=None, share=None,
                 bh_range=None):
    arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
    ref = oracle.attn(scales, radii, *arrs, sm_scale, n_sink, q_scales, rows, bh_range)
    if share is not None:
        assert rows is None
        oracle.cfg_share(scales, ref, share.numpy(), q_scales)
    return ref


def _maxerr(o_gpu, ref):
    return float(np.abs(o_gpu.float().cpu().numpy().astype(np.float64) - ref).max())


# ---- integer work: window tables, masks, index sets --------------------------------

def _window_table_from_oracle(scales, radii, n_sink):
    """[K][K][smax][2] from the oracle's dense mask: the key rows query (k, c, 0) keeps."""
    K, smax = len(scales), max(scales)
    off = oracle.scale_offsets(scales)
    m = oracle.mask_dense(scales, radii, n_sink)
    out = -np.ones((K, K, smax, 2), dtype=np.int16)
    for k in range(K):
        for c in range(scales[k]):
            row = m[off[k] + c * scales[k]]            # query (k, y=c, x=0)
            for j in range(k + 1):
                blk = row[off[j]:off[j + 1]].reshape(scales[j], scales[j])
                ys = np.nonzero(blk.any(axis=1))[0]
                out[k, j, c] = (ys.min(), ys.max())
    return out


@pytest.mark.parametrize("name", ["tiny_f32", "var_d16", "var_d30_kvstep", "var_d36_512"])
@pytest.mark.parametrize("waves", [4, 8, 16])
def test_mask_bit_exact(lv, name, waves):
    w = workloads.get(name)
    radii = oracle.expand_radii(w.scales, w.radius)
    plan = _plan(lv, w, waves)
    lv.litevar_plan_check(plan)
    mask, count = lv.litevar_mask_export_dense(plan)
    ref = oracle.mask_dense(w.scales, radii, w.n_sink, w.q_scales)
    assert (mask.cpu().numpy() == ref).all()
    assert int(count.item()) == int(ref.sum()) == plan.retained_pairs
    if waves == 4:
        win = lv.litevar_window_table_export(plan).cpu().numpy()
        assert (win == _window_table_from_oracle(w.scales, radii, w.n_sink)).all()


def test_tiny_mask_with_sinks(lv):
    w = workloads.get("tiny_f32")
    plan = _plan(lv, w, 4, n_sink=3)
    mask, count = lv.litevar_mask_export_dense(plan)
    ref = oracle.mask_dense(w.scales, [1] * 4, 3)
    assert (mask.cpu().numpy() == ref).all() and int(count.item()) == 471


def test_index_sets_2k(lv):
    w = workloads.get("var_2k_cfg")
    radii = oracle.expand_radii(w.scales, w.radius)
    plan = _plan(lv, w)
    lv.litevar_plan_check(plan)
    assert plan.retained_pairs == 20125483
    rowptr, cols = lv.litevar_mask_export_csr(plan)
    torch.cuda.synchronize()
    print("  csr exported; running the oracle's index sets", flush=True)
    rp_ref, cols_ref = oracle.index_sets(w.scales, radii, w.n_sink)
    assert (rowptr.cpu().numpy() == rp_ref).all()
    assert (cols.cpu().numpy() == cols_ref).all()


@pytest.mark.parametrize("waves", [4, 8, 16])
def test_csr_matches_dense_small(lv, waves):
    scales, radii = (1, 2, 3, 5, 7, 10), [0, 1, 2, 1, 3, 2]
    plan = lv.litevar_mask_build(scales, 0, radii, 1, None, waves_per_group=waves)
    rowptr, cols = lv.litevar_mask_export_csr(plan)
    rp_ref, cols_ref = oracle.index_sets(scales, radii, 1)
    assert (rowptr.cpu().numpy() == rp_ref).all() and (cols.cpu().numpy() == cols_ref).all()


MASK_CASES = [
    # scales, radius or per-key radii, n_sink, q_scales
    ((1,), 0, 0, None),
    ((1, 1, 1), 0, 0, None),
    ((3,), 1, 0, None),
    ((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), 0, 0, None),
    ((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), 1, 3, (4, 8)),
    ((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), [5, 0, 1, 0, 2, 1, 3, -1, 2, 1], 0, None),
    ((7, 2, 9, 4, 17), 1, 0, None),              # non-monotone sides
    ((16, 8, 4, 2, 1), 1, 1, None),              # fine to coarse
    ((1, 2, 3, 4, 6, 9, 13, 18, 24, 32), -1, 0, (8, 10)),   # dense block-causal
    ((5, 21, 33), 2, 0, None),
    ((2, 40), 7, 0, (1, 2)),
    ((1, 3, 70), 40, 0, (2, 3)),                 # window boxes wider than a wave (84 columns, clipped to 70)
    ((1, 3, 70), -1, 0, (2, 3)),                 # dense rows of 70 keys
    ((2, 100), [-1, 45], 0, (1, 2)),             # 94-column boxes inside a 100-column scale
]


@pytest.mark.parametrize("case", range(len(MASK_CASES)))
@pytest.mark.parametrize("waves", [4, 8, 16])
def test_mask_edge_cases(lv, case, waves):
    scales, rad, n_sink, q_scales = MASK_CASES[case]
    per = rad if isinstance(rad, list) else None
    radii = per if per is not None else [rad] * len(scales)
    plan = lv.litevar_mask_build(scales, 0 if per else rad, per, n_sink, q_scales,
                                 waves_per_group=waves)
    lv.litevar_plan_check(plan)
    mask, count = lv.litevar_mask_export_dense(plan)
    ref = oracle.mask_dense(scales, radii, n_sink, q_scales)
    assert (mask.cpu().numpy() == ref).all()
    assert int(count.item()) == int(ref.sum()) == plan.retained_pairs


# ---- attention outputs ----------------------------------------------------------------

def test_tiny_f32(lv):
    w = workloads.get("tiny_f32")
    q, k, v = workloads.make_workload_qkv(w)
    for n_sink in (0, 3):
        for waves in (4, 8, 16):
            plan = _plan(lv, w, waves, n_sink=n_sink)
            o = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
            ref = _oracle_attn(w.scales, [1] * 4, q, k, v, w.sm_scale, n_sink)
            assert _maxerr(o, ref) <= TOL["f32"]


def test_tiny_bf16_kernel_on_tiny_shape(lv):
    w = workloads.get("tiny_f32")
    q, k, v = workloads.make_qkv(w.scales, 1, 1, 64, "bf16", 0)
    for waves in (4, 8, 16):
        plan = _plan(lv, w, waves)
        o = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
        ref = _oracle_attn(w.scales, [1] * 4, q, k, v, w.sm_scale)
        assert _maxerr(o, ref) <= TOL["bf16"]


@pytest.mark.parametrize("waves", [4, 8, 16])
def test_var_d16(lv, waves):
    w = workloads.get("var_d16")
    q, k, v = workloads.make_workload_qkv(w)
    plan = _plan(lv, w, waves)
    o = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
    ref = _oracle_attn(w.scales, [w.radius] * 10, q, k, v, w.sm_scale)
    err = _maxerr(o, ref)
    print(f"  var_d16 waves={waves} max-abs err {err:.3e}", flush=True)
    assert err <= TOL["bf16"]
    # first token sees only itself: its output is V[..., 0, :] exactly, even in bf16
    assert torch.equal(o[:, :, 0].cpu(), v[:, :, 0])


@pytest.mark.parametrize("waves", [0, 4, 8, 16, (4, 64, 2, 1), (8, 64, 2, 1),
                                   (16, 0, 0, -1, 1), (16, 0, 0, -1, 2)])   # (.., patches per wave)
def test_var_d30_kv_step(lv, waves):
    w = workloads.get("var_d30_kvstep")
    q, k, v = workloads.make_workload_qkv(w)
    plan = _plan(lv, w, waves)
    o = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
    ref = _oracle_attn(w.scales, [w.radius] * 10, q, k, v, w.sm_scale, 0, w.q_scales)
    err = _maxerr(o, ref)
    print(f"  var_d30_kvstep waves={plan.waves_per_group} max-abs err {err:.3e}", flush=True)
    assert err <= TOL["bf16"]


def test_var_d36_windowed_and_dense(lv):
    w = workloads.get("var_d36_512")
    q, k, v = workloads.make_workload_qkv(w)
    plan = _plan(lv, w)
    o = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
    print("  running the fp64 oracle on all 288 (batch, head) pairs", flush=True)
    ref = _oracle_attn(w.scales, [w.radius] * 10, q, k, v, w.sm_scale)
    err = _maxerr(o, ref)
    print(f"  var_d36_512 windowed max-abs err {err:.3e}", flush=True)
    assert err <= TOL["bf16"]
    # dense block-causal path on the same inputs; the oracle checks 8 (batch, head) pairs
    dense = _plan(lv, w, radius=-1)
    od = _gpu_attn(lv, dense, q, k, v, w.sm_scale)
    refd = _oracle_attn(w.scales, [-1] * 10, q, k, v, w.sm_scale, bh_range=(140, 148))
    got = od.float().cpu().numpy().reshape(288, 2240, 64)[140:148]
    errd = float(np.abs(got - refd.reshape(288, 2240, 64)[140:148]).max())
    print(f"  var_d36_512 dense max-abs err {errd:.3e}", flush=True)
    assert errd <= TOL["bf16"]
    # the window changes the result (it is an approximation of dense attention)
    assert float((o.float() - od.float()).abs().max()) > 0.05


def test_var_2k_cfg_share(lv):
    w = workloads.get("var_2k_cfg")
    q, k, v = workloads.make_workload_qkv(w)
    share = workloads.make_cfg_share(w.heads, len(w.scales), w.seed)
    plan = _plan(lv, w)
    o = _gpu_attn(lv, plan, q, k, v, w.sm_scale, share=share)
    o_plain = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
    # sampled rows against the oracle: every scale's first/last rows plus random ones
    off = oracle.scale_offsets(w.scales)
    rng = np.random.default_rng(11)
    rows = sorted(set([off[i] for i in range(14)] + [off[i + 1] - 1 for i in range(14)] +
                      rng.integers(0, off[-1], size=160).tolist()))
    print(f"  oracle on {len(rows)} sampled query rows x 32 (batch, head)", flush=True)
    ref = _oracle_attn(w.scales, [w.radius] * 14, q, k, v, w.sm_scale, rows=rows)
    got = o_plain[:, :, rows].float().cpu().numpy()
    err = float(np.abs(got - ref).max())
    print(f"  var_2k max-abs err on sampled rows {err:.3e}", flush=True)
    assert err <= TOL["bf16"]
    # every query row of four heads, conditional and unconditional (8 of the 32 (batch, head)
    # pairs, 273 920 rows): every group, patch and phase of the 2K plan goes through the float
    # comparison, without sharing and, against the oracle's own cond -> uncond copy, with it
    heads = [0, 5, 10, 15]
    sub = [t[:, heads].contiguous() for t in (q, k, v)]
    print(f"  oracle on all {off[-1]} rows of heads {heads}, cond and uncond", flush=True)
    ref_full = _oracle_attn(w.scales, [w.radius] * 14, *sub, w.sm_scale)
    got_full = o_plain[:, heads].float().cpu().numpy()
    err_full = float(np.abs(got_full - ref_full).max())
    ref_shared = ref_full.copy()
    oracle.cfg_share(w.scales, ref_shared, share[heads].numpy())
    assert not np.array_equal(ref_shared, ref_full)
    err_shared = float(np.abs(o[:, heads].float().cpu().numpy() - ref_shared).max())
    print(f"  var_2k compared rows: {ref_full.shape[0] * ref_full.shape[1] * ref_full.shape[2]} "
          f"(all rows of 8 pairs); max-abs err {err_full:.3e} plain, {err_shared:.3e} shared", flush=True)
    assert err_full <= TOL["bf16"] and err_shared <= TOL["bf16"]
    # CFG sharing, checked everywhere: shared uncond rows equal their cond rows bit for
    # bit, every other row equals the flag-off run bit for bit
    o, o_plain = o.cpu(), o_plain.cpu()
    for h in range(w.heads):
        for kq in range(14):
            sl = slice(off[kq], off[kq + 1])
            if share[h, kq]:
                assert torch.equal(o[1, h, sl], o_plain[0, h, sl])
            else:
                assert torch.equal(o[1, h, sl], o_plain[1, h, sl])
    assert torch.equal(o[0], o_plain[0])


# ---- edge cases and invariants on the float path ------------------------------------------

def _rand_case(scales, B, H, dtype, seed, q_scales=None, scale=1.0):
    return workloads.make_qkv(scales, B, H, 64, dtype, seed, scale, q_scales)


ATTN_CASES = [
    ((1,), 0, 0, None, 2, 3),
    ((1, 2, 3, 5, 7, 10), [0, 1, 2, 1, 3, 2], 1, None, 2, 2),
    ((7, 2, 9, 4, 17), 1, 0, None, 1, 5),
    ((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), 1, 3, (4, 8), 3, 2),
    ((1, 2, 3, 4, 6, 9, 13, 18, 24, 32), 0, 0, None, 1, 2),
    ((2, 40), 7, 0, (1, 2), 2, 1),
    ((5, 21, 33), 2, 0, None, 1, 3),
    ((1, 3, 70), 40, 0, (2, 3), 1, 1),           # window boxes wider than a wave
    # dense key lists of 55, 91, 128, 140, 192, 204 and 285 keys: one to five 64-key chunks,
    # with and without a ragged last chunk (the 16-patch kernel's first phase is one chunk,
    # the others two)
    ((1, 2, 3, 4, 5), -1, 0, (4, 5), 1, 2),
    ((1, 2, 3, 4, 5, 6), -1, 0, (5, 6), 1, 2),
    ((8, 8), -1, 0, (1, 2), 1, 2),
    ((1, 2, 3, 4, 5, 6, 7), -1, 0, (6, 7), 1, 2),
    ((8, 8, 8), -1, 0, (2, 3), 1, 1),
    ((1, 2, 3, 4, 5, 6, 7, 8), -1, 0, (7, 8), 1, 1),
    ((1, 2, 3, 4, 5, 6, 7, 8, 9), -1, 0, (8, 9), 1, 1),
]


@pytest.mark.parametrize("case", range(len(ATTN_CASES)))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("waves", [4, 8, (16, 0, 0, -1, 1), (16, 0, 0, -1, 2)])   # 16 patches: one and two per wave
def test_attn_edge_cases(lv, case, dtype, waves):
    scales, rad, n_sink, q_scales, B, H = ATTN_CASES[case]
    per = rad if isinstance(rad, list) else None
    radii = per if per is not None else [rad] * len(scales)
    q, k, v = _rand_case(scales, B, H, dtype, 100 + case, q_scales)
    plan = lv.litevar_mask_build(scales, 0 if per else rad, per, n_sink, q_scales,
                                 waves_per_group=waves)
    o = _gpu_attn(lv, plan, q, k, v, 0.125)
    ref = _oracle_attn(scales, radii, q, k, v, 0.125, n_sink, q_scales)
    assert _maxerr(o, ref) <= TOL[dtype]


def test_constant_values_give_constant_output(lv):
    # softmax rows sum to 1: with V == 1 every output element is exactly 1 (in f32: ~1)
    w = workloads.get("var_d16")
    q, k, v = workloads.make_workload_qkv(w)
    plan = _plan(lv, w)
    o = _gpu_attn(lv, plan, q, k, torch.ones_like(v), w.sm_scale)
    assert float((o.float() - 1).abs().max()) <= 2 ** -8


def test_zero_queries_average_values(lv):
    scales, radii = (1, 2, 3, 5, 7, 10), [0, 1, 2, 1, 3, 2]
    q, k, v = _rand_case(scales, 1, 2, "f32", 5)
    plan = lv.litevar_mask_build(scales, 0, radii)
    o = _gpu_attn(lv, plan, torch.zeros_like(q), k, v, 0.125).cpu().double().numpy()
    rowptr, cols = oracle.index_sets(scales, radii, 0)
    vv = v.double().numpy()
    for ql in range(o.shape[2]):
        idx = cols[rowptr[ql]:rowptr[ql + 1]]
        assert np.abs(o[:, :, ql] - vv[:, :, idx].mean(axis=2)).max() <= 1e-5


def test_kv_cache_step_equals_tail_of_full_call(lv):
    w = workloads.get("var_d16")
    q, k, v = workloads.make_workload_qkv(w)
    full = _gpu_attn(lv, _plan(lv, w, 8), q, k, v, w.sm_scale)
    step = _gpu_attn(lv, _plan(lv, w, 8, q_scales=(9, 10)), q[:, :, 424:].contiguous(), k, v, w.sm_scale)
    assert torch.equal(full[:, :, 424:], step)


def test_strided_inputs_and_outputs(lv):
    # [B, L, H, D] storage viewed as [B, H, L, D]: token stride H*D, head stride D
    scales, B, H = (1, 2, 3, 5, 7, 10), 2, 3
    q, k, v = _rand_case(scales, B, H, "bf16", 9)
    plan = lv.litevar_mask_build(scales, 1)
    ref = _gpu_attn(lv, plan, q, k, v, 0.125)

    def blhd(t):
        return t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)
    qs, ks, vs = blhd(q), blhd(k), blhd(v)
    out = torch.zeros_like(qs.permute(0, 2, 1, 3).contiguous()).permute(0, 2, 1, 3)
    assert not qs.is_contiguous() and not out.is_contiguous()
    lv.litevar_windowed_attn_fwd(plan, qs, ks, vs, 0.125, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out.contiguous(), ref)


def test_cfg_share_small_f32_and_bf16(lv):
    scales = (1, 2, 3, 5, 7, 10)
    for dtype in ("f32", "bf16"):
        q, k, v = _rand_case(scales, 4, 3, dtype, 21)
        share = workloads.make_cfg_share(3, len(scales), 5)
        plan = lv.litevar_mask_build(scales, 1)
        o = _gpu_attn(lv, plan, q, k, v, 0.125, share=share)
        ref = _oracle_attn(scales, [1] * 6, q, k, v, 0.125, share=share)
        assert _maxerr(o, ref) <= TOL[dtype]
        # KV-cache step with sharing: the table is indexed by the query scale
        plan2 = lv.litevar_mask_build(scales, 1, q_scales=(4, 6))
        q2 = q[:, :, 39:].contiguous()
        o2 = _gpu_attn(lv, plan2, q2, k, v, 0.125, share=share)
        ref2 = _oracle_attn(scales, [1] * 6, q2, k, v, 0.125, q_scales=(4, 6), share=share)
        assert _maxerr(o2, ref2) <= TOL[dtype]


def test_repeat_launch_is_deterministic(lv):
    w = workloads.get("var_d30_kvstep")
    q, k, v = workloads.make_workload_qkv(w)
    plan = _plan(lv, w)
    a = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
    b = _gpu_attn(lv, plan, q, k, v, w.sm_scale)
    assert torch.equal(a, b)


# ---- one radius per (query scale, part) (Section 2, step (3)) ------------------------

PAIR_CASES = [
    ((1, 2, 3, 4), 0, None),
    ((1, 2, 3, 5, 7, 10), 1, None),
    ((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), 3, None),
    ((1, 2, 3, 4, 5, 6, 8, 10, 13, 16), 0, (9, 10)),     # the KV-cache step
    ((7, 2, 9, 4, 17), 0, (2, 5)),
]


@pytest.mark.parametrize("case", range(len(PAIR_CASES)))
@pytest.mark.parametrize("waves", [4, 8, 16])
def test_pair_radius_tables(lv, case, waves):
    """masks bit-exact and attention within tolerance when every (query scale, key scale)
    part has its own radius (some of them dense)"""
    scales, n_sink, q_scales = PAIR_CASES[case]
    K = len(scales)
    rng = np.random.default_rng(500 + case)
    tab = rng.integers(-1, 5, size=(K, K)).tolist()
    print(f"  pair radii: scales={scales} waves={waves} q_scales={q_scales}", flush=True)
    plan = lv.litevar_mask_build(scales, 0, tab, n_sink, q_scales, waves_per_group=waves)
    lv.litevar_plan_check(plan)
    mask, _ = lv.litevar_mask_export_dense(plan)
    want = oracle.mask_dense(scales, tab, n_sink, q_scales)
    assert np.array_equal(mask.cpu().numpy(), want)
    assert plan.retained_pairs == int(want.sum())
    for dtype in ("bf16", "f32"):
        q, k, v = _rand_case(scales, 1, 2, dtype, 900 + case, q_scales)
        o = _gpu_attn(lv, plan, q, k, v, 0.125)
        ref = _oracle_attn(scales, tab, q, k, v, 0.125, n_sink, q_scales)
        assert _maxerr(o, ref) <= TOL[dtype]


def test_calibrated_table_feeds_the_plan(lv):
    """calibration -> radius table of one head -> plan: the plan's mask is the oracle's mask
    of that table"""
    scales = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    p = workloads.make_attn_map(scales, 1, 2, 19).cuda()
    rad = lv.litevar_window_calibrate(scales, p, 0.9).cpu().numpy()
    tab = np.maximum(rad[1], 0).tolist()          # head 1; the unused upper triangle as radius 0
    plan = lv.litevar_mask_build(scales, 0, tab, 3)
    mask, _ = lv.litevar_mask_export_dense(plan)
    assert np.array_equal(mask.cpu().numpy(), oracle.mask_dense(scales, tab, 3))


def test_random_configurations_sweep(lv):
    """forty-eight seeded random problems (scale lists in any order, per-part radii with dense
    parts, dense leading scales, query-scale ranges, all three kernels): masks bit-exact,
    index sets through the CSR export, attention within tolerance"""
    rng = np.random.default_rng(20241127)
    for it in range(48):
        K = int(rng.integers(1, 7))
        scales = [int(x) for x in rng.integers(1, 20, size=K)]
        if it % 4 == 0:
            scales = sorted(scales)
        tab = rng.integers(-1, 6, size=(K, K)).tolist()
        radii = tab if it % 2 else [int(x) for x in rng.integers(-1, 6, size=K)]
        n_sink = int(rng.integers(0, K + 1)) if it % 3 == 0 else 0
        qb = int(rng.integers(0, K))
        q_scales = (qb, int(rng.integers(qb + 1, K + 1))) if it % 5 else None
        waves = (4, 8, (16, 0, 0, -1, 1), (16, 0, 0, -1, 2))[it % 4]
        dtype = "bf16" if it % 2 == 0 else "f32"
        print(f"  sweep {it}: scales={scales} radii={radii} n_sink={n_sink} q_scales={q_scales} "
              f"waves={waves} {dtype}", flush=True)
        plan = lv.litevar_mask_build(scales, 0, radii, n_sink, q_scales, waves_per_group=waves)
        lv.litevar_plan_check(plan)
        want = oracle.mask_dense(scales, radii, n_sink, q_scales)
        mask, _ = lv.litevar_mask_export_dense(plan)
        assert np.array_equal(mask.cpu().numpy(), want), it
        rowptr, cols = lv.litevar_mask_export_csr(plan)
        rp = rowptr.cpu().numpy()
        assert np.array_equal(np.diff(rp), want.sum(axis=1)), it
        assert np.array_equal(cols.cpu().numpy(), np.nonzero(want)[1]), it
        q, k, v = _rand_case(scales, 1, 2, dtype, 3000 + it, q_scales)
        o = _gpu_attn(lv, plan, q, k, v, 0.125)
        ref = _oracle_attn(scales, radii, q, k, v, 0.125, n_sink, q_scales)
        assert _maxerr(o, ref) <= TOL[dtype], it


# ---- failure handling: every kernel exits normally ----------------------------------------

@pytest.mark.parametrize("waves", [4, 8, 16])
def test_zeroed_plan_makes_the_launch_a_no_op(lv, waves):
    """a blob without the header's magic (zeroed, stale, half-built) is not walked: the
    attention kernels return at once, the output is untouched, litevar_plan_check says so"""
    w = workloads.get("var_d16")
    for dtype in ("bf16", "f32"):
        q, k, v = workloads.make_qkv(w.scales, 1, 2, 64, dtype, 3)
        plan = _plan(lv, w, waves)
        torch.cuda.synchronize()
        plan.blob.zero_()
        out = torch.full(q.shape, 7.0, dtype=q.dtype, device="cuda")
        print(f"  zeroed plan: waves={waves} {dtype}", flush=True)
        lv.litevar_windowed_attn_fwd(plan, q.cuda(), k.cuda(), v.cuda(), w.sm_scale, out=out)
        torch.cuda.synchronize()
        assert bool((out == 7.0).all())
        with pytest.raises(lv.LitevarError) as e:
            lv.litevar_plan_check(plan)
        assert e.value.status == -5


@pytest.mark.parametrize("waves", [4, 8])
def test_bounded_wait_gives_up_and_reports(lv, waves):
    """with a spin limit of one poll the compute waves' first wait for the loader runs out:
    the launch still ends (every wave exits normally), the plan's header carries the mark
    and litevar_plan_check reports it; a plan with the default limit is unaffected"""
    w = workloads.get("var_d16")
    q, k, v = workloads.make_qkv(w.scales, 1, 2, 64, "bf16", 3)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    good = _plan(lv, w, waves)
    want = lv.litevar_windowed_attn_fwd(good, qd, kd, vd, w.sm_scale)
    tiny = lv.litevar_mask_build(w.scales, w.radius, None, w.n_sink, w.q_scales,
                                 waves_per_group=waves, spin_limit=1)
    lv.litevar_plan_check(tiny)
    print(f"  spin limit 1: waves={waves}", flush=True)
    lv.litevar_windowed_attn_fwd(tiny, qd, kd, vd, w.sm_scale)
    torch.cuda.synchronize()
    with pytest.raises(lv.LitevarError) as e:
        lv.litevar_plan_check(tiny)
    assert e.value.status == -5 and "gave up" in str(e.value)
    lv.litevar_plan_check(good)
    again = lv.litevar_windowed_attn_fwd(good, qd, kd, vd, w.sm_scale)
    torch.cuda.synchronize()
    assert torch.equal(want, again)


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("qk_scale", [3.0, 6.0])
def test_peaked_attention_keeps_the_tolerance(lv, waves, qk_scale):
    """Scores of some tens (Q and K drawn wide, V unit): a few keys carry each row.  The
    softmax scale must be applied in fp32: folding it into Q with a second bf16 rounding of
    Q passes the N(0,1) workloads and fails here by a factor of three to ten."""
    scales = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    g = torch.Generator(device="cpu").manual_seed(7)
    L = sum(s * s for s in scales)
    q = (torch.randn(2, 4, L, 64, generator=g) * qk_scale).to(torch.bfloat16)
    k = (torch.randn(2, 4, L, 64, generator=g) * qk_scale).to(torch.bfloat16)
    v = torch.randn(2, 4, L, 64, generator=g).to(torch.bfloat16)
    ref = _oracle_attn(scales, oracle.expand_radii(scales, 3), q, k, v, 0.125)
    plan = lv.litevar_mask_build(scales, 3, waves_per_group=waves)
    err = _maxerr(_gpu_attn(lv, plan, q, k, v, 0.125), ref)
    print(f"  peaked x{qk_scale} waves={waves}: max-abs err {err:.3e}")
    assert err <= TOL["bf16"]
