"""Band mask mode (paper Section 2, step (2), literal) and one radius table per head inside
one plan (step (3)) through the C ABI against the oracle: masks and index sets bit-exact per
head, attention within the bf16 / fp32 tolerances, one launch for all heads."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}
BAND = 1
VAR = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
WAVES = [4, 8, (16, 0, 0, -1, 1), (16, 0, 0, -1, 2)]


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    m.load_library()
    return m


def _attn(lv, plan, q, k, v):
    o = lv.litevar_windowed_attn_fwd(plan, q.cuda(), k.cuda(), v.cuda(), 0.125)
    torch.cuda.synchronize()
    return o.float().cpu().numpy().astype(np.float64)


BAND_CASES = [
    # scales, radius or per-key-scale radii, n_sink, q_scales
    ((1, 2, 3, 4), 1, 0, None),
    ((1, 2, 3, 4), 1, 3, None),
    ((1,), 0, 0, None),
    ((1, 2), 0, 0, None),
    (VAR, 2, 0, None),
    (VAR, 24, 0, (9, 10)),
    (VAR, [0, 1, 2, 3, 5, 8, -1, 13, 40, 100], 3, None),
    (VAR, 700, 0, None),                       # every part fully covered: dense block-causal
    ((7, 2, 9, 4, 17), 6, 0, None),            # sides in any order: parts wider than the query scale
    ((3, 20), 9, 0, (1, 2)),
    ((1, 2, 3, 4, 6, 9, 13, 18, 24, 32), 30, 0, (8, 10)),
]


@pytest.mark.parametrize("case", range(len(BAND_CASES)))
@pytest.mark.parametrize("waves", [4, 8, 16])
def test_band_masks_bit_exact(lv, case, waves):
    scales, rad, n_sink, q_scales = BAND_CASES[case]
    per = rad if isinstance(rad, list) else None
    radii = per if per is not None else [rad] * len(scales)
    print(f"  band mask: scales={scales} rad={rad} n_sink={n_sink} q_scales={q_scales} waves={waves}", flush=True)
    plan = lv.litevar_mask_build(scales, 0 if per else rad, per, n_sink, q_scales, waves_per_group=waves,
                                 mask_mode=BAND)
    lv.litevar_plan_check(plan)
    want = oracle.mask_dense(scales, radii, n_sink, q_scales, mode=BAND)
    mask, count = lv.litevar_mask_export_dense(plan)
    assert np.array_equal(mask.cpu().numpy(), want)
    assert int(count.item()) == int(want.sum()) == plan.retained_pairs
    rowptr, cols = lv.litevar_mask_export_csr(plan)
    rp, cc = oracle.index_sets(scales, radii, n_sink, q_scales, mode=BAND)
    assert np.array_equal(rowptr.cpu().numpy(), rp) and np.array_equal(cols.cpu().numpy(), cc)


@pytest.mark.parametrize("case", range(len(BAND_CASES)))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_band_attention(lv, case, dtype):
    scales, rad, n_sink, q_scales = BAND_CASES[case]
    per = rad if isinstance(rad, list) else None
    radii = per if per is not None else [rad] * len(scales)
    q, k, v = workloads.make_qkv(scales, 1, 2, 64, dtype, 700 + case, 1.0, q_scales)
    arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
    ref = oracle.attn(scales, radii, *arrs, 0.125, n_sink, q_scales, mode=BAND)
    for waves in WAVES:
        print(f"  band attn: case {case} {dtype} waves={waves}", flush=True)
        plan = lv.litevar_mask_build(scales, 0 if per else rad, per, n_sink, q_scales, waves_per_group=waves,
                                     mask_mode=BAND)
        assert np.abs(_attn(lv, plan, q, k, v) - ref).max() <= TOL[dtype]


def test_band_plan_has_no_window_table(lv):
    plan = lv.litevar_mask_build((1, 2, 3, 4), 1, mask_mode=BAND)
    with pytest.raises(lv.LitevarError) as e:
        lv.litevar_window_table_export(plan)
    assert e.value.status == -2


# ---- one radius table per head ---------------------------------------------------------------

def _head_tables(scales, H, seed, distinct):
    g = np.random.default_rng(seed)
    K = len(scales)
    base = g.integers(-1, 6, size=(distinct, K, K))
    return base[g.integers(0, distinct, size=H)] if distinct < H else base[:H]


@pytest.mark.parametrize("mode", [0, BAND])
@pytest.mark.parametrize("waves", [4, 8, 16])
def test_per_head_masks_bit_exact(lv, mode, waves):
    scales, H = VAR, 7
    tabs = _head_tables(scales, H, 11 + mode, 4)          # seven heads, at most four distinct tables
    print(f"  per-head masks: mode={mode} waves={waves}", flush=True)
    plan = lv.litevar_mask_build(scales, 0, tabs.tolist(), 1, None, waves_per_group=waves, mask_mode=mode)
    lv.litevar_plan_check(plan)
    assert plan.n_heads == H and plan.n_head_groups == len({t.tobytes() for t in np.where(
        np.triu(np.ones((10, 10), dtype=bool), 1), 0, np.minimum(tabs, 32767))})
    total = 0
    for h in range(H):
        want = oracle.mask_dense(scales, tabs[h], 1, mode=mode)
        mask, count = lv.litevar_mask_export_dense(plan, head=h)
        assert np.array_equal(mask.cpu().numpy(), want), h
        assert int(count.item()) == int(want.sum())
        rowptr, cols = lv.litevar_mask_export_csr(plan, head=h)
        rp, cc = oracle.index_sets(scales, tabs[h], 1, mode=mode)
        assert np.array_equal(rowptr.cpu().numpy(), rp) and np.array_equal(cols.cpu().numpy(), cc)
        if mode == 0:
            g0 = lv.litevar_mask_build(scales, 0, tabs[h].tolist(), 1, None, waves_per_group=waves)
            assert torch.equal(lv.litevar_window_table_export(plan, head=h), lv.litevar_window_table_export(g0))
    for hg in range(plan.n_head_groups):
        total += int(plan.retained_pairs_of_group[hg])
    assert total == plan.retained_pairs


@pytest.mark.parametrize("mode", [0, BAND])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_per_head_attention_in_one_launch(lv, mode, dtype):
    for scales, q_scales, H in ((VAR, None, 5), (VAR, (9, 10), 6), ((7, 2, 9, 4, 17), (2, 5), 3)):
        tabs = _head_tables(scales, H, 23 + mode, H)
        q, k, v = workloads.make_qkv(scales, 2, H, 64, dtype, 60 + H, 1.0, q_scales)
        arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
        ref = oracle.attn(scales, tabs, *arrs, 0.125, 0, q_scales, mode=mode)
        for waves in WAVES:
            print(f"  per-head attn: scales={scales} q_scales={q_scales} H={H} mode={mode} {dtype} waves={waves}", flush=True)
            plan = lv.litevar_mask_build(scales, 0, tabs.tolist(), 0, q_scales, waves_per_group=waves, mask_mode=mode)
            assert np.abs(_attn(lv, plan, q, k, v) - ref).max() <= TOL[dtype]
        # the head count of the call must be the plan's
        with pytest.raises(lv.LitevarError):
            lv.litevar_windowed_attn_fwd(plan, q[:, :H - 1].contiguous().cuda(), k[:, :H - 1].contiguous().cuda(),
                                         v[:, :H - 1].contiguous().cuda(), 0.125)


def test_calibrated_radii_of_thirty_heads_feed_one_plan(lv):
    """litevar_window_calibrate's [H][K][K] output goes straight into litevar_mask_build; one
    attention launch then serves the thirty heads, each with its own windows"""
    H = 30
    p = workloads.make_attn_map(VAR, 1, H, 5).cuda()
    rad = lv.litevar_window_calibrate(VAR, p, 0.9)
    torch.cuda.synchronize()
    tabs = rad.cpu().numpy()
    plan = lv.litevar_mask_build(VAR, 0, np.maximum(tabs, 0).tolist(), 3, (9, 10))
    assert plan.n_heads == H and 1 < plan.n_head_groups <= H
    for h in (0, 13, 29):
        mask, _ = lv.litevar_mask_export_dense(plan, head=h)
        assert np.array_equal(mask.cpu().numpy(), oracle.mask_dense(VAR, np.maximum(tabs[h], 0), 3, (9, 10)))
    q, k, v = workloads.make_qkv(VAR, 2, H, 64, "bf16", 77, 1.0, (9, 10))
    arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
    ref = oracle.attn(VAR, np.maximum(tabs, 0), *arrs, 0.125, 3, (9, 10))
    share = workloads.make_cfg_share(H, 10, 3)
    o = lv.litevar_windowed_attn_fwd(plan, q.cuda(), k.cuda(), v.cuda(), 0.125)
    torch.cuda.synchronize()
    assert np.abs(o.float().cpu().numpy() - ref).max() <= TOL["bf16"]
    o2 = lv.litevar_windowed_attn_fwd(plan, q.cuda(), k.cuda(), v.cuda(), 0.125, cfg_share=share.cuda())
    torch.cuda.synchronize()
    oracle.cfg_share(VAR, ref, share.numpy(), (9, 10))
    assert np.abs(o2.float().cpu().numpy() - ref).max() <= TOL["bf16"]
