"""The bounds-checking build of the library (-DLITEVAR_DEBUG_BOUNDS): every token, query row and
LDS offset that an attention kernel takes from the plan is compared with its limit before use.
On the product's own plans it must find nothing and change nothing; a planted bad LDS offset
(harmless: the offset stays inside the workgroup's LDS) must be reported, with every kernel
exiting normally."""
import os

import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu

SEC_STEP_ADDR = 8      # index of the step-descriptor section in litevar_plan.off


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    m.load_library()
    return m


@pytest.fixture(scope="module")
def debug_lib():
    from paper_2411_17178_amd import build
    if not os.path.exists(build.LIB_DEBUG_BOUNDS):
        pytest.skip("the bounds-checking library is not built (python -m paper_2411_17178_amd.build --debug-bounds)")
    return build.LIB_DEBUG_BOUNDS


CASES = [("tiny_f32", "f32", 0, None), ("var_d16", "bf16", 4, None), ("var_d16", "bf16", 8, None),
         ("var_d16", "bf16", 16, None), ("var_d30_kvstep", "bf16", 16, (9, 10)), ("var_d30_kvstep", "bf16", 4, (9, 10))]


@pytest.mark.parametrize("name,dtype,waves,q_scales", CASES)
def test_checked_build_finds_nothing_and_changes_nothing(lv, debug_lib, name, dtype, waves, q_scales):
    w = workloads.get(name)
    q, k, v = workloads.make_qkv(w.scales, 2, 2, 64, dtype, 5, w.input_scale, q_scales)
    share = workloads.make_cfg_share(2, len(w.scales), 9).cuda()
    plan = lv.litevar_mask_build(w.scales, w.radius, None, 0, q_scales, waves_per_group=waves)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    print(f"  checked build: {name} {dtype} waves={plan.waves_per_group}", flush=True)
    want = lv.litevar_windowed_attn_fwd(plan, qd, kd, vd, 0.125, cfg_share=share)
    with lv.use_library(debug_lib):
        got = lv.litevar_windowed_attn_fwd(plan, qd, kd, vd, 0.125, cfg_share=share)
        torch.cuda.synchronize()
        lv.litevar_plan_check(plan)                      # no out-of-range mark
    assert torch.equal(got, want)


def test_checked_build_on_8_bit_operands(lv, debug_lib):
    w = workloads.get("var_d30_kvstep")
    q, k, v = workloads.make_qkv(w.scales, 2, 3, 64, "bf16", 6, 1.0, w.q_scales)
    plan = lv.litevar_mask_build(w.scales, w.radius, None, 0, w.q_scales, waves_per_group=16)
    ops = []
    for t in (q, k, v):
        ops += list(lv.litevar_qkv8_quantize(t.cuda()))
    want = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125)
    with lv.use_library(debug_lib):
        got = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125)
        torch.cuda.synchronize()
        lv.litevar_plan_check(plan)
    assert torch.equal(got, want)


@pytest.mark.parametrize("waves", [16, 4])
def test_checked_build_reports_a_bad_lds_offset(lv, debug_lib, waves):
    """One K offset of the first step descriptor is set beyond the K ring (but inside the
    workgroup's LDS, so that even an unchecked read would be harmless): the checked kernels
    replace it by 0, finish, and mark the plan."""
    scales = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    q, k, v = workloads.make_qkv(scales, 1, 2, 64, "bf16", 7)
    plan = lv.litevar_mask_build(scales, 2, waves_per_group=waves)
    ring_bytes = plan.ring_chunks * plan.chunk_keys * 128
    words = plan.blob[int(plan.off[SEC_STEP_ADDR]):].view(torch.int32)
    bad = ring_bytes + 0x100
    assert bad < 0xffff and bad + 16 <= 2 * ring_bytes
    torch.cuda.synchronize()
    words[0] = (int(words[0].item()) & ~0xffff) | bad     # lane 0 of step 0: first K row offset
    torch.cuda.synchronize()
    with lv.use_library(debug_lib):
        print(f"  planted LDS offset {bad} >= {ring_bytes}, waves={plan.waves_per_group}", flush=True)
        lv.litevar_windowed_attn_fwd(plan, q.cuda(), k.cuda(), v.cuda(), 0.125)
        torch.cuda.synchronize()
        with pytest.raises(lv.LitevarError, match="out of range"):
            lv.litevar_plan_check(plan)
