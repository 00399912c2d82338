"""QKV8 (paper Section 4) through the C ABI against the oracle: the quantiser's codes and
parameters bit for bit (integer work decided in binary32 on both sides), the dequantised
values exactly, the attention output within the tolerance derived below.

Tolerance of the attention output: the library dequantises the 8-bit operands once and rounds
them to bf16 for its bf16 MFMA kernels.  On top of the bf16 path's own bound (2e-2: P and O
rounded to bf16, fp32 accumulation) that rounding moves every operand by at most 2^-9
relative; through V this moves an output by at most 2^-9 max|v| (a convex combination of
rows, each off by that much), through Q and K it perturbs a score by at most about
2 * 2^-9 * sm_scale * |q||k|, well below the first term for the N(0,1) workloads.  With
|v| <= 5: 2e-2 + 1e-2 = 3e-2."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu
TOL_QKV8 = 3e-2


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    m.load_library()
    return m


def _special_rows():
    rows = [[5.0] * 64, [0.0] * 64, [-3.25] * 64]                      # constant rows: s = 0
    rows.append([-127.0, -126.5, 0.0, 63.5, 127.0] + [1.0] * 59)      # ties at s = 1
    rows.append([-1.0, 0.0, 0.5, 3.0] + [1.0] * 60)                   # the hand-derived row
    rows.append([10.0, 10.25] * 32)
    rows.append(list(np.linspace(-1e-3, 1e-3, 64)))
    rows.append(list(np.linspace(-300, 900, 64)))
    return np.array(rows, dtype=np.float32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_quantiser_codes_and_parameters_bit_exact(lv, dtype):
    g = np.random.default_rng(17)
    x = np.concatenate([_special_rows(), g.standard_normal((4099, 64)).astype(np.float32) * 2,
                        (g.standard_normal((64, 64)) * 1e-4 + 7).astype(np.float32)])
    t = torch.from_numpy(x)
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    print(f"  quantise {tuple(t.shape)} {dtype}", flush=True)
    codes, sz = lv.litevar_qkv8_quantize(t.cuda())
    torch.cuda.synchronize()
    want_c, want_s, want_z = oracle.quantize_rows(workloads.to_oracle_array(t))
    assert np.array_equal(codes.cpu().numpy().astype(np.int32), want_c)
    sz = sz.cpu().numpy().astype(np.float64)
    assert np.array_equal(sz[:, 0], want_s) and np.array_equal(sz[:, 1], want_z)
    # dequantised values: bf16(fma(s, code, z)) against the oracle's fp64 s*code + z rounded
    # to binary32 and then to bf16
    back = lv.litevar_qkv8_dequantize(codes, torch.from_numpy(sz.astype(np.float32)).cuda())
    torch.cuda.synchronize()
    want = torch.from_numpy(oracle.dequantize_rows(want_c, want_s, want_z).astype(np.float32)).to(torch.bfloat16)
    assert torch.equal(back.cpu(), want)


def _qkv8_case(lv, scales, radius, n_sink, q_scales, B, H, seed, input_scale=1.0, waves=0, share=None,
               src_dtype="bf16"):
    q, k, v = workloads.make_qkv(scales, B, H, 64, src_dtype, seed, input_scale, q_scales)
    plan = lv.litevar_mask_build(scales, radius, None, n_sink, q_scales, waves_per_group=waves)
    ops = []
    for t in (q, k, v):
        ops += list(lv.litevar_qkv8_quantize(t.cuda()))
    print(f"  qkv8 attn: scales={scales} B={B} H={H} waves={plan.waves_per_group}", flush=True)
    o = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125, cfg_share=share.cuda() if share is not None else None)
    torch.cuda.synchronize()
    arrs = [workloads.to_oracle_array(t) for t in (q, k, v)]
    ref = oracle.attn_qkv8(scales, [radius] * len(scales), *arrs, 0.125, n_sink, q_scales)
    if share is not None:
        oracle.cfg_share(scales, ref, share.numpy(), q_scales)
    return float(np.abs(o.float().cpu().numpy() - ref).max())


def test_qkv8_tiny_and_edge_shapes(lv):
    for scales, radius, n_sink, q_scales in [((1, 2, 3, 4), 1, 0, None), ((1,), 0, 0, None),
                                             ((7, 2, 9, 4, 17), 1, 0, None), ((2, 40), 7, 0, (1, 2)),
                                             ((1, 2, 3, 4, 5, 6, 7, 8, 9), -1, 0, (8, 9))]:
        for waves in (4, 16):
            assert _qkv8_case(lv, scales, radius, n_sink, q_scales, 2, 2, 40, waves=waves) <= TOL_QKV8
    assert _qkv8_case(lv, (1, 2, 3, 4), 1, 0, None, 2, 2, 41, src_dtype="f32") <= TOL_QKV8


def test_qkv8_var_d16_with_sharing(lv):
    w = workloads.get("var_d16")
    share = workloads.make_cfg_share(w.heads, len(w.scales), w.seed)
    err = _qkv8_case(lv, w.scales, w.radius, 0, None, w.batch, w.heads, w.seed, w.input_scale, share=share)
    print(f"  qkv8 var_d16 max-abs err {err:.3e}", flush=True)
    assert err <= TOL_QKV8


def test_qkv8_var_d30_kv_step(lv):
    w = workloads.get("var_d30_kvstep")
    err = _qkv8_case(lv, w.scales, w.radius, 0, w.q_scales, w.batch, w.heads, w.seed)
    print(f"  qkv8 var_d30_kvstep (all 480 pairs) max-abs err {err:.3e}", flush=True)
    assert err <= TOL_QKV8


def test_qkv8_var_d36_subset(lv):
    w = workloads.get("var_d36_512")
    err = _qkv8_case(lv, w.scales, w.radius, 0, None, 1, 6, w.seed)     # six (batch, head) pairs of the shape
    print(f"  qkv8 var_d36_512 (6 pairs) max-abs err {err:.3e}", flush=True)
    assert err <= TOL_QKV8


def test_qkv8_constant_value_rows_pass_through(lv):
    """V rows that are constant dequantise exactly: with one constant per key every output
    row is a constant between the values it can see, and the first token returns V[0]"""
    scales = (1, 2, 3, 5)
    q, k, _ = workloads.make_qkv(scales, 1, 2, 64, "bf16", 3)
    L = 39
    v = (torch.arange(1, L + 1, dtype=torch.float32)[None, None, :, None] * 0.5).expand(1, 2, L, 64).contiguous()
    plan = lv.litevar_mask_build(scales, -1)
    ops = []
    for t in (q, k, v.to(torch.bfloat16)):
        ops += list(lv.litevar_qkv8_quantize(t.cuda()))
    o = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125).float().cpu()
    assert bool((o[:, :, 0] == 0.5).all())
    assert float((o - o[..., :1]).abs().max()) <= 2 ** -6


@pytest.mark.parametrize("ppw", [1, 2])
@pytest.mark.parametrize("case", ["full", "kv_step", "cfg", "kv_step_cfg"])
def test_qkv8_in_kernel_conversion_equals_bf16_kernel_on_dequantised_copy(lv, ppw, case):
    """Plans with 16 patches per group can take the 8-bit operands straight into the attention
    kernel, which converts them on their way into LDS.  What it puts there is what
    litevar_qkv8_dequantize writes, so the output must equal, bit for bit, that of the bf16
    kernel on such a copy (same plan, both wave layouts), sharing included.  The library
    takes that route by itself while the groups stream few rows twice (no workspace then);
    the flag asks for it whatever the shape."""
    scales = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    q_scales = (9, 10) if case.startswith("kv_step") else None
    B, H = 4, 3
    q, k, v = workloads.make_qkv(scales, B, H, 64, "bf16", 11, 1.0, q_scales)
    share = workloads.make_cfg_share(H, len(scales), 5).cuda() if case.endswith("cfg") else None
    plan = lv.litevar_mask_build(scales, 3, None, 0, q_scales, waves_per_group=(16, 0, 0, -1, ppw))
    assert plan.waves_per_group == 16
    # (the documented rule: in the kernel while the groups stream at most 1.25 (q_len + 2 kv_len) rows)
    by_itself = 4 * plan.n_union_keys <= 5 * (plan.q_len + 2 * plan.kv_len)
    assert by_itself                             # holds for this short sequence, full or KV step
    assert (lv.litevar_windowed_attn_qkv8_workspace_bytes(plan, B, H) == 0) == by_itself
    ops = []
    for t in (q, k, v):
        ops += list(lv.litevar_qkv8_quantize(t.cuda()))
    print(f"  in-kernel qkv8 vs bf16 on copy: case={case} patches per wave={ppw}", flush=True)
    forced = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125, cfg_share=share, in_kernel=True)
    default = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125, cfg_share=share)
    copies = [lv.litevar_qkv8_dequantize(ops[i], ops[i + 1]) for i in (0, 2, 4)]
    plain = lv.litevar_windowed_attn_fwd(plan, *copies, 0.125, cfg_share=share)
    torch.cuda.synchronize()
    assert torch.equal(forced, plain)
    assert torch.equal(default, plain)


def test_qkv8_in_kernel_flag_needs_16_patch_plan(lv):
    scales = (1, 2, 3, 4)
    q, k, v = workloads.make_qkv(scales, 2, 2, 64, "bf16", 3)
    plan = lv.litevar_mask_build(scales, 1, waves_per_group=4)
    ops = []
    for t in (q, k, v):
        ops += list(lv.litevar_qkv8_quantize(t.cuda()))
    with pytest.raises(lv.LitevarError):
        lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125, in_kernel=True)


def test_qkv8_long_sequences_take_the_workspace_route(lv):
    w = workloads.get("var_d36_512")
    plan = lv.litevar_mask_build(w.scales, w.radius, waves_per_group=16)
    assert 4 * plan.n_union_keys > 5 * (plan.q_len + 2 * plan.kv_len)
    assert lv.litevar_windowed_attn_qkv8_workspace_bytes(plan, 1, 6) == 6 * 3 * plan.kv_len * 64 * 2
    # both routes agree bit for bit here too
    q, k, v = workloads.make_qkv(w.scales, 1, 6, 64, "bf16", w.seed)
    ops = []
    for t in (q, k, v):
        ops += list(lv.litevar_qkv8_quantize(t.cuda()))
    a = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125)
    b = lv.litevar_windowed_attn_qkv8_fwd(plan, *ops, 0.125, in_kernel=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
