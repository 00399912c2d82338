"""Host-side checks of the C-ABI library that need no GPU: the library loads, exports
every symbol the header declares, validates arguments before any HIP call, and its
host sizing pass reproduces the closed-form pair counts."""
import ctypes as C
import os
import re

import pytest

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    if not os.path.exists(m.lib_path()):
        from paper_2411_17178_amd import build
        build.build()
    m.load_library()
    return m


def test_library_exports_every_declared_symbol(lv):
    header = open(os.path.join(ROOT, "include", "litevar.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(litevar_[a-z_0-9]+)\s*\(", header))
    assert {"litevar_mask_build", "litevar_windowed_attn_fwd", "litevar_mask_plan_bytes"} <= names
    lib = lv.load_library()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in litevar.h but not exported"
    assert lib.litevar_version() >= 100
    assert lib.litevar_status_string(0) == b"ok"


def test_plan_struct_matches_header(lv, tmp_path):
    # the ctypes mirrors must have the C structs' sizes and field offsets (asked of gcc)
    import subprocess
    from paper_2411_17178_amd.binding import _MaskDesc, _Plan, _PlanOpts
    src = tmp_path / "sz.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "litevar.h"\n'
                   'int main(void){printf("%zu %zu %zu %zu %zu %zu\\n", sizeof(litevar_plan), '
                   'sizeof(litevar_plan_opts), sizeof(litevar_mask_desc), offsetof(litevar_plan, n_steps), '
                   'offsetof(litevar_plan, off), offsetof(litevar_plan, n_sink_scales));'
                   'printf("%zu %zu %zu %zu\\n", offsetof(litevar_plan, head_group), '
                   'offsetof(litevar_plan, retained_pairs_of_group), offsetof(litevar_mask_desc, radius_per_head), '
                   'offsetof(litevar_mask_desc, mask_mode));return 0;}\n')
    exe = tmp_path / "sz"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert got == [C.sizeof(_Plan), C.sizeof(_PlanOpts), C.sizeof(_MaskDesc), _Plan.n_steps.offset,
                   _Plan.off.offset, _Plan.n_sink_scales.offset, _Plan.head_group.offset,
                   _Plan.retained_pairs_of_group.offset, _MaskDesc.radius_per_head.offset,
                   _MaskDesc.mask_mode.offset]


def _totals():
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "pair_counts.txt")):
        parts = line.split()
        if len(parts) == 3 and not line.startswith("#") and ":" not in line:
            out[parts[0]] = int(parts[1])
    return out


@pytest.mark.parametrize("waves", [0, 4, 8, 16])
def test_host_sizing_reproduces_pair_counts(lv, waves):
    totals = _totals()
    for name, w in workloads.CONFIGS.items():
        st = lv.litevar_mask_plan_stats(w.scales, w.radius, None, w.n_sink, w.q_scales, waves)
        assert st.retained_pairs == totals[name]
        assert st.kv_len == workloads.seq_len(w.scales)
        assert st.computed_pairs == st.n_steps * 512 >= st.retained_pairs
        assert st.blob_bytes == lv.litevar_mask_plan_bytes(w.scales, w.radius, None, w.n_sink,
                                                           w.q_scales, waves)
        assert st.magic == 0 and not st.d_blob
    st = lv.litevar_mask_plan_stats((1, 2, 3, 4), 1, None, 3)
    assert st.retained_pairs == 471
    st = lv.litevar_mask_plan_stats((1, 2, 3, 4), -1)
    assert st.retained_pairs == 627


def test_descriptor_validation(lv):
    E = lv.LitevarError
    bad = [
        dict(scales=[], radius=1),
        dict(scales=[1] * 33, radius=1),
        dict(scales=[1, 0, 3], radius=1),
        dict(scales=[1, 2000], radius=1),
        dict(scales=[1, 2, 3], radius=-2),
        dict(scales=[1, 2, 3], radius=1, radius_per_key_scale=[1, -3, 0]),
        dict(scales=[1, 2, 3], radius=1, n_sink_scales=4),
        dict(scales=[1, 2, 3], radius=1, q_scales=(2, 2)),
        dict(scales=[1, 2, 3], radius=1, q_scales=(0, 4)),
        dict(scales=[1, 2, 3], radius=1, waves_per_group=5),
        dict(scales=[1, 2, 3], radius=1, waves_per_group=(4, 48, 2)),
        dict(scales=[1, 2, 3], radius=1, waves_per_group=(4, 32, 5, 0)),
    ]
    for kw in bad:
        with pytest.raises(E) as ei:
            lv.litevar_mask_plan_bytes(**kw)
        assert ei.value.status == -1, kw
    assert lv.litevar_mask_plan_bytes([1, 2, 3], 1) > 0


def test_entry_points_reject_bad_arguments_before_touching_the_gpu(lv):
    from paper_2411_17178_amd.binding import _MaskDesc, _Plan
    lib = lv.load_library()
    sc = (C.c_int32 * 3)(1, 2, 3)
    d = _MaskDesc(3, sc, 1, None, 0, 0, 3)
    plan = _Plan()
    # NULL blob, NULL plan, misaligned blob, too-small blob
    assert lib.litevar_mask_build(C.byref(d), None, None, C.c_size_t(1 << 20), None, C.byref(plan)) == -1
    assert lib.litevar_mask_build(C.byref(d), None, C.c_void_p(256), C.c_size_t(1 << 20), None, None) == -1
    assert lib.litevar_mask_build(C.byref(d), None, C.c_void_p(257), C.c_size_t(1 << 20), None, C.byref(plan)) == -1
    assert lib.litevar_mask_build(C.byref(d), None, C.c_void_p(256), C.c_size_t(16), None, C.byref(plan)) == -3
    assert b"bytes" in lib.litevar_last_error()
    assert lib.litevar_mask_plan_bytes(None, None, C.byref(C.c_size_t())) == -1
    assert lib.litevar_mask_plan_bytes(C.byref(d), None, None) == -1
    # a handle that was never built is refused by every device entry point
    stats = lv.litevar_mask_plan_stats([1, 2, 3], 1).handle
    p = C.c_void_p(4096)
    rc = lib.litevar_windowed_attn_fwd(C.byref(stats), p, p, p, p, 1, 1, 64, 0, None, None, None,
                                       C.c_float(0.125), None, C.c_uint32(0), None)
    assert rc == -5
    assert lib.litevar_mask_export_dense(C.byref(stats), 0, p, C.c_size_t(1 << 20), None, None) == -5
    assert lib.litevar_mask_export_csr(C.byref(stats), 0, p, p, C.c_size_t(1 << 20), None) == -5
    assert lib.litevar_window_table_export(C.byref(stats), 0, p, C.c_size_t(1 << 20), None) == -5
    assert lib.litevar_plan_check(None, None) == -1
    # forge a "built" handle to reach the argument checks of the attention call (still no HIP call)
    stats.magic = 0x4c56415257494e32
    stats.d_blob = 4096
    f = lambda **kw: lib.litevar_windowed_attn_fwd(  # noqa: E731
        C.byref(stats), kw.get("q", p), p, p, kw.get("o", C.c_void_p(8192)), kw.get("B", 2),
        kw.get("H", 1), kw.get("D", 64), kw.get("dt", 0), kw.get("qs"), None, None,
        C.c_float(kw.get("scale", 0.125)), kw.get("share"), C.c_uint32(kw.get("flags", 0)), None)
    assert f(q=None) == -1
    assert f(B=0) == -1
    assert f(D=128) == -2
    assert f(dt=7) == -2
    assert f(scale=0.0) == -1
    assert f(scale=float("nan")) == -1
    assert f(flags=2) == -1
    assert f(flags=1, B=3, share=p) == -1
    assert f(flags=1, B=2, share=None) == -1
    assert f(o=p) == -1
    assert f(q=C.c_void_p(4100)) == -1
    assert f(qs=(C.c_int64 * 3)(640, 640, 60)) == -1
    assert f(qs=(C.c_int64 * 3)(641, 640, 64)) == -1


def test_calibrate_validation_needs_no_gpu(lv):
    """Argument errors of the window calibration are found before any HIP call."""
    lib = lv.load_library()
    sc = (C.c_int32 * 3)(1, 2, 3)
    n = C.c_size_t(0)
    assert lib.litevar_window_calibrate_workspace_bytes(sc, 3, 2, C.byref(n)) == 0
    # [H][K][K][splits][tiles][smax] doubles: side 3 -> 25 offsets -> one tile of 256, 16 splits
    assert n.value == 2 * 3 * 3 * 4 * 1 * 3 * 8
    assert lib.litevar_window_calibrate_workspace_bytes(sc, 3, 0, C.byref(n)) == -1
    assert lib.litevar_window_calibrate_workspace_bytes(None, 3, 2, C.byref(n)) == -1
    bad = (C.c_int32 * 2)(4, 0)
    assert lib.litevar_window_calibrate_workspace_bytes(bad, 2, 1, C.byref(n)) == -1
    call = lib.litevar_window_calibrate
    ptr = C.c_void_p(4096)
    assert call(sc, 3, ptr, 1, 2, C.c_float(1.5), ptr, C.c_size_t(1 << 20), ptr, None, None) == -1
    assert b"r0" in lib.litevar_last_error()
    assert call(sc, 3, ptr, 1, 2, C.c_float(0.0), ptr, C.c_size_t(1 << 20), ptr, None, None) == -1
    assert call(sc, 3, None, 1, 2, C.c_float(0.9), ptr, C.c_size_t(1 << 20), ptr, None, None) == -1
    assert call(sc, 3, ptr, 0, 2, C.c_float(0.9), ptr, C.c_size_t(1 << 20), ptr, None, None) == -1
    assert call(sc, 3, ptr, 1, 2, C.c_float(0.9), ptr, C.c_size_t(8), ptr, None, None) == -1
    assert b"workspace" in lib.litevar_last_error()
    assert call(sc, 3, ptr, 1, 2, C.c_float(0.9), C.c_void_p(4097), C.c_size_t(1 << 20), ptr, None, None) == -1


def test_batch_heads_hint_picks_smaller_groups(lv):
    """KV step of the 10-scale list (one 16-patch group per (batch, head) pair): few pairs get
    8 or 4 patches per group so that the launch has enough workgroups; no hint, many pairs or
    an explicit group size leave the choice alone."""
    sc, q = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16), (9, 10)
    st = lambda **kw: lv.litevar_mask_plan_stats(sc, 3, None, 0, q, **kw)
    assert st().waves_per_group == 16 and st().n_groups == 1
    assert st(batch_heads=480).waves_per_group == 16
    assert st(batch_heads=240).waves_per_group == 16
    assert st(batch_heads=120).waves_per_group == 8 and st(batch_heads=120).n_groups == 2
    assert st(batch_heads=60).waves_per_group == 4 and st(batch_heads=60).n_groups == 4
    assert st(batch_heads=60, waves_per_group=16).waves_per_group == 16
    assert st(batch_heads=60).retained_pairs == st().retained_pairs
    with pytest.raises(lv.LitevarError):
        st(batch_heads=-1)
    # query scales of side <= 8 use 4 patches per group whatever the hint
    assert lv.litevar_mask_plan_stats(sc, 3, None, 0, (6, 7), batch_heads=4).waves_per_group == 4


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message that says why (one GPU only)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_host_sizing_of_band_mode_and_per_head_plans_matches_the_oracle(lv):
    import numpy as np
    import oracle
    scales = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    for waves in (4, 8, 16):
        for rad, q_scales in ((2, None), (24, (9, 10)), (0, None)):
            st = lv.litevar_mask_plan_stats(scales, rad, None, 0, q_scales, waves, mask_mode=1)
            assert st.mask_mode == 1
            assert st.retained_pairs == int(oracle.row_counts(scales, [rad] * 10, 0, q_scales, mode=1).sum())
    g = np.random.default_rng(3)
    tabs = g.integers(-1, 5, size=(3, 10, 10))
    tabs = tabs[[0, 1, 0, 2, 1]]                      # five heads, three distinct tables
    for mode in (0, 1):
        st = lv.litevar_mask_plan_stats(scales, 0, tabs.tolist(), 2, None, 16, mask_mode=mode)
        assert st.n_heads == 5 and st.n_head_groups == 3
        assert [st.head_group[h] for h in range(5)] == [0, 1, 0, 2, 1]
        per_group = [int(oracle.row_counts(scales, tabs[h], 2, mode=mode).sum()) for h in (0, 1, 3)]
        assert [int(st.retained_pairs_of_group[i]) for i in range(3)] == per_group
        assert st.retained_pairs == sum(per_group)
    E = lv.LitevarError
    import pytest as _pytest
    with _pytest.raises(E):
        lv.litevar_mask_plan_stats(scales, 1, mask_mode=2)
