"""litevar_window_calibrate_static -- the entry point for callers that cannot allocate --
through the C ABI against litevar_window_calibrate (caller-owned workspace): same kernels, so
radii and in-window sums must be identical bit for bit; two calls in a row on the library's
static scratch array, the second with a smaller input (what the first call left in the
array must not leak into it)."""
import ctypes as C

import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu

VAR_SCALES = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)


@pytest.fixture(scope="module")
def lv():
    import paper_2411_17178_amd as m
    m.load_library()
    return m


def _static(lv, scales, p, r0):
    from paper_2411_17178_amd import binding
    lib = lv.load_library()
    N, H, L, _ = p.shape
    K = len(scales)
    sc = (C.c_int32 * K)(*scales)
    radius = torch.full((H, K, K), -7, dtype=torch.int32, device=p.device)
    mass = torch.full((H, K, K, max(scales)), -1.0, dtype=torch.float64, device=p.device)
    before = torch.cuda.memory_allocated()
    rc = lib.litevar_window_calibrate_static(
        sc, C.c_int32(K), C.c_void_p(p.data_ptr()), C.c_int32(N), C.c_int32(H), C.c_float(r0),
        C.c_void_p(radius.data_ptr()), C.c_void_p(mass.data_ptr()),
        C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, lib.litevar_last_error().decode()
    assert torch.cuda.memory_allocated() == before
    return radius, mass


def test_static_scratch_entry_matches_the_workspace_entry(lv):
    big = workloads.make_attn_map(VAR_SCALES, 2, 3, 31).cuda()
    small_scales = (1, 2, 3, 5)
    small = workloads.make_attn_map(small_scales, 1, 2, 7).cuda()
    for scales, p, r0 in ((VAR_SCALES, big, 0.9), (small_scales, small, 0.8), (VAR_SCALES, big, 0.6)):
        print(f"  static calibrate: scales={scales} map{tuple(p.shape)} r0={r0}", flush=True)
        want_r, want_m = lv.litevar_window_calibrate(scales, p, r0, with_mass=True)
        got_r, got_m = _static(lv, scales, p, r0)
        torch.cuda.synchronize()
        assert torch.equal(got_r, want_r)
        assert torch.equal(got_m, want_m)


def test_static_scratch_entry_rejects_what_does_not_fit(lv):
    lib = lv.load_library()
    scales = (1, 2, 3, 4, 6, 9, 13, 18, 24, 32, 48, 64)     # partial sums far beyond 8 MiB
    sc = (C.c_int32 * len(scales))(*scales)
    dummy = torch.zeros(16, device="cuda")
    rc = lib.litevar_window_calibrate_static(
        sc, C.c_int32(len(scales)), C.c_void_p(dummy.data_ptr()), C.c_int32(1), C.c_int32(16),
        C.c_float(0.9), C.c_void_p(dummy.data_ptr()), None, None)
    assert rc == -2 and b"static scratch" in lib.litevar_last_error()
