"""ctypes binding of liblitevar.so: argument marshalling only.

Function names match include/litevar.h.  Tensors are torch CUDA(HIP) tensors; the
binding passes their data pointers and the current stream handle to the library.
"""
import contextlib
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblitevar.so")
_lib = None

MAX_SCALES = 32
MAX_HEADS = 256
MASK_WINDOW_2D, MASK_BAND_1D = 0, 1
FLAG_CFG_SHARE = 1
FLAG_QKV8_IN_KERNEL = 2
DT_BF16, DT_F32 = 0, 1


class LitevarError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"litevar status {status}: {message}")
        self.status = status


class _MaskDesc(C.Structure):
    _fields_ = [("n_scales", C.c_int32), ("scales", C.POINTER(C.c_int32)),
                ("radius", C.c_int32), ("radius_per_key_scale", C.POINTER(C.c_int32)),
                ("n_sink_scales", C.c_int32), ("q_scale_begin", C.c_int32),
                ("q_scale_end", C.c_int32), ("radius_per_scale_pair", C.POINTER(C.c_int32)),
                ("n_heads", C.c_int32), ("radius_per_head", C.POINTER(C.c_int32)),
                ("mask_mode", C.c_int32)]


class _PlanOpts(C.Structure):
    _fields_ = [("waves_per_group", C.c_int32), ("chunk_keys", C.c_int32),
                ("prefetch_chunks", C.c_int32), ("spare_chunks", C.c_int32),
                ("patches_per_wave", C.c_int32), ("batch_heads_hint", C.c_int32),
                ("spin_limit", C.c_int32), ("reserved", C.c_int32 * 1)]


class _Plan(C.Structure):
    _fields_ = [("magic", C.c_uint64), ("d_blob", C.c_void_p), ("blob_bytes", C.c_uint64),
                ("n_scales", C.c_int32), ("q_scale_begin", C.c_int32), ("q_scale_end", C.c_int32),
                ("kv_len", C.c_int32), ("q_len", C.c_int32), ("q_token_begin", C.c_int32),
                ("side_max", C.c_int32), ("waves_per_group", C.c_int32),
                ("chunk_keys", C.c_int32), ("ring_chunks", C.c_int32),
                ("prefetch_chunks", C.c_int32), ("n_groups", C.c_int32), ("n_patches", C.c_int32),
                ("n_steps", C.c_int64), ("n_union_keys", C.c_int64),
                ("retained_pairs", C.c_int64), ("computed_pairs", C.c_int64),
                ("off", C.c_uint64 * 12), ("scales", C.c_int32 * MAX_SCALES),
                ("radii", C.c_int32 * MAX_SCALES), ("n_sink_scales", C.c_int32),
                ("patches_per_wave", C.c_int32), ("spin_limit", C.c_int32), ("mask_mode", C.c_int32),
                ("n_heads", C.c_int32), ("n_head_groups", C.c_int32), ("head_group", C.c_uint8 * MAX_HEADS),
                ("retained_pairs_of_group", C.c_int64 * MAX_HEADS)]


def lib_path():
    return _LIB_PATH


def load_library():
    """Load liblitevar.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2411_17178_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback")
    lib = C.CDLL(_LIB_PATH)
    lib.litevar_status_string.restype = C.c_char_p
    lib.litevar_last_error.restype = C.c_char_p
    lib.litevar_version.restype = C.c_int32
    for name in ("litevar_scale_offsets", "litevar_mask_plan_bytes", "litevar_mask_plan_stats", "litevar_mask_build", "litevar_plan_check",
                 "litevar_window_table_export", "litevar_mask_export_dense",
                 "litevar_mask_export_csr", "litevar_windowed_attn_fwd",
                 "litevar_window_calibrate_workspace_bytes", "litevar_window_calibrate",
                 "litevar_window_calibrate_static", "litevar_window_calibrate_band_workspace_bytes",
                 "litevar_window_calibrate_band", "litevar_peak_copy", "litevar_peak_read", "litevar_peak_mfma_bf16", "litevar_qkv8_quantize",
                 "litevar_qkv8_dequantize", "litevar_windowed_attn_qkv8_workspace_bytes",
                 "litevar_windowed_attn_qkv8_fwd"):
        getattr(lib, name).restype = C.c_int32
    _lib = lib
    return lib


@contextlib.contextmanager
def use_library(path):
    """Inside the block the binding's calls go to another build of the library at `path` (the
    bounds-checking one: paper_2411_17178_amd.build.LIB_DEBUG_BOUNDS).  Plans are plain data
    plus a device blob and may cross between builds."""
    global _lib, _LIB_PATH
    saved = (_lib, _LIB_PATH)
    _lib, _LIB_PATH = None, path
    try:
        load_library()
        yield
    finally:
        _lib, _LIB_PATH = saved


def _check(rc):
    if rc != 0:
        raise LitevarError(rc, load_library().litevar_last_error().decode())


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _make_desc(scales, radius, radius_per_key_scale, n_sink_scales, q_scales, mask_mode=0):
    K = len(scales)
    sc = (C.c_int32 * K)(*[int(s) for s in scales])
    # radius_per_key_scale: [K] (one radius per key scale), a table [K][K] ([query scale][key
    # scale], one window size per scale and part) or one such table per head, [H][K][K]
    rp = pair = heads = None
    n_heads = 0
    if radius_per_key_scale is not None:
        rows = list(radius_per_key_scale)
        if len(rows) and hasattr(rows[0], "__len__") and len(rows[0]) and hasattr(rows[0][0], "__len__"):
            n_heads = len(rows)
            assert all(len(t) == K and all(len(r) == K for r in t) for t in rows), "radius tables must be [H][K][K]"
            heads = (C.c_int32 * (n_heads * K * K))(*[int(r) for t in rows for row in t for r in row])
        elif len(rows) and hasattr(rows[0], "__len__"):
            assert len(rows) == K and all(len(r) == K for r in rows), "radius table must be [K][K]"
            pair = (C.c_int32 * (K * K))(*[int(r) for row in rows for r in row])
        else:
            assert len(rows) == K, "one radius per key scale"
            rp = (C.c_int32 * K)(*[int(r) for r in rows])
    qb, qe = (0, K) if q_scales is None else q_scales
    d = _MaskDesc(K, sc, int(radius), rp, int(n_sink_scales), int(qb), int(qe), pair, n_heads, heads,
                  int(mask_mode))
    d._keep = (sc, rp, pair, heads)
    return d


def _make_opts(waves_per_group, batch_heads=0, spin_limit=0):
    """waves_per_group: an int, or a tuple (waves, chunk_keys, prefetch_chunks, spare_chunks,
    patches_per_wave); 0 (spare: -1) = library default."""
    o = _PlanOpts()
    o.spare_chunks = -1
    o.batch_heads_hint = int(batch_heads)
    o.spin_limit = int(spin_limit)
    if isinstance(waves_per_group, (tuple, list)):
        vals = [int(x) for x in waves_per_group] + [0, 0, -1]
        o.waves_per_group, o.chunk_keys, o.prefetch_chunks = vals[0], vals[1], vals[2]
        o.spare_chunks = vals[3] if len(waves_per_group) > 3 else -1
        o.patches_per_wave = vals[4] if len(waves_per_group) > 4 else 0
    else:
        o.waves_per_group = int(waves_per_group)
    return o


class Plan:
    """A built plan: the host handle plus the torch tensor that owns the device blob."""

    def __init__(self, handle, blob):
        self.handle = handle
        self.blob = blob

    def __getattr__(self, name):
        return getattr(self.handle, name)

    @property
    def scales(self):
        return [self.handle.scales[i] for i in range(self.handle.n_scales)]


def litevar_scale_offsets(scales):
    """[first token of scale 0, ..., of scale K-1, sequence length] (the library's scale table)."""
    K = len(scales)
    sc = (C.c_int32 * K)(*[int(s) for s in scales])
    out = (C.c_int64 * (K + 1))()
    _check(load_library().litevar_scale_offsets(sc, C.c_int32(K), out))
    return [int(x) for x in out]


def litevar_mask_plan_bytes(scales, radius, radius_per_key_scale=None, n_sink_scales=0,
                            q_scales=None, waves_per_group=0, batch_heads=0, mask_mode=0):
    d = _make_desc(scales, radius, radius_per_key_scale, n_sink_scales, q_scales, mask_mode)
    o = _make_opts(waves_per_group, batch_heads)
    n = C.c_size_t(0)
    _check(load_library().litevar_mask_plan_bytes(C.byref(d), C.byref(o), C.byref(n)))
    return int(n.value)


def litevar_mask_plan_stats(scales, radius, radius_per_key_scale=None, n_sink_scales=0,
                            q_scales=None, waves_per_group=0, batch_heads=0, mask_mode=0):
    """Host-only dry run: a Plan without a device blob (sizes and pair counts only)."""
    d = _make_desc(scales, radius, radius_per_key_scale, n_sink_scales, q_scales, mask_mode)
    o = _make_opts(waves_per_group, batch_heads)
    handle = _Plan()
    _check(load_library().litevar_mask_plan_stats(C.byref(d), C.byref(o), C.byref(handle)))
    return Plan(handle, None)


def litevar_mask_build(scales, radius, radius_per_key_scale=None, n_sink_scales=0, q_scales=None,
                       waves_per_group=0, device="cuda", stream=None, blob=None, batch_heads=0,
                       spin_limit=0, mask_mode=0):
    """Build a plan on the device.  `blob` (optional uint8 CUDA tensor, large enough and
    256-byte aligned) is reused as the plan's storage instead of a fresh allocation.
    `batch_heads` (optional): B * H of the launches the plan is for, which lets the library
    pick smaller groups for small batches."""
    lib = load_library()
    d = _make_desc(scales, radius, radius_per_key_scale, n_sink_scales, q_scales, mask_mode)
    o = _make_opts(waves_per_group, batch_heads, spin_limit)
    n = C.c_size_t(0)
    _check(lib.litevar_mask_plan_bytes(C.byref(d), C.byref(o), C.byref(n)))
    if blob is None:
        blob = torch.empty(n.value, dtype=torch.uint8, device=device)
    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    handle = _Plan()
    _check(lib.litevar_mask_build(C.byref(d), C.byref(o), C.c_void_p(blob.data_ptr()),
                                  C.c_size_t(blob.numel()), _stream_handle(stream),
                                  C.byref(handle)))
    return Plan(handle, blob)


def litevar_plan_check(plan, stream=None):
    _check(load_library().litevar_plan_check(C.byref(plan.handle), _stream_handle(stream)))


def litevar_window_table_export(plan, stream=None, head=0):
    K, smax = plan.n_scales, plan.side_max
    out = torch.empty((K, K, smax, 2), dtype=torch.int16, device=plan.blob.device)
    _check(load_library().litevar_window_table_export(
        C.byref(plan.handle), C.c_int32(head), C.c_void_p(out.data_ptr()), C.c_size_t(out.numel() * 2),
        _stream_handle(stream)))
    return out


def litevar_mask_export_dense(plan, stream=None, head=0):
    """(uint8 [q_len, kv_len] mask of head `head`, number of work-list entries)."""
    mask = torch.empty((plan.q_len, plan.kv_len), dtype=torch.uint8, device=plan.blob.device)
    count = torch.empty(1, dtype=torch.int64, device=plan.blob.device)
    _check(load_library().litevar_mask_export_dense(
        C.byref(plan.handle), C.c_int32(head), C.c_void_p(mask.data_ptr()), C.c_size_t(mask.numel()),
        C.c_void_p(count.data_ptr()), _stream_handle(stream)))
    return mask, count


def litevar_mask_export_csr(plan, stream=None, head=0):
    kept = int(plan.retained_pairs_of_group[plan.head_group[head] if plan.n_heads else 0])
    rowptr = torch.empty(plan.q_len + 1, dtype=torch.int64, device=plan.blob.device)
    cols = torch.empty(max(1, kept), dtype=torch.int32, device=plan.blob.device)
    _check(load_library().litevar_mask_export_csr(
        C.byref(plan.handle), C.c_int32(head), C.c_void_p(rowptr.data_ptr()), C.c_void_p(cols.data_ptr()),
        C.c_size_t(cols.numel()), _stream_handle(stream)))
    return rowptr, cols[:kept]


def _strides(t):
    assert t.dim() == 4 and t.stride(3) == 1, "expected [B, H, tokens, D] with contiguous D"
    return (C.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def litevar_windowed_attn_fwd(plan, q, k, v, sm_scale, out=None, cfg_share=None, stream=None):
    """out[B,H,q_len,D] = windowed attention of q against k, v under `plan`.

    cfg_share: optional uint8 CUDA tensor [H, K]; when given, the CFG shared-output
    flag is set and rows b + B/2 reuse rows b where the table is non-zero.
    """
    lib = load_library()
    assert q.is_cuda and k.is_cuda and v.is_cuda
    assert q.dtype == k.dtype == v.dtype
    if q.dtype == torch.bfloat16:
        dt = DT_BF16
    elif q.dtype == torch.float32:
        dt = DT_F32
    else:
        raise TypeError(f"unsupported dtype {q.dtype}")
    B, H, Lq, D = q.shape
    assert Lq == plan.q_len and k.shape == (B, H, plan.kv_len, D) and v.shape == k.shape
    if out is None:
        out = torch.empty_like(q)
    assert out.shape == q.shape and out.dtype == q.dtype and out.is_cuda
    flags, share_ptr = 0, None
    if cfg_share is not None:
        assert cfg_share.is_cuda and cfg_share.dtype == torch.uint8 and cfg_share.is_contiguous()
        assert cfg_share.shape == (H, plan.n_scales)
        flags, share_ptr = FLAG_CFG_SHARE, C.c_void_p(cfg_share.data_ptr())
    assert k.stride() == v.stride(), "k and v must share strides"
    _check(lib.litevar_windowed_attn_fwd(
        C.byref(plan.handle), C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
        C.c_void_p(v.data_ptr()), C.c_void_p(out.data_ptr()), C.c_int32(B), C.c_int32(H),
        C.c_int32(D), C.c_int32(dt), _strides(q), _strides(k), _strides(out),
        C.c_float(sm_scale), share_ptr, C.c_uint32(flags), _stream_handle(stream)))
    return out


def litevar_window_calibrate(scales, attn_map, r0, with_mass=False, stream=None):
    """Window radii [H, K, K] (int32, -1 above the diagonal) from post-softmax attention maps
    `attn_map` [N, H, L, L] (float32 CUDA tensor); with_mass also returns the in-window sums
    [H, K, K, smax] (float64)."""
    lib = load_library()
    assert attn_map.is_cuda and attn_map.dtype == torch.float32 and attn_map.is_contiguous()
    N, H, L, L2 = attn_map.shape
    K = len(scales)
    sc = (C.c_int32 * K)(*[int(s) for s in scales])
    n = C.c_size_t(0)
    _check(lib.litevar_window_calibrate_workspace_bytes(sc, C.c_int32(K), C.c_int32(H), C.byref(n)))
    assert L == L2 == litevar_scale_offsets(scales)[-1]
    dev = attn_map.device
    work = torch.empty(max(1, (n.value + 7) // 8), dtype=torch.float64, device=dev)
    radius = torch.empty((H, K, K), dtype=torch.int32, device=dev)
    mass = torch.empty((H, K, K, max(int(s) for s in scales)), dtype=torch.float64, device=dev) \
        if with_mass else None
    _check(lib.litevar_window_calibrate(
        sc, C.c_int32(K), C.c_void_p(attn_map.data_ptr()), C.c_int32(N), C.c_int32(H),
        C.c_float(r0), C.c_void_p(work.data_ptr()), C.c_size_t(work.numel() * 8),
        C.c_void_p(radius.data_ptr()), C.c_void_p(mass.data_ptr()) if with_mass else None,
        _stream_handle(stream)))
    return (radius, mass) if with_mass else radius


def litevar_window_calibrate_band(scales, attn_map, r0, with_mass=False, stream=None):
    """Band radii (the band mask mode's parts) from post-softmax maps [N][H][L][L] (float32 CUDA
    tensor): int32 [H][K][K] (and the in-band sums, float64 [H][K][K][C], when asked)."""
    lib = load_library()
    assert attn_map.is_cuda and attn_map.dtype == torch.float32 and attn_map.is_contiguous()
    N, H, L, L2 = attn_map.shape
    K = len(scales)
    sq = [int(s) * int(s) for s in scales]
    assert L == L2 == sum(sq)
    sc = (C.c_int32 * K)(*[int(s) for s in scales])
    n = C.c_size_t(0)
    _check(lib.litevar_window_calibrate_band_workspace_bytes(sc, C.c_int32(K), C.c_int32(H), C.byref(n)))
    work = torch.empty(n.value, dtype=torch.uint8, device=attn_map.device)
    radius = torch.empty((H, K, K), dtype=torch.int32, device=attn_map.device)
    cols = max([sum(sq[:3])] + sq[3:])
    mass = torch.empty((H, K, K, cols), dtype=torch.float64, device=attn_map.device) if with_mass else None
    _check(lib.litevar_window_calibrate_band(
        sc, C.c_int32(K), C.c_void_p(attn_map.data_ptr()), C.c_int32(N), C.c_int32(H), C.c_float(r0),
        C.c_void_p(work.data_ptr()), C.c_size_t(n.value), C.c_void_p(radius.data_ptr()),
        C.c_void_p(mass.data_ptr()) if with_mass else None, _stream_handle(stream)))
    return (radius, mass) if with_mass else radius


def litevar_window_calibrate_static(scales, attn_map, r0, radius, mass=None, stream=None):
    """litevar_window_calibrate on the library's static scratch array: allocates nothing, the
    caller brings the outputs `radius` [H, K, K] int32 and, optionally, `mass`
    [H, K, K, smax] float64."""
    lib = load_library()
    assert attn_map.is_cuda and attn_map.dtype == torch.float32 and attn_map.is_contiguous()
    N, H, L, L2 = attn_map.shape
    K = len(scales)
    assert L == L2 == litevar_scale_offsets(scales)[-1] and radius.is_cuda and radius.dtype == torch.int32 and radius.shape == (H, K, K)
    assert radius.is_contiguous()
    if mass is not None:
        assert mass.is_cuda and mass.dtype == torch.float64 and mass.is_contiguous()
        assert mass.shape == (H, K, K, max(int(s) for s in scales))
    sc = (C.c_int32 * K)(*[int(s) for s in scales])
    _check(lib.litevar_window_calibrate_static(
        sc, C.c_int32(K), C.c_void_p(attn_map.data_ptr()), C.c_int32(N), C.c_int32(H),
        C.c_float(r0), C.c_void_p(radius.data_ptr()),
        C.c_void_p(mass.data_ptr()) if mass is not None else None, _stream_handle(stream)))
    return radius


def litevar_qkv8_quantize(x, stream=None):
    """Per-token 8-bit min-max quantisation of x [..., 64] (bf16 or fp32 CUDA tensor, packed):
    returns (codes int8 like x, scale_zero float32 [..., 2])."""
    assert x.is_cuda and x.is_contiguous() and x.shape[-1] == 64
    dt = {torch.bfloat16: DT_BF16, torch.float32: DT_F32}[x.dtype]
    rows = x.numel() // 64
    codes = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    sz = torch.empty(x.shape[:-1] + (2,), dtype=torch.float32, device=x.device)
    _check(load_library().litevar_qkv8_quantize(
        C.c_void_p(x.data_ptr()), C.c_int32(dt), C.c_int64(rows), C.c_int64(64), C.c_int32(64),
        C.c_void_p(codes.data_ptr()), C.c_void_p(sz.data_ptr()), _stream_handle(stream)))
    return codes, sz


def litevar_qkv8_dequantize(codes, scale_zero, stream=None):
    assert codes.is_cuda and codes.dtype == torch.int8 and codes.is_contiguous() and codes.shape[-1] == 64
    assert scale_zero.is_cuda and scale_zero.dtype == torch.float32 and scale_zero.is_contiguous()
    assert scale_zero.shape == codes.shape[:-1] + (2,)
    out = torch.empty(codes.shape, dtype=torch.bfloat16, device=codes.device)
    _check(load_library().litevar_qkv8_dequantize(
        C.c_void_p(codes.data_ptr()), C.c_void_p(scale_zero.data_ptr()), C.c_int64(codes.numel() // 64),
        C.c_int32(64), C.c_void_p(out.data_ptr()), _stream_handle(stream)))
    return out


def litevar_windowed_attn_qkv8_workspace_bytes(plan, B, H):
    n = C.c_size_t(0)
    _check(load_library().litevar_windowed_attn_qkv8_workspace_bytes(C.byref(plan.handle), C.c_int32(B),
                                                                      C.c_int32(H), C.byref(n)))
    return n.value


def litevar_windowed_attn_qkv8_fwd(plan, q8, q_sz, k8, k_sz, v8, v_sz, sm_scale, out=None,
                                   cfg_share=None, workspace=None, stream=None, in_kernel=False):
    """Windowed attention on 8-bit Q, K, V (codes int8 [B,H,L,64] + (scale, zero) float32
    [B,H,L,2], as litevar_qkv8_quantize returns them); output bf16 [B,H,q_len,64].
    in_kernel: pass LITEVAR_FLAG_QKV8_IN_KERNEL."""
    lib = load_library()
    B, H, Lq, D = q8.shape
    for t, sz in ((q8, q_sz), (k8, k_sz), (v8, v_sz)):
        assert t.is_cuda and t.dtype == torch.int8 and t.is_contiguous()
        assert sz.is_cuda and sz.dtype == torch.float32 and sz.is_contiguous() and sz.shape == t.shape[:-1] + (2,)
    assert Lq == plan.q_len and k8.shape == (B, H, plan.kv_len, D) and v8.shape == k8.shape
    n = C.c_size_t(0)
    _check(lib.litevar_windowed_attn_qkv8_workspace_bytes(C.byref(plan.handle), C.c_int32(B), C.c_int32(H), C.byref(n)))
    if workspace is None:
        workspace = torch.empty(n.value, dtype=torch.uint8, device=q8.device)
    assert workspace.is_cuda and workspace.numel() * workspace.element_size() >= n.value
    if out is None:
        out = torch.empty(q8.shape, dtype=torch.bfloat16, device=q8.device)
    assert out.dtype == torch.bfloat16 and out.shape == q8.shape and out.is_contiguous()
    flags, share_ptr = 0, None
    if cfg_share is not None:
        assert cfg_share.is_cuda and cfg_share.dtype == torch.uint8 and cfg_share.is_contiguous()
        assert cfg_share.shape == (H, plan.n_scales)
        flags, share_ptr = FLAG_CFG_SHARE, C.c_void_p(cfg_share.data_ptr())
    if in_kernel:
        flags |= FLAG_QKV8_IN_KERNEL
    _check(lib.litevar_windowed_attn_qkv8_fwd(
        C.byref(plan.handle), C.c_void_p(q8.data_ptr()), C.c_void_p(q_sz.data_ptr()),
        C.c_void_p(k8.data_ptr()), C.c_void_p(k_sz.data_ptr()), C.c_void_p(v8.data_ptr()),
        C.c_void_p(v_sz.data_ptr()), C.c_void_p(out.data_ptr()), C.c_int32(B), C.c_int32(H), C.c_int32(D),
        C.c_float(sm_scale), share_ptr, C.c_uint32(flags), C.c_void_p(workspace.data_ptr()),
        C.c_size_t(workspace.numel() * workspace.element_size()), _stream_handle(stream)))
    return out


def litevar_peak_copy(src, dst, stream=None):
    """Enqueue the library's streaming copy of src into dst (uint8 CUDA tensors of one size)."""
    assert src.is_cuda and dst.is_cuda and src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _check(load_library().litevar_peak_copy(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()),
                                            C.c_size_t(src.numel() * src.element_size()), _stream_handle(stream)))


def litevar_peak_read(src, out, stream=None):
    """Enqueue the library's read-only pass over src (a CUDA tensor); out: 4 bytes, CUDA."""
    _check(load_library().litevar_peak_read(C.c_void_p(src.data_ptr()),
                                            C.c_size_t(src.numel() * src.element_size()),
                                            C.c_void_p(out.data_ptr()), _stream_handle(stream)))


def litevar_peak_mfma_bf16(iters, out, stream=None):
    """Enqueue the library's register-only bf16 MFMA loop; returns the flops it performs."""
    flops = C.c_double(0.0)
    _check(load_library().litevar_peak_mfma_bf16(C.c_int32(iters), C.c_void_p(out.data_ptr()),
                                                 C.byref(flops), _stream_handle(stream)))
    return flops.value


def prepare_attn_call(plan, q, k, v, sm_scale, out, cfg_share=None, stream=None):
    """Marshal the arguments of litevar_windowed_attn_fwd once; returns a zero-argument
    callable that enqueues the call (for launch-rate-sensitive loops).  The tensors, the
    plan and the stream must outlive the callable."""
    lib = load_library()
    assert q.is_cuda and q.dtype == k.dtype == v.dtype == out.dtype
    dt = {torch.bfloat16: DT_BF16, torch.float32: DT_F32}[q.dtype]
    B, H, Lq, D = q.shape
    assert Lq == plan.q_len and k.shape == (B, H, plan.kv_len, D) and v.shape == k.shape
    assert out.shape == q.shape and k.stride() == v.stride()
    flags, share_ptr = 0, None
    if cfg_share is not None:
        assert cfg_share.is_cuda and cfg_share.dtype == torch.uint8 and cfg_share.is_contiguous()
        assert cfg_share.shape == (H, plan.n_scales)
        flags, share_ptr = FLAG_CFG_SHARE, C.c_void_p(cfg_share.data_ptr())
    args = (C.byref(plan.handle), C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
            C.c_void_p(v.data_ptr()), C.c_void_p(out.data_ptr()), C.c_int32(B), C.c_int32(H),
            C.c_int32(D), C.c_int32(dt), _strides(q), _strides(k), _strides(out),
            C.c_float(sm_scale), share_ptr, C.c_uint32(flags), _stream_handle(stream))
    fn = lib.litevar_windowed_attn_fwd

    def call():
        rc = fn(*args)
        if rc != 0:
            _check(rc)
    call._keep = (plan, q, k, v, out, cfg_share, args)
    return call
