"""ctypes front-end of oracle/litevar_oracle.c (test infrastructure only).

Argument marshalling only; all arithmetic is in the C file.  Inputs may be
float64 / float32 numpy arrays or uint16 arrays holding bf16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def _L():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _lib.lvo_seq_len.restype = C.c_int64
        _lib.lvo_scale_offset.restype = C.c_int64
    return _lib


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _rtab(scales, radii):
    """The C side's [K][K] radius table ([query scale][key scale]) from either one radius
    per key scale (the same for every query scale) or a full table."""
    K = len(scales)
    r = np.asarray(radii, dtype=np.int32)
    if r.ndim == 1:
        assert r.shape == (K,)
        r = np.tile(r, (K, 1))
    assert r.shape == (K, K)
    return np.ascontiguousarray(r)


def expand_radii(scales, radius, radius_per_key_scale=None):
    """One radius per key scale; a negative radius means a dense part."""
    K = len(scales)
    if radius_per_key_scale is not None:
        r = [int(x) for x in radius_per_key_scale]
        assert len(r) == K
        return r
    return [int(radius)] * K


def seq_len(scales):
    s = _i32(scales)
    return int(_L().lvo_seq_len(C.c_int32(len(s)), _p(s)))


def scale_offsets(scales):
    s = _i32(scales)
    return [int(_L().lvo_scale_offset(C.c_int32(len(s)), _p(s), C.c_int32(k)))
            for k in range(len(s) + 1)]


def token_coords(scales, t):
    s = _i32(scales)
    k, y, x = C.c_int32(), C.c_int32(), C.c_int32()
    rc = _L().lvo_token_coords(C.c_int32(len(s)), _p(s), C.c_int64(t),
                               C.byref(k), C.byref(y), C.byref(x))
    if rc:
        raise ValueError("token out of range")
    return k.value, y.value, x.value


def allowed(scales, radii, n_sink, tq, tk, mode=0):
    s, r = _i32(scales), _rtab(scales, radii)
    rc = _L().lvo_allowed(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(n_sink), C.c_int32(mode),
                          C.c_int64(tq), C.c_int64(tk))
    if rc < 0:
        raise ValueError("token out of range")
    return bool(rc)


def _qrange(scales, q_scales):
    K = len(scales)
    qb, qe = (0, K) if q_scales is None else q_scales
    off = scale_offsets(scales)
    return qb, qe, off[qe] - off[qb]


def mask_dense(scales, radii, n_sink=0, q_scales=None, mode=0):
    """mode 0: square window in the key scale's grid; mode 1: band around each part's diagonal"""
    s, r = _i32(scales), _rtab(scales, radii)
    qb, qe, Lq = _qrange(scales, q_scales)
    m = np.empty((Lq, seq_len(scales)), dtype=np.uint8)
    rc = _L().lvo_mask_dense(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(mode), C.c_int32(n_sink),
                             C.c_int32(qb), C.c_int32(qe), _p(m))
    if rc:
        raise ValueError(f"lvo_mask_dense failed: {rc}")
    return m


def row_counts(scales, radii, n_sink=0, q_scales=None, mode=0):
    s, r = _i32(scales), _rtab(scales, radii)
    qb, qe, Lq = _qrange(scales, q_scales)
    cnt = np.empty(Lq, dtype=np.int64)
    rc = _L().lvo_row_counts(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(mode), C.c_int32(n_sink),
                             C.c_int32(qb), C.c_int32(qe), _p(cnt))
    if rc:
        raise ValueError(f"lvo_row_counts failed: {rc}")
    return cnt


def index_sets(scales, radii, n_sink=0, q_scales=None, mode=0):
    """(rowptr[Lq+1] int64, cols int32): ascending allowed keys of every query."""
    s, r = _i32(scales), _rtab(scales, radii)
    qb, qe, Lq = _qrange(scales, q_scales)
    cnt = row_counts(scales, radii, n_sink, q_scales, mode)
    rowptr = np.zeros(Lq + 1, dtype=np.int64)
    np.cumsum(cnt, out=rowptr[1:])
    cols = np.empty(int(rowptr[-1]), dtype=np.int32)
    rc = _L().lvo_index_sets(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(mode), C.c_int32(n_sink),
                             C.c_int32(qb), C.c_int32(qe), _p(rowptr), _p(cols),
                             C.c_int64(cols.size))
    if rc:
        raise ValueError(f"lvo_index_sets failed: {rc}")
    return rowptr, cols


def _dtype_code(a):
    if a.dtype == np.float64:
        return 0
    if a.dtype == np.float32:
        return 1
    if a.dtype == np.uint16:
        return 2
    raise TypeError("inputs must be float64, float32 or uint16 (bf16 bits)")


def attn(scales, radii, q, k, v, sm_scale, n_sink=0, q_scales=None, rows=None,
         bh_range=None, mode=0):
    """fp64 windowed attention.  q [B,H,Lq,D]; k,v [B,H,L,D]; returns [B,H,n_rows,D].
    radii: [K], [K][K], or one table per head [H][K][K]."""
    s = _i32(scales)
    rr = np.asarray(radii, dtype=np.int32)
    per_head = rr.ndim == 3
    if per_head:
        assert rr.shape == (q.shape[1], len(s), len(s))
        r = np.ascontiguousarray(rr)
    else:
        r = _rtab(scales, radii)
    qb, qe, Lq = _qrange(scales, q_scales)
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    code = _dtype_code(q)
    assert _dtype_code(k) == code and _dtype_code(v) == code
    B, H, lq, D = q.shape
    assert lq == Lq and k.shape == (B, H, seq_len(scales), D) and v.shape == k.shape
    if rows is not None:
        rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        n_rows = rows.size
    else:
        n_rows = Lq
    b0, b1 = (0, B * H) if bh_range is None else bh_range
    out = np.zeros((B, H, n_rows, D), dtype=np.float64)
    rc = _L().lvo_attn(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(n_sink),
                       C.c_int32(mode), C.c_int32(1 if per_head else 0),
                       C.c_int32(qb), C.c_int32(qe), _p(q), _p(k), _p(v),
                       C.c_int32(code), C.c_int32(B), C.c_int32(H), C.c_int32(D),
                       C.c_double(sm_scale), C.c_int64(n_rows),
                       _p(rows) if rows is not None else None,
                       C.c_int64(b0), C.c_int64(b1), _p(out))
    if rc:
        raise ValueError(f"lvo_attn failed: {rc}")
    return out


def attn_probs(scales, radii, q, k, v, sm_scale, bh, ql, n_sink=0, q_scales=None, mode=0):
    """(probs[L], out[D]) of one (b*H+h, local query) pair, fp64."""
    s, r = _i32(scales), _rtab(scales, radii)
    qb, qe, Lq = _qrange(scales, q_scales)
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    code = _dtype_code(q)
    B, H, lq, D = q.shape
    probs = np.zeros(seq_len(scales), dtype=np.float64)
    out = np.zeros(D, dtype=np.float64)
    rc = _L().lvo_attn_probs(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(n_sink), C.c_int32(mode),
                             C.c_int32(qb), C.c_int32(qe), _p(q), _p(k), _p(v),
                             C.c_int32(code), C.c_int32(B), C.c_int32(H), C.c_int32(D),
                             C.c_double(sm_scale), C.c_int64(bh), C.c_int64(ql),
                             _p(probs), _p(out))
    if rc:
        raise ValueError(f"lvo_attn_probs failed: {rc}")
    return probs, out


def cfg_share(scales, o, share, q_scales=None):
    """In-place cond -> uncond copy of o [B,H,Lq,D] fp64 for share[H,K] != 0."""
    s = _i32(scales)
    qb, qe, Lq = _qrange(scales, q_scales)
    assert o.dtype == np.float64 and o.flags.c_contiguous
    B, H, lq, D = o.shape
    assert lq == Lq
    share = np.ascontiguousarray(np.asarray(share, dtype=np.uint8))
    assert share.shape == (H, len(s))
    rc = _L().lvo_cfg_share(C.c_int32(len(s)), _p(s), C.c_int32(qb), C.c_int32(qe),
                            _p(share), C.c_int32(B), C.c_int32(H), C.c_int32(D), _p(o))
    if rc:
        raise ValueError(f"lvo_cfg_share failed: {rc}")
    return o


def calibrate(scales, p, r0, with_mass=False):
    """Window radii from a post-softmax attention map p[N][H][L][L] (float64): the smallest
    radius per (head, query scale, key scale) whose window holds the fraction r0 of the
    part's values.  Returns radius[H][K][K] (and mass[H][K][K][smax] when asked)."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    N, H, L, L2 = p.shape
    K = len(scales)
    assert L == L2 == seq_len(scales)
    smax = int(max(scales))
    radius = np.zeros((H, K, K), dtype=np.int32)
    mass = np.zeros((H, K, K, smax), dtype=np.float64) if with_mass else None
    sc = _i32(scales)
    rc = _L().lvo_calibrate(C.c_int32(K), _p(sc), _p(p), C.c_int32(N), C.c_int32(H),
                            C.c_double(float(r0)), _p(radius), _p(mass) if with_mass else None,
                            C.c_int32(smax))
    assert rc == 0, rc
    return (radius, mass) if with_mass else radius


def band_part_columns(scales):
    """Largest number of columns of a part of the band reading (first three key scales merged)."""
    s = [int(x) * int(x) for x in scales]
    return max([sum(s[:3])] + s[3:])


def calibrate_band(scales, p, r0, with_mass=False):
    """Band radii (Section 2 step (2) read literally: parts with the first three key scales
    merged, a band around each part's diagonal) from a post-softmax map p[N][H][L][L]: the
    smallest radius per (head, query scale, part) whose band holds the fraction r0 of the
    part's values, written to every key scale of the part.  Returns radius[H][K][K] (and
    mass[H][K][K][band_part_columns(scales)] when asked)."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    N, H, L, L2 = p.shape
    K = len(scales)
    assert L == L2 == seq_len(scales)
    mcols = band_part_columns(scales)
    radius = np.zeros((H, K, K), dtype=np.int32)
    mass = np.zeros((H, K, K, mcols), dtype=np.float64) if with_mass else None
    sc = _i32(scales)
    rc = _L().lvo_calibrate_band(C.c_int32(K), _p(sc), _p(p), C.c_int32(N), C.c_int32(H),
                                 C.c_double(float(r0)), _p(radius), _p(mass) if with_mass else None,
                                 C.c_int32(mcols))
    assert rc == 0, rc
    return (radius, mass) if with_mass else radius


def quantize_rows(x, bits=8):
    """Section 4 min-max quantiser, one (scale, zero) per row of the last axis.
    Returns (codes int32 like x, scale float64 [rows], zero float64 [rows])."""
    x = np.ascontiguousarray(x)
    code = _dtype_code(x)
    D = x.shape[-1]
    rows = x.size // D
    codes = np.empty(x.shape, dtype=np.int32)
    scale = np.empty(x.shape[:-1], dtype=np.float64)
    zero = np.empty(x.shape[:-1], dtype=np.float64)
    rc = _L().lvo_quantize_rows(_p(x), C.c_int32(code), C.c_int64(rows), C.c_int32(D),
                                C.c_int32(bits), _p(codes), _p(scale), _p(zero))
    if rc:
        raise ValueError(f"lvo_quantize_rows failed: {rc}")
    return codes, scale, zero


def dequantize_rows(codes, scale, zero):
    codes = np.ascontiguousarray(codes, dtype=np.int32)
    scale = np.ascontiguousarray(scale, dtype=np.float64)
    zero = np.ascontiguousarray(zero, dtype=np.float64)
    D = codes.shape[-1]
    out = np.empty(codes.shape, dtype=np.float64)
    rc = _L().lvo_dequantize_rows(_p(codes), _p(scale), _p(zero), C.c_int64(codes.size // D),
                                  C.c_int32(D), _p(out))
    if rc:
        raise ValueError(f"lvo_dequantize_rows failed: {rc}")
    return out


def attn_qkv8(scales, radii, q, k, v, sm_scale, n_sink=0, q_scales=None, bits=8, bh_range=None,
              mode=0):
    """fp64 windowed attention on Q, K, V quantised per token row to `bits` bits and
    dequantised (Section 4).  Shapes as attn(); returns [B,H,Lq,D]."""
    s, r = _i32(scales), _rtab(scales, radii)
    qb, qe, Lq = _qrange(scales, q_scales)
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    code = _dtype_code(q)
    assert _dtype_code(k) == code and _dtype_code(v) == code
    B, H, lq, D = q.shape
    assert lq == Lq and k.shape == (B, H, seq_len(scales), D) and v.shape == k.shape
    b0, b1 = (0, B * H) if bh_range is None else bh_range
    out = np.zeros((B, H, Lq, D), dtype=np.float64)
    rc = _L().lvo_attn_qkv8(C.c_int32(len(s)), _p(s), _p(r), C.c_int32(n_sink), C.c_int32(mode), C.c_int32(qb),
                            C.c_int32(qe), _p(q), _p(k), _p(v), C.c_int32(code), C.c_int32(B),
                            C.c_int32(H), C.c_int32(D), C.c_double(sm_scale), C.c_int32(bits),
                            C.c_int64(b0), C.c_int64(b1), _p(out))
    if rc:
        raise ValueError(f"lvo_attn_qkv8 failed: {rc}")
    return out


def num_threads():
    return int(_L().lvo_num_threads())
