"""Pins of the oracle's QKV8 functions (paper Section 4: min-max quantiser with dynamic
parameters) against things other than themselves (CPU only): hand-derived rows, closed
forms and bounds, an independent numpy statement of the quantiser, and special cases in
which quantised attention reduces to plain attention."""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantizer_rows.txt")


def _golden_rows():
    rows, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":")
        vals = [float(x) for x in val.split()]
        if key == "row":
            cur = {"row": vals}
            rows.append(cur)
        else:
            cur[key] = vals
    return rows


def test_hand_derived_rows():
    for g in _golden_rows():
        x = np.array([g["row"]], dtype=np.float32)
        codes, s, z = oracle.quantize_rows(x)
        assert codes[0].tolist() == [int(c) for c in g["codes"]], g
        assert z[0] == g["zero"][0]
        assert s[0] == float(np.float32(g["scale_times_127"][0]) / np.float32(127)), g
        back = oracle.dequantize_rows(codes, s, z)
        assert np.all(np.abs(back[0] - x[0]) <= s[0] / 2 + 1e-6 * max(1.0, np.abs(x).max()))


def _numpy_quantiser(x, bits):
    """independent statement in numpy binary32: same formula, numpy's own rounding"""
    x = x.astype(np.float32)
    qmax = np.float32(2 ** (bits - 1) - 1)
    mx, mn = x.max(axis=-1, keepdims=True), x.min(axis=-1, keepdims=True)
    z = (mx + mn) * np.float32(0.5)
    s = ((mx - mn) * np.float32(0.5)) / qmax
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(s > 0, (x - z) / s, np.float32(0))
    t = np.clip(t, -np.float32(2 ** (bits - 1)), qmax)
    return np.rint(t).astype(np.int32), s[..., 0].astype(np.float64), z[..., 0].astype(np.float64)


@settings(max_examples=60, deadline=None)
@given(seed=st.integers(0, 10 ** 6), rows=st.integers(1, 5), D=st.sampled_from([1, 2, 7, 64]),
       bits=st.sampled_from([4, 6, 8]), spread=st.sampled_from([1e-3, 1.0, 300.0]))
def test_numpy_statement_agrees(seed, rows, D, bits, spread):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((rows, D)) * spread + g.standard_normal((rows, 1))).astype(np.float32)
    codes, s, z = oracle.quantize_rows(x, bits)
    c2, s2, z2 = _numpy_quantiser(x, bits)
    assert np.array_equal(codes, c2) and np.array_equal(s, s2) and np.array_equal(z, z2)


def test_code_range_extremes_and_round_trip_bound():
    g = np.random.default_rng(5)
    x = g.standard_normal((200, 64)).astype(np.float32) * 3
    for bits in (4, 8):
        qmax = 2 ** (bits - 1) - 1
        codes, s, z = oracle.quantize_rows(x, bits)
        assert codes.min() >= -qmax - 1 and codes.max() <= qmax
        # the row's maximum and minimum sit half a range from z: codes +qmax and -qmax
        assert np.all(codes[np.arange(200), x.argmax(axis=1)] == qmax)
        assert np.all(codes[np.arange(200), x.argmin(axis=1)] == -qmax)
        back = oracle.dequantize_rows(codes, s, z)
        assert np.all(np.abs(back - x) <= s[:, None] * 0.5 * (1 + 1e-5) + 1e-6)
        # finer codes, smaller error
        if bits == 8:
            err8 = np.abs(back - x).max()
        else:
            err4 = np.abs(back - x).max()
    assert err8 < err4 / 8


def test_inputs_of_any_dtype_quantise_alike():
    g = np.random.default_rng(2)
    import torch
    xb = torch.from_numpy(g.standard_normal((7, 64)).astype(np.float32)).to(torch.bfloat16)
    bits16 = workloads.bf16_bits(xb)
    as32 = xb.float().numpy()
    a = oracle.quantize_rows(bits16)
    b = oracle.quantize_rows(as32)
    c = oracle.quantize_rows(as32.astype(np.float64))
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    for u, v in zip(a, c):
        assert np.array_equal(u, v)


def test_quantised_attention_of_exactly_representable_inputs_is_plain_attention():
    """rows whose values are z + s * integer codes, with the extremes present, survive the
    quantiser unchanged: QKV8 attention then equals the unquantised oracle"""
    scales = (1, 2, 3, 4)
    g = np.random.default_rng(9)

    def grid(shape):
        c = g.integers(-127, 128, size=shape).astype(np.float32)
        c[..., 0], c[..., 1] = -127, 127
        return c / np.float32(32)           # s = 1/32 exactly, z = 0
    q, k, v = grid((1, 2, 30, 64)), grid((1, 2, 30, 64)), grid((1, 2, 30, 64))
    want = oracle.attn(scales, [1] * 4, q, k, v, 0.125)
    got = oracle.attn_qkv8(scales, [1] * 4, q, k, v, 0.125)
    assert np.abs(want - got).max() < 1e-12


def test_quantised_attention_is_attention_of_the_dequantised_tensors_and_close_to_plain():
    w = workloads.get("tiny_f32")
    q, k, v = [t.numpy() for t in workloads.make_qkv(w.scales, 2, 2, 64, "f32", 4)]
    got = oracle.attn_qkv8(w.scales, [1] * 4, q, k, v, 0.125)
    deq = [oracle.dequantize_rows(*oracle.quantize_rows(t)) for t in (q, k, v)]
    want = oracle.attn(w.scales, [1] * 4, *deq, 0.125)
    assert np.array_equal(got, want)
    plain = oracle.attn(w.scales, [1] * 4, q, k, v, 0.125)
    err = np.abs(got - plain).max()
    assert 1e-5 < err < 5e-2          # 8 bits: visible, small
    coarse = oracle.attn_qkv8(w.scales, [1] * 4, q, k, v, 0.125, bits=4)
    assert np.abs(coarse - plain).max() > 4 * err


def test_constant_value_rows_are_exact():
    scales = (1, 2, 3)
    q = np.random.default_rng(1).standard_normal((1, 1, 14, 64)).astype(np.float32)
    k = np.random.default_rng(2).standard_normal((1, 1, 14, 64)).astype(np.float32)
    v = np.repeat(np.arange(1, 15, dtype=np.float32)[None, None, :, None], 64, axis=3)
    out = oracle.attn_qkv8(scales, [-1] * 3, q, k, v, 0.125)
    # every V row is constant: it dequantises exactly (to its zero point), so each output row
    # is constant too, lies between the smallest and largest value it can see, and the first
    # token (which sees only itself) returns V[0] = 1
    assert np.abs(out - out[..., :1]).max() < 1e-12 and np.all(out[0, 0, 0] == 1.0)
    assert np.all(out[0, 0, 1:5] >= 1.0) and np.all(out[0, 0, 1:5] <= 5.0)
