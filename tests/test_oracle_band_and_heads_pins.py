"""Pins of the oracle's band reading (paper Section 2, step (2), literal) and of its per-head
radius tables (Section 2, step (3)) against things other than the oracle (CPU only)."""
import os

import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import workloads
from _bruteforce import dense_mask, dense_mask_band, masked_attention

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tiny_band_r1_rows.txt")
BAND = 1


def _read_golden():
    rows, sums, totals = {}, None, {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#") or line == "rows:":
            continue
        if line.startswith("row_sums:"):
            sums = [int(x) for x in line.split(":")[1].split()]
        elif ":" in line:
            key, val = line.split(":")
            totals[key.strip()] = int(val)
        else:
            idx, pat = line.split()
            rows[int(idx)] = [c == "1" for c in pat.replace("|", "")]
    return rows, sums, totals


def test_band_worked_example():
    rows, sums, totals = _read_golden()
    scales = (1, 2, 3, 4)
    m = oracle.mask_dense(scales, [1] * 4, 0, mode=BAND)
    for qi, pat in rows.items():
        assert m[qi].astype(bool).tolist() == pat, f"row {qi}"
    assert m.sum(axis=1).tolist() == sums
    assert int(m.sum()) == totals["total"]
    assert int(oracle.mask_dense(scales, [1] * 4, 3, mode=BAND).sum()) == totals["total_n_sink_3"]
    assert oracle.row_counts(scales, [1] * 4, 0, mode=BAND).tolist() == sums
    rowptr, cols = oracle.index_sets(scales, [1] * 4, 0, mode=BAND)
    for qi in range(30):
        assert cols[rowptr[qi]:rowptr[qi + 1]].tolist() == np.nonzero(m[qi])[0].tolist()
        for t in (0, 3, 9, 20, 29):
            assert oracle.allowed(scales, [1] * 4, 0, qi, t, mode=BAND) == bool(m[qi, t])


def test_band_closed_forms():
    # the part of a scale with itself is square: its diagonal is the identity, so a radius-r
    # band keeps min(i, r) + min(m - 1 - i, r) + 1 columns of the scale's own m
    scales = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
    off = oracle.scale_offsets(scales)
    for r in (0, 2, 7):
        m = oracle.mask_dense(scales, [r] * 10, 0, mode=BAND)
        for k in range(3, 10):
            n = scales[k] ** 2
            own = m[off[k]:off[k + 1], off[k]:off[k + 1]]
            want = [min(i, r) + min(n - 1 - i, r) + 1 for i in range(n)]
            assert own.sum(axis=1).tolist() == want
            assert all(own[i, i] for i in range(n))
        # never a key of a later scale; radius 0 keeps one column per part
        assert not np.triu(np.ones((10, 10), dtype=bool), 1)[
            np.repeat(np.arange(10), [s * s for s in scales])][:, np.repeat(np.arange(10), [s * s for s in scales])][m.astype(bool)].any()
        if r == 0:
            parts = [1 if k < 3 else k - 1 for k in range(10)]
            assert m.sum(axis=1).tolist() == np.repeat(parts, [s * s for s in scales]).tolist()
    # a radius that covers every part gives the dense block-causal mask
    dense = oracle.mask_dense(scales, [-1] * 10, 0)
    assert np.array_equal(oracle.mask_dense(scales, [700] * 10, 0, mode=BAND), dense)
    assert np.array_equal(oracle.mask_dense(scales, [-1] * 10, 0, mode=BAND), dense)


@settings(max_examples=40, deadline=None)
@given(scales=st.lists(st.integers(1, 6), min_size=1, max_size=6), seed=st.integers(0, 10 ** 6),
       n_sink=st.integers(0, 4), kv_step=st.booleans(), table=st.booleans())
def test_band_bruteforce(scales, seed, n_sink, kv_step, table):
    g = np.random.default_rng(seed)
    K = len(scales)
    n_sink = min(n_sink, K)
    radii = g.integers(-1, 9, size=(K, K)).tolist() if table else g.integers(-1, 9, size=K).tolist()
    q_scales = (K - 1, K) if kv_step else None
    want = dense_mask_band(scales, radii, n_sink, q_scales)
    got = oracle.mask_dense(scales, radii, n_sink, q_scales, mode=BAND).astype(bool)
    assert np.array_equal(got, want)
    Lq, L = want.shape
    q, k, v = g.standard_normal((Lq, 4)), g.standard_normal((L, 4)), g.standard_normal((L, 4))
    ref, _ = masked_attention(q, k, v, want, 0.3)
    out = oracle.attn(scales, radii, q[None, None], k[None, None], v[None, None], 0.3, n_sink, q_scales, mode=BAND)
    assert np.abs(out[0, 0] - ref).max() < 1e-10


def test_the_two_readings_on_the_var_scale_list():
    """how the readings differ on the 680-token sequence: the square window of radius 2 against
    bands of the same width per part, and against bands as wide as the window's footprint"""
    scales = workloads.CONFIGS["var_d16"].scales
    win = int(oracle.row_counts(scales, [2] * 10, 0).sum())
    band_same = int(oracle.row_counts(scales, [2] * 10, 0, mode=BAND).sum())
    # (a band of width 5 keeps at most 5 columns per part, a window of radius 2 up to 25 keys)
    assert win == 72496 and band_same == int(dense_mask_band(scales, [2] * 10).sum()) and band_same < win / 3
    # the first token of every scale keeps column 0 of each part in both readings
    off = oracle.scale_offsets(scales)
    m = oracle.mask_dense(scales, [2] * 10, 0, mode=BAND)
    for k in range(10):
        assert m[off[k], 0] == 1


# ---- one radius table per head (Section 2, step (3)) ------------------------------------

def test_per_head_tables_hand_built():
    """two heads on the worked example's scales: head 0 with radius 0 everywhere (one key per
    part: 1, 2, 3, 4 keys per query of scales 1..4), head 1 dense; V = one-hot rows make the
    output read the kept set off directly"""
    scales = (1, 2, 3, 4)
    L = 30
    tabs = np.stack([np.zeros((4, 4), dtype=np.int32), -np.ones((4, 4), dtype=np.int32)])
    q = np.zeros((1, 2, L, 32))
    k = np.zeros((1, 2, L, 32))
    v = np.zeros((1, 2, L, 32))
    v[0, :, np.arange(L), np.arange(L)] = 1.0        # V[t] = e_t (first 30 of 32 dims)
    out = oracle.attn(scales, tabs, q, k, v, 1.0)
    kept0 = (out[0, 0] > 0).sum(axis=1)
    kept1 = (out[0, 1] > 0).sum(axis=1)
    assert kept0.tolist() == [1] + [2] * 4 + [3] * 9 + [4] * 16
    assert kept1.tolist() == [1] + [5] * 4 + [14] * 9 + [30] * 16
    # uniform weights over the kept keys (zero scores)
    assert np.allclose(out[0, 0].sum(axis=1), 1) and np.allclose(out[0, 1, 29, :30], 1 / 30)
    # head 0's kept keys are the centre keys of the worked example (side 4 -> side 3: 0,1,1,2)
    assert np.nonzero(out[0, 0, 29])[0].tolist() == [0, 4, 13, 29]


@settings(max_examples=20, deadline=None)
@given(scales=st.lists(st.integers(1, 5), min_size=1, max_size=4), seed=st.integers(0, 10 ** 6),
       H=st.integers(1, 3), band=st.booleans())
def test_per_head_tables_bruteforce(scales, seed, H, band):
    g = np.random.default_rng(seed)
    K = len(scales)
    L = sum(s * s for s in scales)
    tabs = g.integers(-1, 4, size=(H, K, K))
    q, k, v = (g.standard_normal((2, H, L, 8)) for _ in range(3))
    out = oracle.attn(scales, tabs, q, k, v, 0.25, mode=1 if band else 0)
    for h in range(H):
        mask = (dense_mask_band if band else dense_mask)(scales, tabs[h].tolist())
        for b in range(2):
            ref, _ = masked_attention(q[b, h], k[b, h], v[b, h], mask, 0.25)
            assert np.abs(out[b, h] - ref).max() < 1e-10
        # and it equals the single-table call for that head
        single = oracle.attn(scales, tabs[h], q[:, h:h + 1], k[:, h:h + 1], v[:, h:h + 1], 0.25,
                             mode=1 if band else 0)
        assert np.array_equal(single[:, 0], out[:, h])
