"""Pins of the oracle's band calibration (paper Section 2, step (2) read literally: the map of a
query scale is cut into parts, the first three key scales together, and in every part the
window -- a band around the part's diagonal -- grows from zero until it holds the fraction
R_0 of the part's values).  Hand-placed mass at known distances from the diagonal, the
closed form of a uniform map, an independent numpy brute force, invariants."""
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from _bruteforce import dense_mask_band

SCALES = (1, 2, 3, 4)
OFF = (0, 1, 5, 14, 30)


def _diag(i, m, n):
    """the part's diagonal at query i of m, in a part of n columns (exact)"""
    return int((Fraction(2 * i + 1, 2 * m) * n) // 1)


def _brute(scales, p, r0):
    """smallest band radius per (head, query scale, part) from dense masks built by the
    independent brute force; written to every key scale of the part"""
    K = len(scales)
    off = [0]
    for s in scales:
        off.append(off[-1] + s * s)
    N, H = p.shape[:2]
    out = -np.ones((H, K, K), dtype=np.int64)
    for k in range(K):
        parts = [(0, min(2, k))] + [(j, j) for j in range(3, k + 1)]
        for first, last in parts:
            n = off[last + 1] - off[first]
            cols = slice(off[first], off[last + 1])
            rows = slice(off[k], off[k + 1])
            for h in range(H):
                block = p[:, h, rows, cols].sum(axis=0)
                total = block.sum()
                found = n - 1
                for r in range(n):
                    m = dense_mask_band(scales, [r] * K)[rows, cols]
                    if total == 0 or block[m].sum() / total >= r0:
                        found = r
                        break
                out[h, k, first:last + 1] = found
    return out


def test_hand_placed_mass_in_the_last_part():
    """Query scale 4 (16 queries), last part = key scale 4 itself (16 columns): the diagonal is
    the identity, so mass at column i + d of row i sits at distance d."""
    p = np.zeros((1, 1, 30, 30))
    for i in range(16):
        p[0, 0, OFF[3] + i, OFF[3] + i] = 0.9                     # distance 0
        if i + 3 < 16:
            p[0, 0, OFF[3] + i, OFF[3] + i + 3] = 0.1             # distance 3
    assert oracle.calibrate_band(SCALES, p, 0.95)[0, 3, 3] == 3
    # 13 rows carry the far value: 0.9 * 16 / (0.9 * 16 + 0.1 * 13) = 0.9172...
    assert oracle.calibrate_band(SCALES, p, 0.91)[0, 3, 3] == 0
    assert oracle.calibrate_band(SCALES, p, 0.92)[0, 3, 3] == 3


def test_hand_placed_mass_in_the_merged_part():
    """The first part of query scale 4 spans key scales 1..3 (14 columns); its diagonal at row i
    is floor((2 i + 1) 14 / 32), by hand: i = 0 -> floor(14 / 32) = 0, i = 8 -> floor(238 / 32)
    = 7, i = 15 -> floor(434 / 32) = 13."""
    assert _diag(0, 16, 14) == 0 and _diag(15, 16, 14) == 13 and _diag(8, 16, 14) == 7
    p = np.zeros((1, 1, 30, 30))
    p[0, 0, OFF[3] + 0, 0 + 2] = 1.0          # row 0: column 2 of the merged part, distance 2
    p[0, 0, OFF[3] + 15, 13 - 4] = 1.0        # row 15: column 9, distance 4
    rad = oracle.calibrate_band(SCALES, p, 0.99)
    assert list(rad[0, 3]) == [4, 4, 4, 0]     # one radius for the three merged key scales; empty last part: 0
    assert oracle.calibrate_band(SCALES, p, 0.5)[0, 3, 0] == 2
    # query scales below the fourth have the single merged part, cut at their own scale
    assert list(rad[0, 1]) == [0, 0, -1, -1] and list(rad[0, 0]) == [0, -1, -1, -1]


def test_uniform_map_closed_form():
    """A uniform part: R_w(r) = sum_i |{c in [0, n): |c - diag_i| <= r}| / (m n)."""
    scales = (2, 3, 1, 5)
    p = np.ones((1, 1, 39, 39))
    got = oracle.calibrate_band(scales, p, 0.8)
    off = (0, 4, 13, 14, 39)
    k, first, last = 3, 3, 3
    m, n = 25, 25
    for r in range(n):
        kept = sum(min(n - 1, _diag(i, m, n) + r) - max(0, _diag(i, m, n) - r) + 1 for i in range(m))
        if Fraction(kept, m * n) >= Fraction(8, 10):
            break
    assert got[0, k, last] == r
    # the merged part of that query scale: key scales 0..2, 14 columns
    m, n = 25, 14
    for r2 in range(n):
        kept = sum(min(n - 1, _diag(i, m, n) + r2) - max(0, _diag(i, m, n) - r2) + 1 for i in range(m))
        if Fraction(kept, m * n) >= Fraction(8, 10):
            break
    assert list(got[0, 3, :3]) == [r2, r2, r2]
    assert off[3] - off[0] == 14


@settings(max_examples=25, deadline=None)
@given(st.lists(st.integers(1, 4), min_size=1, max_size=5), st.integers(0, 10 ** 6),
       st.sampled_from([0.5, 0.8, 0.95, 1.0]))
def test_against_the_brute_force(scales, seed, r0):
    rng = np.random.default_rng(seed)
    L = sum(s * s for s in scales)
    p = rng.random((2, 2, L, L)) ** 4          # a few large values per row
    p[rng.random(p.shape) < 0.3] = 0.0
    got = oracle.calibrate_band(tuple(scales), p, r0)
    assert (got == _brute(tuple(scales), p, r0)).all()


def test_invariants():
    rng = np.random.default_rng(3)
    scales = (1, 2, 3, 4, 2)
    L = sum(s * s for s in scales)
    p = rng.random((2, 3, L, L)) ** 3
    r_lo, r_mid, r_hi = (oracle.calibrate_band(scales, p, r0) for r0 in (0.5, 0.8, 0.99))
    assert (r_lo <= r_mid).all() and (r_mid <= r_hi).all()                       # monotone in R_0
    assert (oracle.calibrate_band(scales, 7.5 * p, 0.8) == r_mid).all()           # scale-free
    both = oracle.calibrate_band(scales, np.concatenate([p, p]), 0.8)             # samples add
    assert (both == r_mid).all()
    rad, mass = oracle.calibrate_band(scales, p, 0.8, with_mass=True)
    assert (rad == r_mid).all()
    # in-band sums grow with the radius and end at the part's sum
    assert (np.diff(mass, axis=-1) >= -1e-12).all()
    off = (0, 1, 5, 14, 30, 34)
    total = p[:, 0, off[3]:off[4], off[3]:off[4]].sum()
    assert abs(mass[0, 3, 3, -1] - total) <= 1e-9 * total
    # the radius table feeds the band predicate: every part then holds its fraction
    for h in range(3):
        m = dense_mask_band(scales, rad[h].tolist())
        for k in range(5):
            parts = [(0, min(2, k))] + [(j, j) for j in range(3, k + 1)]
            for first, last in parts:
                blk = p[:, h, off[k]:off[k + 1], off[first]:off[last + 1]].sum(axis=0)
                kept = blk[m[off[k]:off[k + 1], off[first]:off[last + 1]]].sum()
                assert kept / blk.sum() >= 0.8 - 1e-12
