"""Pins of the oracle's window calibration (paper Section 2: R_w = values inside the window
over values of the part; the radius is raised from 0 until that ratio is at least R_0; with
R_0 = 1 the whole part is kept) against things other than itself: hand-placed mass at known distances,
the closed form for a uniform same-scale part, an independent brute force, and invariants."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
import workloads
from _bruteforce import decode_tokens, dense_mask

# centres of query cells in a coarser key scale, from the worked example of the method on
# scales (1, 2, 3, 4) (tests/golden/tiny_r1_rows.txt, last line of its header):
# side 4 -> side 3: 0,1,1,2; side 4 -> side 2: 0,0,1,1
CENTRE_4_TO_3 = (0, 1, 1, 2)
CENTRE_4_TO_2 = (0, 0, 1, 1)
TINY = (1, 2, 3, 4)
OFF = (0, 1, 5, 14)


def _empty_map(scales, H=1, N=1):
    L = oracle.seq_len(scales)
    return np.zeros((N, H, L, L), dtype=np.float64)


def test_golden_header_names_the_centres():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_r1_rows.txt")
    text = open(path).read()
    assert "0,1,1,2" in text.replace(" ", "") and "0,0,1,1" in text.replace(" ", "")


@pytest.mark.parametrize("dist", [0, 1, 2])
def test_mass_at_a_known_distance_from_the_centre(dist):
    """All of part (query side 4, key side 3)'s mass sits `dist` rows below the centre key of
    each query (where that cell exists): the window has to reach exactly that far."""
    p = _empty_map(TINY)
    placed = 0
    for qy in range(4):
        for qx in range(4):
            cy, cx = CENTRE_4_TO_3[qy], CENTRE_4_TO_3[qx]
            if cy + dist < 3:
                p[0, 0, OFF[3] + qy * 4 + qx, OFF[2] + (cy + dist) * 3 + cx] = 0.25
                placed += 1
    assert placed > 0
    r = oracle.calibrate(TINY, p, 0.95)
    assert r[0, 3, 2] == dist
    assert r[0, 3, 0] == 0 and r[0, 3, 1] == 0          # parts without mass
    assert (r[0][np.triu_indices(4, 1)] == -1).all()    # a query never sees a later scale


def test_split_mass_between_centre_and_ring():
    """A fraction f on the centre key and the rest at distance 1 (part: query side 4, key
    side 2): radius 0 while f >= R_0, else 1 ("until R_w reaches R_0": equality counts; the
    tie case uses values that are exact in binary)."""
    for f, r0, want in [(0.96, 0.95, 0), (0.75, 0.75, 0), (0.90, 0.95, 1), (0.5, 0.6, 1), (0.7, 0.6, 0)]:
        p = _empty_map(TINY)
        for qy in range(4):
            for qx in range(4):
                cy, cx = CENTRE_4_TO_2[qy], CENTRE_4_TO_2[qx]
                q = OFF[3] + qy * 4 + qx
                p[0, 0, q, OFF[1] + cy * 2 + cx] = f
                p[0, 0, q, OFF[1] + (1 - cy) * 2 + cx] = 1.0 - f     # the other row: distance 1
        assert oracle.calibrate(TINY, p, r0)[0, 3, 1] == want, (f, r0)


@pytest.mark.parametrize("s", [4, 7, 16])
@pytest.mark.parametrize("r0", [0.3, 0.6, 0.9, 1.0])
def test_uniform_same_scale_part_closed_form(s, r0):
    """Uniform values over a same-scale part (centre = the query's own cell): the window of
    radius r holds (sum over c of clipped window lengths)^2 of the s^4 values."""
    scales = (s,)
    p = np.full((1, 1, s * s, s * s), 1.0 / (s * s))
    want = None
    for r in range(s):
        n = sum(min(c + r, s - 1) - max(c - r, 0) + 1 for c in range(s))
        if n * n >= r0 * s ** 4 * (1 - 1e-15):
            want = r
            break
    got = oracle.calibrate(scales, p, r0)[0, 0, 0]
    assert got == want


def _bruteforce_radii(scales, p, r0):
    """Independent statement: for each radius the brute-force mask of that radius selects the
    window; masses are summed in numpy."""
    K = len(scales)
    toks = decode_tokens(scales)
    sc = np.array([k for k, _, _ in toks])
    N, H = p.shape[:2]
    out = -np.ones((H, K, K), dtype=np.int64)
    masks = [dense_mask(scales, [r] * K) for r in range(max(scales))]
    for h in range(H):
        for k in range(K):
            for j in range(k + 1):
                rows, cols = np.nonzero(sc == k)[0], np.nonzero(sc == j)[0]
                part = p[:, h][:, rows][:, :, cols].sum(axis=0)
                total = part.sum()
                for r in range(scales[j]):
                    inside = (part * masks[r][np.ix_(rows, cols)]).sum()
                    if total == 0 or inside / total >= r0:
                        out[h, k, j] = r
                        break
    return out


@settings(max_examples=25, deadline=None)
@given(scales=st.lists(st.integers(1, 6), min_size=1, max_size=4),
       r0=st.sampled_from([0.5, 0.8, 0.95, 1.0]), seed=st.integers(0, 10 ** 6))
def test_bruteforce_random_maps(scales, r0, seed):
    p = workloads.make_attn_map(scales, 2, 2, seed).numpy().astype(np.float64)
    got, mass = oracle.calibrate(scales, p, r0, with_mass=True)
    want = _bruteforce_radii(scales, p, r0)
    # a ratio within rounding of the threshold may fall either way: there both are valid
    K = len(scales)
    for h in range(2):
        for k in range(K):
            for j in range(k + 1):
                if got[h, k, j] != want[h, k, j]:
                    total = mass[h, k, j, scales[j] - 1]
                    lo = min(got[h, k, j], want[h, k, j])
                    assert abs(mass[h, k, j, lo] / total - r0) < 1e-12, (h, k, j)
    assert (got[:, np.triu_indices(K, 1)[0], np.triu_indices(K, 1)[1]] == -1).all()


def test_invariants():
    scales = (1, 2, 3, 5, 8)
    p = workloads.make_attn_map(scales, 3, 2, 11).numpy().astype(np.float64)
    base = oracle.calibrate(scales, p, 0.9)
    # a larger threshold never shrinks a window; threshold 1 keeps every non-zero value
    prev = None
    for r0 in (0.5, 0.7, 0.9, 0.99, 1.0):
        r = oracle.calibrate(scales, p, r0)
        if prev is not None:
            assert (r >= prev).all()
        prev = r
    full, mass = oracle.calibrate(scales, p, 1.0, with_mass=True)
    for k in range(5):
        for j in range(k + 1):
            assert mass[0, k, j, full[0, k, j]] == mass[0, k, j, scales[j] - 1]
    # the map's overall scale does not matter; samples add up
    assert (oracle.calibrate(scales, 0.25 * p, 0.9) == base).all()
    assert (oracle.calibrate(scales, p.sum(axis=0, keepdims=True), 0.9) == base).all()
    # mass within the window grows with the radius and ends at the part's sum (rows sum to 1)
    _, m = oracle.calibrate(scales, p, 0.9, with_mass=True)
    assert (np.diff(m, axis=-1) >= -1e-15).all()
    per_row_total = m[0, 4, :, :].max(axis=-1).sum()     # query scale 4 (64 rows), all parts
    assert abs(per_row_total - 3 * 64) < 1e-4            # three samples of 64 rows summing to one (float32 maps)
