"""Independent brute-force statement of the method in Python/numpy loops.

Used only to pin the C oracle on small inputs.  Written from the definition
(Section 2 of the paper plus the readings listed in the design notes), with
its own token decoding, its own predicate and a dense masked softmax.
"""
import numpy as np


def decode_tokens(scales):
    """list of (scale index, row, col) for every token, row-major per scale."""
    out = []
    for k, s in enumerate(scales):
        for y in range(s):
            for x in range(s):
                out.append((k, y, x))
    return out


def centre(c, s_from, s_to):
    # centre-aligned nearest cell: pixel centre (c + 1/2) / s_from mapped to s_to cells
    from fractions import Fraction
    pos = (Fraction(c) + Fraction(1, 2)) / s_from * s_to
    return int(pos // 1)


def dense_mask(scales, radii, n_sink=0, q_scales=None):
    toks = decode_tokens(scales)
    qb, qe = (0, len(scales)) if q_scales is None else q_scales
    qs = [i for i, (k, _, _) in enumerate(toks) if qb <= k < qe]
    m = np.zeros((len(qs), len(toks)), dtype=bool)
    for r, qi in enumerate(qs):
        k, y, x = toks[qi]
        for t, (j, yy, xx) in enumerate(toks):
            if j > k:
                continue
            # one radius per key scale, or a table [query scale][key scale]
            rad = radii[k][j] if hasattr(radii[0], "__len__") else radii[j]
            if j < n_sink or rad < 0:
                m[r, t] = True
                continue
            cy, cx = centre(y, scales[k], scales[j]), centre(x, scales[k], scales[j])
            m[r, t] = max(abs(yy - cy), abs(xx - cx)) <= rad
    return m


def masked_attention(q, k, v, mask, sm_scale):
    """q [Lq,D], k,v [L,D] float64, mask [Lq,L] bool -> (out [Lq,D], probs [Lq,L])."""
    z = sm_scale * (q @ k.T)
    z = np.where(mask, z, -np.inf)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    p = e / e.sum(axis=1, keepdims=True)
    return p @ v, p


def dense_mask_band(scales, radii, n_sink=0, q_scales=None):
    """The band reading, from its definition: parts of the flattened attention map (the first
    spans the first three key scales, every later key scale is a part) and, per part, the
    columns within the radius of the part's diagonal.  Exact fractions for the diagonal."""
    from fractions import Fraction
    K = len(scales)
    off = [0]
    for s in scales:
        off.append(off[-1] + s * s)
    qb, qe = (0, K) if q_scales is None else q_scales
    rows = []
    for k in range(qb, qe):
        m = scales[k] * scales[k]
        # parts as (first key scale, last key scale)
        parts = [(0, min(2, k))] + [(j, j) for j in range(3, k + 1)]
        for i in range(m):
            row = np.zeros(off[-1], dtype=bool)
            for first, last in parts:
                n = off[last + 1] - off[first]
                rad = radii[k][last] if hasattr(radii[0], "__len__") else radii[last]
                if last < n_sink or rad < 0:
                    row[off[first]:off[last + 1]] = True
                    continue
                diag = int((Fraction(2 * i + 1, 2 * m) * n) // 1)
                for c in range(n):
                    if abs(c - diag) <= rad:
                        row[off[first] + c] = True
            rows.append(row)
    return np.array(rows)
