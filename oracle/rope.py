"""CPU oracle: rotary position embedding of tree queries and keys.  TEST INFRASTRUCTURE ONLY.

The paper verifies a whole draft tree in one forward pass of the target model (Sec. 1); a node
at depth d of sequence b then sits at position id prefix_len[b] + d (what tree_pack writes), and
a rotary-embedding target model rotates that node's query and key by its position before
attention.  The rotation itself is the published RoFormer definition, written out in binary64:

    pair i of a head (i = 0 .. rotary_dim/2 - 1) is rotated by the angle
        pos * base ** (-2 i / rotary_dim)
    (x, y) -> (x cos - y sin,  x sin + y cos)

    half-split pairing:   (x, y) = (v[i], v[i + rotary_dim/2])
    interleaved pairing:  (x, y) = (v[2 i], v[2 i + 1])

Elements past rotary_dim are left alone.
"""
from __future__ import annotations

import numpy as np

HALF_SPLIT, INTERLEAVED = 0, 1


def rope(x, position, base=10000.0, rotary_dim=None, pairing=HALF_SPLIT):
    """x: [N, H, D] (any float dtype; taken as binary64), position: [N] ints.  Returns float64."""
    x = np.asarray(x, np.float64)
    N, H, D = x.shape
    rot = D if rotary_dim is None else int(rotary_dim)
    if rot % 2 or not (0 < rot <= D):
        raise ValueError("rotary_dim must be even and at most the head size")
    half = rot // 2
    out = x.copy()
    for n in range(N):
        pos = float(int(position[n]))
        for i in range(half):
            angle = pos * float(base) ** (-2.0 * i / rot)
            c, s = np.cos(angle), np.sin(angle)
            ix, iy = (i, i + half) if pairing == HALF_SPLIT else (2 * i, 2 * i + 1)
            for h in range(H):
                a, b = x[n, h, ix], x[n, h, iy]
                out[n, h, ix] = a * c - b * s
                out[n, h, iy] = a * s + b * c
    return out
