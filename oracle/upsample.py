"""Up-sampling of a cached token map to the next scale (oracle side, test infrastructure).

Eq. "upcache": the cached feature of scale k-1 is brought to the token grid of scale k before it
fills the pruned rows.  The paper does not name the interpolation; the reading used here is
bilinear interpolation with half-pixel centres and edge clamping (the usual image-resize
convention).  It acts on the token axis only, hence linearly:  Up(W G) = Up(W) G, which is what
lets the rank-r form of the cache be up-sampled on its thin factor W alone.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def _axis_taps(n_src: int, n_dst: int):
    """For every destination index: (i0, i1, w1) with value = (1-w1)*src[i0] + w1*src[i1].

    Source coordinate of destination centre y: (y + 1/2) * n_src / n_dst - 1/2, clamped below at 0;
    i1 is clamped to the last source index.  Exact rational arithmetic."""
    taps = []
    for y in range(n_dst):
        s = Fraction(2 * y + 1, 2) * Fraction(n_src, n_dst) - Fraction(1, 2)
        if s < 0:
            s = Fraction(0)
        i0 = int(s)                     # floor, s >= 0
        if i0 > n_src - 1:
            i0 = n_src - 1
        i1 = min(i0 + 1, n_src - 1)
        taps.append((i0, i1, float(s - i0)))
    return taps


def upsample_tokens(src: np.ndarray, hs: int, ws: int, hd: int, wd: int) -> np.ndarray:
    """src:[hs*ws, c] row-major token grid -> [hd*wd, c], fp64 arithmetic, returned as fp64."""
    src = np.asarray(src, np.float64)
    assert src.shape[0] == hs * ws
    c = src.shape[1]
    g = src.reshape(hs, ws, c)
    ty, tx = _axis_taps(hs, hd), _axis_taps(ws, wd)
    out = np.empty((hd, wd, c), np.float64)
    for y, (y0, y1, wy) in enumerate(ty):
        for x, (x0, x1, wx) in enumerate(tx):
            top = (1.0 - wx) * g[y0, x0] + wx * g[y0, x1]
            bot = (1.0 - wx) * g[y1, x0] + wx * g[y1, x1]
            out[y, x] = (1.0 - wy) * top + wy * bot
    return out.reshape(hd * wd, c)
