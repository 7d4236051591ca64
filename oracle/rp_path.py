"""Random-projection input path of the fidelity-refinement stage (oracle side, test infrastructure).

Follows Alg. "FasterVAR" as printed: the block receives the r-row feature F^_r = Q^T F~
(Sec. "Random Projection (RP) for Low-Rank Feature"), its r output rows are taken as the rows of
the full output at the chosen indices I, and every other row is the cached counterpart row
(Eq. "redefine").  The paper gives no correspondence between the r mixed rows and the r indices;
the reading used here is: output row j goes to the j-th smallest index of I.
"""
from __future__ import annotations

import numpy as np

from . import block_forward, scores, topk
from .factors import project, round_bf16


def rp_input(Q: np.ndarray, X: np.ndarray, bf16: bool = False) -> np.ndarray:
    """F^_r = Q^T X for Q:[M,r], X:[M,d], fp64 products and sums, rounded to the storage type."""
    F = project(Q, X)
    return round_bf16(F) if bf16 else F.astype(np.float32)


def cache_fill(y_keep: np.ndarray, keep: np.ndarray, C: np.ndarray) -> np.ndarray:
    """Eq. "redefine": row i of the result is y_keep[j] if i == keep[j], else the cached row C[i]."""
    Y = np.array(C, dtype=np.float32, copy=True)
    for j, i in enumerate(np.asarray(keep)):
        Y[int(i)] = y_keep[j]
    return Y


def rp_step(x, Q, C, w, H, Kc, Vc, length, bf16=False, eps=1e-6, scale=None):
    """One block of the fidelity-refinement stage as in Alg. "FasterVAR" for one sample.

    x:[M,d] block input, Q:[M,r], C:[M,d] cached counterpart (already at M rows).
    Returns dict(f_r, idx_keep, idx_drop, y_keep, y); appends r K/V rows to Kc,Vc in place."""
    r = Q.shape[1]
    f_r = rp_input(Q, x, bf16)
    y_keep = block_forward(f_r, w, H, Kc, Vc, length, eps, scale)
    keep, drop = topk(scores(x), r)
    return dict(f_r=f_r, idx_keep=keep, idx_drop=drop, y_keep=y_keep,
                y=cache_fill(y_keep, keep, C))
