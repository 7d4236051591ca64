"""Rank-r factors of the cached counterpart feature (oracle side, fp64 numpy).

Random Projection (Sec. "Random Projection (RP) for Low-Rank Feature"):
    G = Q^T C,  Q in R^{M x r},  Q_ij ~ N(0, 1/r)   (variance 1/r).
Restoration matrix by linear least squares (Eq. "lstsq", applied to the cached
feature as App. "Construction of W_r^o" prescribes):
    W = argmin_W || G^T W^T - C^T ||_F  =  C G^T (G G^T)^{-1}.
So W G is the orthogonal projection of the rows of C onto rowspace(G).

The standard-normal draws are an input (`z`), so that no random generator is
part of the method's arithmetic.
"""
from __future__ import annotations

import numpy as np


def random_projection_matrix(z: np.ndarray, r: int) -> np.ndarray:
    """Q = z / sqrt(r) for z:[M,r] standard normal draws  =>  Var(Q_ij) = 1/r."""
    z = np.asarray(z, np.float64)
    assert z.shape[1] == r
    return z / np.sqrt(float(r))


def project(Q: np.ndarray, C: np.ndarray) -> np.ndarray:
    """G = Q^T C, [r,d]."""
    return np.asarray(Q, np.float64).T @ np.asarray(C, np.float64)


def restoration_matrix(G: np.ndarray, C: np.ndarray, ridge: float = 0.0) -> np.ndarray:
    """W:[M,r] minimising ||W G - C||_F through the normal equations.

    Cholesky of the r x r Gram matrix in fp64; `ridge` (relative to trace/r) is only for
    r > rank(C), where the Gram matrix is singular and the projection is still well defined.
    """
    G = np.asarray(G, np.float64)
    C = np.asarray(C, np.float64)
    r = G.shape[0]
    gram = G @ G.T
    if ridge:
        gram = gram + np.eye(r) * (ridge * np.trace(gram) / r)
    L = np.linalg.cholesky(gram)
    rhs = G @ C.T                                   # [r, M]
    t = np.linalg.solve(L, rhs)                     # L t = rhs
    Wt = np.linalg.solve(L.T, t)                    # L^T W^T = t
    return Wt.T


def cache_factors(C: np.ndarray, z: np.ndarray, ridge: float = 0.0):
    """(W_c [M,r] fp32, G_c [r,d] fp32) for cached feature C:[M,d] and draws z:[M,r].

    W is solved against the fp64 G and both are rounded to fp32 afterwards."""
    r = z.shape[1]
    Q = random_projection_matrix(z, r)
    G = project(Q, C)
    W = restoration_matrix(G, C, ridge)
    return W.astype(np.float32), G.astype(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bfloat16 precision, returned as fp32."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def stored_factors(C: np.ndarray, Q: np.ndarray, ridge: float = 0.0, bf16: bool = False):
    """(W_c, G_c) when the factors are kept in the storage type of the cache.

    G_c = store(Q^T C) is what the restoration W_c G_c will later be computed from, so the
    least-squares problem of Eq. "lstsq" is posed against that stored G_c (not the unrounded
    product): W_c = store(C G_c^T (G_c G_c^T)^{-1}).  store() rounds to bf16 or to fp32."""
    store = round_bf16 if bf16 else (lambda a: np.asarray(a, np.float32))
    G = store(project(Q, C))
    W = restoration_matrix(G, C, ridge)
    return store(W), G


def energy_rank(C: np.ndarray, alpha: float) -> int:
    """Smallest r with eta_r = sum_{i<=r} sigma_i^2 / sum_i sigma_i^2 >= alpha (Eq. "low_rank_percent")."""
    sv = np.linalg.svd(np.asarray(C, np.float64), compute_uv=False)
    eta = np.cumsum(sv ** 2) / np.sum(sv ** 2)
    return int(np.searchsorted(eta, alpha - 1e-15) + 1)
