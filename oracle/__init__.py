"""CPU oracle (test infrastructure, not a product path).

`fvar_oracle.c` holds the plain loops; this module compiles it with gcc, loads
it through ctypes and wraps it for numpy arrays.  `factors.py` builds the
rank-r factors of the cached feature in fp64 numpy and `rp_path.py` the random-projection
input variant of the fidelity-refinement stage.  Nothing here imports or
is imported by the GPU package; only tests, the smoke check and the
benchmark's CPU-baseline leg use it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fvar_oracle.c")
_LIB = os.path.join(_HERE, "libfvar_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
        "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")]


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class BlockWeights:
    """fp32 weights of one block, `out,in` layout; None = no affine / no bias."""
    w_qkv: np.ndarray
    w_o: np.ndarray
    w_fc1: np.ndarray
    w_fc2: np.ndarray
    ln1_g: Optional[np.ndarray] = None
    ln1_b: Optional[np.ndarray] = None
    b_qkv: Optional[np.ndarray] = None
    b_o: Optional[np.ndarray] = None
    ln2_g: Optional[np.ndarray] = None
    ln2_b: Optional[np.ndarray] = None
    b_fc1: Optional[np.ndarray] = None
    b_fc2: Optional[np.ndarray] = None

    def _c(self):
        keep = {}
        s = _Weights()
        for name, _ in _Weights._fields_:
            v = getattr(self, name)
            if v is not None:
                v = _f32(v)
                keep[name] = v
                setattr(s, name, v.ctypes.data)
            else:
                setattr(s, name, None)
        return s, keep


def scores(x: np.ndarray) -> np.ndarray:
    """Row energies s_i = sum_j x_ij^2 of one sample, x:[M,d] -> [M]."""
    x = _f32(x)
    M, d = x.shape
    s = np.empty(M, np.float32)
    _load().fvo_scores(_p(x), M, d, _p(s))
    return s


def importance(s: np.ndarray) -> np.ndarray:
    s = _f32(s)
    P = np.empty_like(s)
    _load().fvo_importance(_p(s), s.shape[0], _p(P))
    return P


def topk(s: np.ndarray, k: int):
    """(idx_keep ascending, idx_drop ascending) of the k largest scores, ties -> lower index."""
    s = _f32(s)
    M = s.shape[0]
    assert 0 <= k <= M
    keep = np.empty(k, np.int32)
    drop = np.empty(M - k, np.int32)
    _load().fvo_topk(_p(s), M, k, _p(keep), _p(drop))
    return keep, drop


def gather_rows(x: np.ndarray, idx: np.ndarray) -> np.ndarray:
    x = _f32(x)
    idx = np.ascontiguousarray(idx, np.int32)
    out = np.empty((idx.shape[0], x.shape[1]), np.float32)
    _load().fvo_gather_rows(_p(x), _p(idx), idx.shape[0], x.shape[1], _p(out))
    return out


def layernorm(x, gamma=None, beta=None, eps=1e-6) -> np.ndarray:
    x = _f32(x)
    rows, d = x.shape
    g = None if gamma is None else _f32(gamma)
    b = None if beta is None else _f32(beta)
    out = np.empty_like(x)
    _load().fvo_layernorm(_p(x), rows, d, _p(g), _p(b), C.c_float(eps), _p(out))
    return out


def linear(x, W, bias=None) -> np.ndarray:
    x = _f32(x)
    W = _f32(W)
    rows, cin = x.shape
    cout = W.shape[0]
    assert W.shape[1] == cin
    b = None if bias is None else _f32(bias)
    y = np.empty((rows, cout), np.float32)
    _load().fvo_linear(_p(x), rows, cin, _p(W), _p(b), cout, _p(y))
    return y


def gelu_tanh(x) -> np.ndarray:
    y = _f32(x).copy()
    _load().fvo_gelu_tanh(_p(y), C.c_size_t(y.size))
    return y


def attention(q, K, V, scale=None, mask=None, want_stats=False):
    """q:[n,H,Dh], K,V:[L,H,Dh] -> o:[n,H,Dh] (and lse, prob row sums [n,H])."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    n, H, Dh = q.shape
    L = K.shape[0]
    assert K.shape == (L, H, Dh) and V.shape == (L, H, Dh)
    if scale is None:
        scale = 1.0 / np.sqrt(Dh)
    m = None if mask is None else np.ascontiguousarray(mask, np.uint8)
    o = np.empty_like(q)
    lse = np.empty((n, H), np.float32)
    ps = np.empty((n, H), np.float32)
    _load().fvo_attention(_p(q), _p(K), _p(V), n, L, H, Dh, C.c_float(scale), _p(m), _p(o),
                          _p(lse), _p(ps))
    return (o, lse, ps) if want_stats else o


def block_forward(x, w: BlockWeights, H: int, Kc: np.ndarray, Vc: np.ndarray, length: int,
                  eps=1e-6, scale=None) -> np.ndarray:
    """phi on the n rows of one sample; appends n K/V rows to Kc,Vc ([Lcap,H,Dh]) IN PLACE."""
    x = _f32(x)
    n, d = x.shape
    Dh = d // H
    F = w.w_fc1.shape[0]
    assert Kc.dtype == np.float32 and Vc.dtype == np.float32
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    assert Kc.shape[0] >= length + n and Kc.shape[1:] == (H, Dh)
    if scale is None:
        scale = 1.0 / np.sqrt(Dh)
    ws, keep = w._c()
    y = np.empty_like(x)
    _load().fvo_block_forward(_p(x), n, d, H, Dh, F, C.byref(ws), C.c_float(eps), C.c_float(scale),
                              _p(Kc), _p(Vc), length, _p(y))
    del keep
    return y


def lowrank_fill(y_keep, keep, drop, M: int, Wc, Gc) -> np.ndarray:
    y_keep, Wc, Gc = _f32(y_keep), _f32(Wc), _f32(Gc)
    keep = np.ascontiguousarray(keep, np.int32)
    drop = np.ascontiguousarray(drop, np.int32)
    k, d = y_keep.shape if y_keep.size else (0, Gc.shape[1])
    r = Gc.shape[0]
    assert Wc.shape == (M, r) and keep.shape[0] == k and drop.shape[0] == M - k
    Y = np.empty((M, d), np.float32)
    _load().fvo_lowrank_fill(_p(y_keep), _p(keep), _p(drop), M, k, d, r, _p(Wc), _p(Gc), _p(Y))
    return Y


def pruned_step(x, k: int, w: BlockWeights, H: int, Kc, Vc, length: int, Wc, Gc, eps=1e-6,
                scale=None):
    """score -> select -> gather -> phi -> fill for one sample.

    Returns dict(scores, idx_keep, idx_drop, y_keep, y); appends k rows to Kc,Vc in place."""
    x, Wc, Gc = _f32(x), _f32(Wc), _f32(Gc)
    M, d = x.shape
    Dh = d // H
    F = w.w_fc1.shape[0]
    r = Gc.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(Dh)
    ws, hold = w._c()
    s = np.empty(M, np.float32)
    keep = np.empty(k, np.int32)
    drop = np.empty(M - k, np.int32)
    y_keep = np.empty((k, d), np.float32)
    Y = np.empty((M, d), np.float32)
    _load().fvo_pruned_step(_p(x), M, k, d, H, Dh, F, C.byref(ws), C.c_float(eps), C.c_float(scale),
                            _p(Kc), _p(Vc), length, r, _p(Wc), _p(Gc), _p(s), _p(keep), _p(drop),
                            _p(y_keep), _p(Y))
    del hold
    return dict(scores=s, idx_keep=keep, idx_drop=drop, y_keep=y_keep, y=Y)


def pruned_chunk(x, k: int, ws, H: int, caches, length: int, Wc, Gc, eps=1e-6, scale=None):
    """One block CHUNK with a single selection (the paper applies its reduction per block chunk,
    Sec. "Experiments" / App. rank tables "block_chunks"): score and select on the chunk input,
    gather once, run every block of the chunk on the k compact rows (each appends its k K/V rows
    to its own cache), fill once at the end.

    ws: list of BlockWeights; caches: list of (Kc, Vc) per block, modified in place.
    Returns dict(scores, idx_keep, idx_drop, y_keep, y)."""
    x = _f32(x)
    M = x.shape[0]
    s = scores(x)
    keep, drop = topk(s, k)
    rows = gather_rows(x, keep)
    for w, (Kc, Vc) in zip(ws, caches):
        rows = block_forward(rows, w, H, Kc, Vc, length, eps, scale)
    return dict(scores=s, idx_keep=keep, idx_drop=drop, y_keep=rows,
                y=lowrank_fill(rows, keep, drop, M, Wc, Gc))


def keep_count(M: int, num: int, den: int) -> int:
    """k = ceil(M*num/den) in integer arithmetic, clamped to [1, M]."""
    k = -((-M * num) // den)
    return max(1, min(M, k))


def num_threads() -> int:
    """OpenMP threads the C loops run on."""
    return int(_load().fvo_num_threads())
