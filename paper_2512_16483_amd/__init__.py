"""Python binding of libfvar.so (argument marshalling only; all compute is in the HIP kernels).

The functions carry the names of the C entry points in include/fvar.h and take torch tensors
that live on the GPU; PyTorch is used for device memory and streams only.  Loading fails loudly
when the library has not been built (python -m paper_2512_16483_amd.build)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfvar.so")

FVAR_OK, FVAR_ERR_INVALID_ARG, FVAR_ERR_UNSUPPORTED, FVAR_ERR_WORKSPACE, FVAR_ERR_HIP = range(5)
FVAR_F32, FVAR_BF16 = 0, 1

EXPORTS = (
    "fvar_create", "fvar_destroy", "fvar_last_error", "fvar_status_string", "fvar_keep_count",
    "fvar_scale_tokens", "fvar_scale_prev_len", "fvar_select_workspace_bytes",
    "fvar_block_workspace_bytes", "fvar_score_select", "fvar_block_forward_dense",
    "fvar_block_forward_pruned", "fvar_lowrank_fill", "fvar_rp_project", "fvar_cache_fill",
    "fvar_factors_workspace_bytes", "fvar_cache_factors", "fvar_upsample_tokens",
    "fvar_profile_enable",
    "fvar_profile_read", "fvar_debug_checks", "fvar_score_select_static",
    "fvar_fill_scored_workspace_bytes", "fvar_lowrank_fill_scored",
)


class FvarError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"fvar status {status}: {msg}")
        self.status = status


class _Config(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn_hidden", C.c_int32), ("num_scales", C.c_int32),
                ("scale_hw", C.POINTER(C.c_int32)), ("dtype", C.c_int), ("ln_eps", C.c_float),
                ("attn_scale", C.c_float)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
        "w_fc1", "b_fc1", "w_fc2", "b_fc2")]


class _KV(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("capacity", C.c_int32), ("len", C.c_int32)]


class _ProfileEntry(C.Structure):
    _fields_ = [("label", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double)]


_lib = None


def load_library() -> C.CDLL:
    """dlopen libfvar.so and declare the prototypes; raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2512_16483_amd.build` (there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.fvar_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
    lib.fvar_create.restype = C.c_int
    lib.fvar_destroy.argtypes = [vp]
    lib.fvar_destroy.restype = None
    lib.fvar_last_error.argtypes = [vp]
    lib.fvar_last_error.restype = C.c_char_p
    lib.fvar_status_string.argtypes = [C.c_int]
    lib.fvar_status_string.restype = C.c_char_p
    lib.fvar_keep_count.argtypes = [i32, i32, i32]
    lib.fvar_keep_count.restype = i32
    lib.fvar_scale_tokens.argtypes = [vp, i32]
    lib.fvar_scale_tokens.restype = i32
    lib.fvar_scale_prev_len.argtypes = [vp, i32]
    lib.fvar_scale_prev_len.restype = i32
    lib.fvar_select_workspace_bytes.argtypes = [vp, i32, i32]
    lib.fvar_select_workspace_bytes.restype = sz
    lib.fvar_block_workspace_bytes.argtypes = [vp, i32, i32]
    lib.fvar_block_workspace_bytes.restype = sz
    lib.fvar_score_select.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz]
    lib.fvar_score_select.restype = C.c_int
    lib.fvar_block_forward_dense.argtypes = [vp, vp, C.POINTER(_Weights), vp, i32, i32,
                                             C.POINTER(_KV), vp, vp, sz]
    lib.fvar_block_forward_dense.restype = C.c_int
    lib.fvar_block_forward_pruned.argtypes = [vp, vp, C.POINTER(_Weights), vp, i32, i32, vp, i32,
                                              C.POINTER(_KV), vp, vp, sz]
    lib.fvar_block_forward_pruned.restype = C.c_int
    lib.fvar_lowrank_fill.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    lib.fvar_lowrank_fill.restype = C.c_int
    lib.fvar_fill_scored_workspace_bytes.argtypes = [vp, i32, i32]
    lib.fvar_fill_scored_workspace_bytes.restype = sz
    lib.fvar_lowrank_fill_scored.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz]
    lib.fvar_lowrank_fill_scored.restype = C.c_int
    lib.fvar_rp_project.argtypes = [vp, vp, vp, i32, vp, i32, i32, i32, vp]
    lib.fvar_rp_project.restype = C.c_int
    lib.fvar_cache_fill.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.fvar_cache_fill.restype = C.c_int
    lib.fvar_factors_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.fvar_factors_workspace_bytes.restype = sz
    lib.fvar_cache_factors.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, C.c_double, vp, vp, vp, sz]
    lib.fvar_cache_factors.restype = C.c_int
    lib.fvar_upsample_tokens.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
    lib.fvar_upsample_tokens.restype = C.c_int
    lib.fvar_score_select_static.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    lib.fvar_score_select_static.restype = C.c_int
    lib.fvar_debug_checks.argtypes = [vp, i32]
    lib.fvar_debug_checks.restype = C.c_int
    lib.fvar_profile_enable.argtypes = [vp, i32]
    lib.fvar_profile_enable.restype = C.c_int
    lib.fvar_profile_read.argtypes = [vp, C.POINTER(_ProfileEntry), i32]
    lib.fvar_profile_read.restype = i32
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device pointer of a contiguous torch tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to fvar must be contiguous GPU tensors")
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return getattr(stream, "cuda_stream", stream) or None


class Context:
    """Owns one fvar_ctx."""

    def __init__(self, hidden: int, heads: int, head_dim: int, ffn_hidden: int,
                 scales: Sequence[int] = (), dtype: str = "bf16", ln_eps: float = 0.0,
                 attn_scale: float = 0.0):
        self.lib = load_library()
        hw = []
        for s in scales:
            hw += list(s) if isinstance(s, (tuple, list)) else [s, s]
        arr = (C.c_int32 * max(len(hw), 1))(*hw)
        cfg = _Config(hidden, heads, head_dim, ffn_hidden, len(hw) // 2, arr,
                      {"f32": FVAR_F32, "bf16": FVAR_BF16}[dtype], ln_eps, attn_scale)
        h = C.c_void_p()
        st = self.lib.fvar_create(C.byref(cfg), C.byref(h))
        if st != FVAR_OK:
            raise FvarError(st, "fvar_create: " + self.lib.fvar_status_string(st).decode())
        self.handle = h
        self.hidden, self.heads, self.head_dim, self.ffn_hidden = hidden, heads, head_dim, ffn_hidden
        self.dtype = dtype

    def check(self, st: int) -> None:
        if st != FVAR_OK:
            raise FvarError(st, self.lib.fvar_last_error(self.handle).decode())

    def close(self) -> None:
        if getattr(self, "handle", None):
            self.lib.fvar_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def fvar_create(**kw) -> Context:
    return Context(**kw)


def fvar_destroy(ctx: Context) -> None:
    ctx.close()


def fvar_keep_count(M: int, keep_num: int, keep_den: int) -> int:
    return load_library().fvar_keep_count(M, keep_num, keep_den)


def fvar_scale_tokens(ctx: Context, scale_index: int) -> int:
    return ctx.lib.fvar_scale_tokens(ctx.handle, scale_index)


def fvar_scale_prev_len(ctx: Context, scale_index: int) -> int:
    return ctx.lib.fvar_scale_prev_len(ctx.handle, scale_index)


def fvar_select_workspace_bytes(ctx: Context, B: int, M: int) -> int:
    return ctx.lib.fvar_select_workspace_bytes(ctx.handle, B, M)


def fvar_block_workspace_bytes(ctx: Context, B: int, rows: int) -> int:
    return ctx.lib.fvar_block_workspace_bytes(ctx.handle, B, rows)


def fvar_score_select(ctx: Context, x, B: int, M: int, k: int, idx_keep, idx_drop=None,
                      scores_in=None, scores_out=None, ws=None, stream=None) -> None:
    ctx.check(ctx.lib.fvar_score_select(ctx.handle, _stream(stream), _ptr(x), B, M, k,
                                        _ptr(scores_in), _ptr(scores_out), _ptr(idx_keep),
                                        _ptr(idx_drop), _ptr(ws), _nbytes(ws)))


def fvar_score_select_static(ctx: Context, x, B: int, M: int, k: int, idx_keep, idx_drop=None,
                             stream=None) -> None:
    ctx.check(ctx.lib.fvar_score_select_static(ctx.handle, _stream(stream), _ptr(x), B, M, k,
                                               _ptr(idx_keep), _ptr(idx_drop)))


def fvar_debug_checks(ctx: Context, on: bool) -> None:
    ctx.check(ctx.lib.fvar_debug_checks(ctx.handle, 1 if on else 0))


def _weights(w: dict) -> _Weights:
    s = _Weights()
    for name, _ in _Weights._fields_:
        setattr(s, name, _ptr(w.get(name)))
    return s


def fvar_block_forward_dense(ctx: Context, w: dict, x, B: int, M: int, kv_k, kv_v, capacity: int,
                             kv_len: int, y, ws, stream=None) -> None:
    kv = _KV(_ptr(kv_k), _ptr(kv_v), capacity, kv_len)
    ws_ = _weights(w)
    ctx.check(ctx.lib.fvar_block_forward_dense(ctx.handle, _stream(stream), C.byref(ws_), _ptr(x),
                                               B, M, C.byref(kv), _ptr(y), _ptr(ws), _nbytes(ws)))


def fvar_block_forward_pruned(ctx: Context, w: dict, x, B: int, M: int, idx_keep, k: int, kv_k,
                              kv_v, capacity: int, kv_len: int, y_keep, ws, stream=None) -> None:
    kv = _KV(_ptr(kv_k), _ptr(kv_v), capacity, kv_len)
    ws_ = _weights(w)
    ctx.check(ctx.lib.fvar_block_forward_pruned(ctx.handle, _stream(stream), C.byref(ws_), _ptr(x),
                                                B, M, _ptr(idx_keep), k, C.byref(kv), _ptr(y_keep),
                                                _ptr(ws), _nbytes(ws)))


def fvar_lowrank_fill(ctx: Context, y_keep, idx_keep, idx_drop, B: int, M: int, k: int, r: int,
                      w_c, g_c, y, stream=None) -> None:
    ctx.check(ctx.lib.fvar_lowrank_fill(ctx.handle, _stream(stream), _ptr(y_keep), _ptr(idx_keep),
                                        _ptr(idx_drop), B, M, k, r, _ptr(w_c), _ptr(g_c), _ptr(y)))


def fvar_fill_scored_workspace_bytes(ctx: Context, B: int, M: int) -> int:
    return ctx.lib.fvar_fill_scored_workspace_bytes(ctx.handle, B, M)


def fvar_lowrank_fill_scored(ctx: Context, y_keep, idx_keep, idx_drop, B: int, M: int, k: int, r: int,
                             w_c, g_c, y, scores_out, ws, stream=None) -> None:
    ctx.check(ctx.lib.fvar_lowrank_fill_scored(ctx.handle, _stream(stream), _ptr(y_keep),
                                               _ptr(idx_keep), _ptr(idx_drop), B, M, k, r, _ptr(w_c),
                                               _ptr(g_c), _ptr(y), _ptr(scores_out), _ptr(ws),
                                               _nbytes(ws)))


def fvar_rp_project(ctx: Context, qt, q_per_sample: bool, x, B: int, M: int, rows: int, out,
                    stream=None) -> None:
    ctx.check(ctx.lib.fvar_rp_project(ctx.handle, _stream(stream), _ptr(qt), 1 if q_per_sample else 0,
                                      _ptr(x), B, M, rows, _ptr(out)))


def fvar_cache_fill(ctx: Context, y_keep, idx_keep, idx_drop, B: int, M: int, k: int, cache, y,
                    stream=None) -> None:
    ctx.check(ctx.lib.fvar_cache_fill(ctx.handle, _stream(stream), _ptr(y_keep), _ptr(idx_keep),
                                      _ptr(idx_drop), B, M, k, _ptr(cache), _ptr(y)))


def fvar_factors_workspace_bytes(ctx: Context, B: int, M: int, r: int) -> int:
    return ctx.lib.fvar_factors_workspace_bytes(ctx.handle, B, M, r)


def fvar_cache_factors(ctx: Context, cache, qt, q_per_sample: bool, B: int, M: int, r: int,
                       ridge: float, w_c, g_c, ws, stream=None) -> None:
    ctx.check(ctx.lib.fvar_cache_factors(ctx.handle, _stream(stream), _ptr(cache), _ptr(qt),
                                         1 if q_per_sample else 0, B, M, r, float(ridge), _ptr(w_c),
                                         _ptr(g_c), _ptr(ws), _nbytes(ws)))


def fvar_upsample_tokens(ctx: Context, src, B: int, hs: int, ws: int, c: int, hd: int, wd: int, dst,
                         stream=None) -> None:
    ctx.check(ctx.lib.fvar_upsample_tokens(ctx.handle, _stream(stream), _ptr(src), B, hs, ws, c, hd,
                                           wd, _ptr(dst)))


def fvar_profile_enable(ctx: Context, on: bool) -> None:
    ctx.check(ctx.lib.fvar_profile_enable(ctx.handle, 1 if on else 0))


def fvar_profile_read(ctx: Context) -> dict:
    """{label: (launches, total_ms)} since the last read."""
    buf = (_ProfileEntry * 64)()
    n = ctx.lib.fvar_profile_read(ctx.handle, buf, 64)
    return {buf[i].label.decode(): (int(buf[i].launches), float(buf[i].total_ms))
            for i in range(min(n, 64))}
