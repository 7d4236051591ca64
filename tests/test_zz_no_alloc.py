"""fvar_score_select_static, the selection entry point that takes no workspace and allocates
nothing (its scores live in a device array built into the library), against fvar_score_select on
the same inputs: index sets bit-identical, on two calls in a row, the second one smaller (the
built-in array then still holds the first call's scores behind the second call's)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2512_16483_amd as fv
import workloads as wl

pytestmark = pytest.mark.gpu


def _select_both(lib, ctx, x, B, M, k):
    dev = lambda *shape: torch.full(shape, -7, dtype=torch.int32, device="cuda")
    keep_a, drop_a, keep_b, drop_b = dev(B, k), dev(B, M - k), dev(B, k), dev(B, M - k)
    ws = torch.empty(fv.fvar_select_workspace_bytes(ctx, B, M), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream or None
    st = lib.fvar_score_select(ctx.handle, stream, x.data_ptr(), B, M, k, None, None,
                               keep_a.data_ptr(), drop_a.data_ptr(), ws.data_ptr(), ws.numel())
    assert st == fv.FVAR_OK, lib.fvar_last_error(ctx.handle)
    # raw C-ABI call: context, stream, x, B, M, k, idx_keep, idx_drop -- no workspace
    st = lib.fvar_score_select_static(ctx.handle, stream, x.data_ptr(), B, M, k, keep_b.data_ptr(),
                                      drop_b.data_ptr())
    assert st == fv.FVAR_OK, lib.fvar_last_error(ctx.handle)
    torch.cuda.synchronize()
    return keep_a, drop_a, keep_b, drop_b


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_selection_matches_workspace_selection_twice(dtype):
    lib = fv.load_library()
    d = 256
    ctx = fv.Context(hidden=d, heads=4, head_dim=64, ffn_hidden=256, dtype=dtype)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for B, M, k in [(3, 1500, 431), (2, 257, 64)]:          # second call smaller than the first
        x = torch.from_numpy(wl.activations_lowrank(B, M, d, seed=31 + M, bf16=dtype == "bf16")
                             ).cuda().to(tdt).contiguous()
        keep_a, drop_a, keep_b, drop_b = _select_both(lib, ctx, x, B, M, k)
        assert torch.equal(keep_a, keep_b) and torch.equal(drop_a, drop_b)
        kh = keep_b.cpu().numpy()
        assert (np.diff(kh, axis=1) > 0).all() and kh.min() >= 0 and kh.max() < M


def test_static_selection_rejects_oversize_and_bad_arguments():
    lib = fv.load_library()
    ctx = fv.Context(hidden=64, heads=1, head_dim=64, ffn_hidden=64, dtype="bf16")
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    h = ctx.handle
    # beyond the built-in array (2^20 scores): rejected before anything is touched
    assert lib.fvar_score_select_static(h, None, x.data_ptr(), 1025, 1024, 4, out.data_ptr(), None) == fv.FVAR_ERR_UNSUPPORTED
    assert b"scratch" in lib.fvar_last_error(h)
    assert lib.fvar_score_select_static(h, None, x.data_ptr(), 1, 8, 9, out.data_ptr(), None) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_score_select_static(h, None, None, 1, 8, 2, out.data_ptr(), None) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_score_select_static(h, None, x.data_ptr(), 1, 8, 2, None, None) == fv.FVAR_ERR_INVALID_ARG
