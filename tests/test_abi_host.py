"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2512_16483_amd as fv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fvar.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fvar_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = fv.load_library()
    names = _declared()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), f"{n} declared in fvar.h but not exported"
    assert sorted(fv.EXPORTS) == names


def test_keep_count_and_schedule_helpers():
    assert fv.fvar_keep_count(1600, 3, 10) == 480
    assert fv.fvar_keep_count(2304, 3, 10) == 692
    assert fv.fvar_keep_count(576, 2, 5) == 231
    assert fv.fvar_keep_count(10, 0, 7) == 1 and fv.fvar_keep_count(10, 9, 7) == 10
    assert fv.fvar_keep_count(0, 1, 2) == -1 and fv.fvar_keep_count(5, 1, 0) == -1
    c = fv.Context(hidden=2048, heads=16, head_dim=128, ffn_hidden=8192,
                   scales=(1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64))
    assert fv.fvar_scale_tokens(c, 12) == 4096 and fv.fvar_scale_prev_len(c, 12) == 6425
    assert fv.fvar_scale_prev_len(c, 10) == 2521 and fv.fvar_scale_tokens(c, 13) == -1
    r = fv.Context(hidden=128, heads=2, head_dim=64, ffn_hidden=256, scales=((3, 5), (4, 7)))
    assert fv.fvar_scale_tokens(r, 1) == 28 and fv.fvar_scale_prev_len(r, 1) == 15
    # workspace: four [rows,d] buffers, the fp32 residual stream [rows,d], one [rows,F] buffer and,
    # for a problem this small, 8 key-range partials of the attention ([rows,d] + 2 [rows,H] fp32)
    assert fv.fvar_block_workspace_bytes(r, 2, 10) == 4 * 5120 + 10240 + 10240 + 8 * 20 * (128 + 4) * 4
    big = fv.Context(hidden=1920, heads=30, head_dim=64, ffn_hidden=7680)
    rows = 8 * 410
    assert fv.fvar_block_workspace_bytes(big, 8, 410) == sum(
        (n + 255) // 256 * 256 for n in [rows * 1920 * 2] * 4 + [rows * 1920 * 4, rows * 7680 * 2])
    assert fv.fvar_select_workspace_bytes(r, 3, 100) == 1280


@pytest.mark.parametrize("kw", [
    dict(hidden=128, heads=3, head_dim=64, ffn_hidden=256),      # heads * head_dim != hidden
    dict(hidden=96, heads=3, head_dim=32, ffn_hidden=256),       # head_dim not 64 / 128
    dict(hidden=128, heads=2, head_dim=64, ffn_hidden=100),      # ffn not a multiple of 64
    dict(hidden=16384, heads=128, head_dim=128, ffn_hidden=256),  # row does not fit one wavefront
    dict(hidden=0, heads=0, head_dim=64, ffn_hidden=64),
])
def test_create_rejects_bad_geometry(kw):
    with pytest.raises(fv.FvarError):
        fv.Context(**kw)


def _call(lib, name, *args):
    return getattr(lib, name)(*args)


def test_entry_points_reject_bad_arguments_without_launching():
    lib = fv.load_library()
    c = fv.Context(hidden=128, heads=2, head_dim=64, ffn_hidden=256, dtype="bf16")
    h = c.handle
    fake = 0x1000          # aligned, never dereferenced on the host
    # k out of range, null outputs, misaligned pointer, missing workspace
    assert lib.fvar_score_select(h, None, fake, 1, 10, 11, None, None, fake, None, None, 0) == fv.FVAR_ERR_INVALID_ARG
    assert b"k<=M" in lib.fvar_last_error(h)
    assert lib.fvar_score_select(h, None, fake, 1, 10, 0, None, None, fake, None, None, 0) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_score_select(h, None, fake, 1, 10, 5, None, None, None, None, None, 0) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_score_select(h, None, None, 1, 10, 5, None, None, fake, None, None, 0) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_score_select(h, None, fake + 2, 1, 10, 5, None, None, fake, None, None, 0) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_score_select(h, None, fake, 1, 10, 5, None, None, fake, None, None, 0) == fv.FVAR_ERR_WORKSPACE
    assert lib.fvar_score_select(h, None, fake, 1, (1 << 20) + 1, 5, None, None, fake, None, fake, 1 << 30) == fv.FVAR_ERR_UNSUPPORTED

    w = fv._Weights()
    for n, _ in fv._Weights._fields_:
        setattr(w, n, None)
    kv = fv._KV(fake, fake, 100, 95)
    # weights missing
    assert lib.fvar_block_forward_pruned(h, None, C.byref(w), fake, 1, 10, fake, 5, C.byref(kv), fake, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    for n in ("w_qkv", "w_o", "w_fc1", "w_fc2"):
        setattr(w, n, fake)
    # cache overflow: len 95 + 10 rows > capacity 100
    assert lib.fvar_block_forward_dense(h, None, C.byref(w), fake, 1, 10, C.byref(kv), fake, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    assert b"capacity" in lib.fvar_last_error(h)
    kv.len = 0
    # k > M, NULL index list with k < M, workspace too small
    assert lib.fvar_block_forward_pruned(h, None, C.byref(w), fake, 1, 10, fake, 11, C.byref(kv), fake, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_block_forward_pruned(h, None, C.byref(w), fake, 1, 10, None, 5, C.byref(kv), fake, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    need = fv.fvar_block_workspace_bytes(c, 1, 5)
    assert lib.fvar_block_forward_pruned(h, None, C.byref(w), fake, 1, 10, fake, 5, C.byref(kv), fake, fake, need - 1) == fv.FVAR_ERR_WORKSPACE
    assert lib.fvar_block_forward_pruned(h, None, C.byref(w), fake, 1, 10, fake, 5, C.byref(kv), fake, None, 0) == fv.FVAR_ERR_WORKSPACE
    # fill: rank must be a multiple of 8 for bf16 and at most 256; factors required when k < M
    assert lib.fvar_lowrank_fill(h, None, fake, fake, fake, 1, 10, 5, 12, fake, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_lowrank_fill(h, None, fake, fake, fake, 1, 10, 5, 264, fake, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_lowrank_fill(h, None, fake, fake, fake, 1, 10, 5, 16, None, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_lowrank_fill(h, None, fake, fake, None, 1, 10, 5, 16, fake, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_lowrank_fill(h, None, fake, fake, fake, 1, 10, 11, 16, fake, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_status_string(fv.FVAR_ERR_WORKSPACE) == b"workspace too small"
    # random projection: rows in [1,M], M a multiple of 8 for bf16, pointers present and aligned
    assert lib.fvar_rp_project(h, None, fake, 0, fake, 1, 16, 17, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_rp_project(h, None, fake, 0, fake, 1, 16, 0, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_rp_project(h, None, None, 0, fake, 1, 16, 4, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_rp_project(h, None, fake + 4, 0, fake, 1, 16, 4, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_rp_project(h, None, fake, 0, fake, 1, 12, 4, fake) == fv.FVAR_ERR_UNSUPPORTED
    # raw-cache fill: the cache and the pruned index list are required when rows are pruned
    assert lib.fvar_cache_fill(h, None, fake, fake, fake, 1, 10, 11, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_cache_fill(h, None, fake, fake, None, 1, 10, 5, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_cache_fill(h, None, fake, fake, fake, 1, 10, 5, None, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_cache_fill(h, None, None, fake, fake, 1, 10, 5, fake, fake) == fv.FVAR_ERR_INVALID_ARG
    # up-sampling: sizes >= 1, channels a multiple of the 16-byte chunk
    assert lib.fvar_upsample_tokens(h, None, fake, 1, 0, 4, 8, 8, 8, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_upsample_tokens(h, None, None, 1, 4, 4, 8, 8, 8, fake) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_upsample_tokens(h, None, fake, 1, 4, 4, 12, 8, 8, fake) == fv.FVAR_ERR_UNSUPPORTED
    # factors: rank limits, ridge sign, workspace
    need = fv.fvar_factors_workspace_bytes(c, 2, 64, 16)
    assert need == 2 * 2 * 64 * 16 * 4 + (8 + 1) * (2 * 16 * 16 * 8)     # 2 slices of T, 8 partial Gram matrices, inverse
    assert lib.fvar_cache_factors(h, None, fake, fake, 0, 2, 64, 136, 0.0, fake, fake, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_cache_factors(h, None, fake, fake, 0, 2, 256, 136, 0.0, fake, fake, fake, 1 << 30) == fv.FVAR_ERR_UNSUPPORTED
    assert lib.fvar_cache_factors(h, None, fake, fake, 0, 2, 64, 12, 0.0, fake, fake, fake, 1 << 30) == fv.FVAR_ERR_UNSUPPORTED
    assert lib.fvar_cache_factors(h, None, fake, fake, 0, 2, 64, 16, -1.0, fake, fake, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_cache_factors(h, None, fake, fake, 0, 2, 64, 16, 0.0, fake, None, fake, 1 << 30) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_cache_factors(h, None, fake, fake, 0, 2, 64, 16, 0.0, fake, fake, fake, need - 1) == fv.FVAR_ERR_WORKSPACE


def test_block_calls_reject_operands_beyond_32bit_tile_offsets():
    """The linear-layer kernels address an operand matrix with 32-bit byte offsets: a call whose
    widest operand (B*rows x max(hidden, ffn_hidden) elements) reaches 4 GiB must be refused
    before anything is launched, not wrap silently."""
    lib = fv.load_library()
    c = fv.Context(hidden=2048, heads=16, head_dim=128, ffn_hidden=8192, dtype="bf16")
    h, fake = c.handle, 0x1000
    w = fv._Weights()
    for n, _ in fv._Weights._fields_:
        setattr(w, n, None)
    for n in ("w_qkv", "w_o", "w_fc1", "w_fc2"):
        setattr(w, n, fake)
    kv = fv._KV(fake, fake, 1 << 20, 0)
    # 64 x 4096 rows x 8192 columns x 2 bytes = 4 GiB exactly: refused
    assert lib.fvar_block_forward_dense(h, None, C.byref(w), fake, 64, 4096, C.byref(kv), fake, fake, 1 << 60) == fv.FVAR_ERR_UNSUPPORTED
    assert b"4 GiB" in lib.fvar_last_error(h)
    # one row less per sample is inside the limit: the call gets as far as the workspace check
    assert lib.fvar_block_forward_dense(h, None, C.byref(w), fake, 64, 4095, C.byref(kv), fake, fake, 16) == fv.FVAR_ERR_WORKSPACE
    # batch beyond the launch grid's third dimension (8 key ranges per sample)
    assert lib.fvar_block_forward_dense(h, None, C.byref(w), fake, 8192, 8, C.byref(kv), fake, fake, 1 << 60) == fv.FVAR_ERR_UNSUPPORTED
    # the selection without workspace: size limit and argument checks need no GPU either
    assert lib.fvar_score_select_static(h, None, fake, 1025, 1024, 4, fake, None) == fv.FVAR_ERR_UNSUPPORTED
    assert lib.fvar_score_select_static(h, None, fake, 1, 8, 9, fake, None) == fv.FVAR_ERR_INVALID_ARG
    assert lib.fvar_debug_checks(h, 1) == fv.FVAR_OK and lib.fvar_debug_checks(h, 0) == fv.FVAR_OK


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(fv, "_lib", None)
    monkeypatch.setattr(fv, "LIB_PATH", "/nonexistent/libfvar.so")
    with pytest.raises(ImportError):
        fv.load_library()
