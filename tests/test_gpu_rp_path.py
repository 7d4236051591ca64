"""GPU parity of the random-projection input path and of the on-GPU factor construction: the HIP
kernels through the C ABI against the CPU oracle on the same seeded inputs.

Bars as for the main path: copies and index work bit-exact; bf16 outputs within 2e-2, fp32
outputs within 1e-4, measured as max_i |g_i - o_i| / max(|o_i|, rms(o))."""
import numpy as np
import pytest
import torch

import oracle
from oracle import factors, rp_path
import paper_2512_16483_amd as fv
import workloads as wl

pytestmark = pytest.mark.gpu

from gpu_util import TOL, GpuBlock, rel_err, tdtype, to_dev, to_np  # noqa: E402


def _ctx(d, dtype, H=None):
    H = H or d // 64
    return fv.Context(hidden=d, heads=H, head_dim=d // H, ffn_hidden=4 * d, dtype=dtype)


def _q(B, M, r, seed, dtype, per_sample):
    """Q = z / sqrt(r) in the storage type, [B or 1, M, r]."""
    z = wl.normal_draws(B if per_sample else 1, M, r, seed=seed)
    Q = (z / np.sqrt(float(r))).astype(np.float32)
    return wl.round_to_bf16(Q) if dtype == "bf16" else Q


def _qt_dev(Q, dtype):
    return to_dev(np.ascontiguousarray(np.swapaxes(Q, 1, 2)), dtype)      # [B or 1, r, M]


# ----------------------------------------------------------------------------- projection
@pytest.mark.parametrize("dtype,B,M,rows,d,per_sample", [
    ("bf16", 2, 72, 5, 128, False),          # one full chunk of 64 tokens + a ragged one
    ("bf16", 3, 200, 130, 192, True),        # two row tiles, ragged rows, ragged column tile
    ("bf16", 1, 576, 231, 1920, False),      # scale 24 of the depth-30 model
    ("bf16", 2, 1024, 64, 256, True),
    ("bf16", 1, 8, 1, 64, False),            # minimal
    ("f32", 2, 36, 7, 64, True),
    ("f32", 1, 256, 32, 1024, False),        # the fp32 configuration
])
def test_rp_project_parity(dtype, B, M, rows, d, per_sample):
    x = wl.activations_lowrank(B, M, d, seed=50 + M, bf16=dtype == "bf16")
    Q = _q(B, M, rows, 60 + M, dtype, per_sample)
    ctx = _ctx(d, dtype)
    out = torch.full((B, rows, d), float("nan"), dtype=tdtype(dtype), device="cuda")
    fv.fvar_rp_project(ctx, _qt_dev(Q, dtype), per_sample, to_dev(x, dtype), B, M, rows, out)
    torch.cuda.synchronize()
    got = to_np(out)
    for b in range(B):
        ref = rp_path.rp_input(Q[b if per_sample else 0], x[b], bf16=dtype == "bf16")
        assert rel_err(got[b], ref) <= TOL[dtype], (b, rel_err(got[b], ref))


@pytest.mark.parametrize("B,M,rows,d,per_sample", [
    (12, 128, 128, 4096, False),     # 128x256 tiles, two k-tiles on a three-stage ring
    (12, 64, 64, 4096, True),        # a single k-tile, Q per sample
    (24, 320, 320, 2048, True),      # rows of one and a quarter 256-row tiles
    (16, 256, 250, 3136, False),     # 256x256 tiles, ragged rows and columns
    (16, 192, 192, 3072, True),      # 192x256 tiles, three k-tiles
    (32, 512, 500, 384, False),      # 256x128 tiles, ragged rows
    (3, 1024, 700, 4096, True),      # long contraction, several rounds of workgroups
])
def test_rp_project_tiled_path(B, M, rows, d, per_sample):
    """Shapes on whole 64-token k-tiles with enough output tiles to fill the chip run on the tiled
    MFMA kernel of the linear layers with the token map as a k-major operand: every tile
    configuration it can pick, against the oracle on every sample."""
    x = wl.activations_lowrank(B, M, d, seed=150 + M + rows, bf16=True)
    Q = _q(B, M, rows, 160 + M + rows, "bf16", per_sample)
    ctx = _ctx(d, "bf16")
    out = torch.full((B, rows, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    fv.fvar_rp_project(ctx, _qt_dev(Q, "bf16"), per_sample, to_dev(x, "bf16"), B, M, rows, out)
    torch.cuda.synchronize()
    got = to_np(out)
    assert np.isfinite(got).all()
    for b in range(B):
        ref = rp_path.rp_input(Q[b if per_sample else 0], x[b], bf16=True)
        assert rel_err(got[b], ref) <= TOL["bf16"], (b, rel_err(got[b], ref))


def test_rp_project_tiled_path_selection_matrix_bitexact():
    # products with 1 and 0 are exact: a column-selection Q reproduces the rows bit for bit
    B, M, rows, d = 12, 128, 128, 4096
    x = wl.activations_iid(B, M, d, seed=171, bf16=True)
    rng = np.random.default_rng(6)
    Q = np.zeros((B, M, rows), np.float32)
    idx = np.stack([rng.permutation(M)[:rows] for _ in range(B)])
    for b in range(B):
        Q[b, idx[b], np.arange(rows)] = 1.0
    ctx = _ctx(d, "bf16")
    out = torch.empty((B, rows, d), dtype=torch.bfloat16, device="cuda")
    fv.fvar_rp_project(ctx, _qt_dev(Q, "bf16"), True, to_dev(x, "bf16"), B, M, rows, out)
    torch.cuda.synchronize()
    for b in range(B):
        assert np.array_equal(to_np(out[b]), x[b][idx[b]])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rp_project_with_selection_matrix_is_the_gather(dtype):
    # products with 1 and 0 are exact, so a column-selection Q must reproduce the rows bit for bit
    B, M, rows, d = 2, 136, 40, 192
    x = wl.activations_iid(B, M, d, seed=71, bf16=dtype == "bf16")
    rng = np.random.default_rng(5)
    Q = np.zeros((B, M, rows), np.float32)
    idx = np.stack([np.sort(rng.choice(M, rows, replace=False)) for _ in range(B)])
    for b in range(B):
        Q[b, idx[b], np.arange(rows)] = 1.0
    ctx = _ctx(d, dtype)
    out = torch.empty((B, rows, d), dtype=tdtype(dtype), device="cuda")
    fv.fvar_rp_project(ctx, _qt_dev(Q, dtype), True, to_dev(x, dtype), B, M, rows, out)
    torch.cuda.synchronize()
    for b in range(B):
        assert np.array_equal(to_np(out[b]), x[b][idx[b]])


# ----------------------------------------------------------------------------- raw-cache fill
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,M,k,d", [(2, 37, 11, 128), (1, 64, 0, 64), (3, 50, 50, 192), (2, 576, 231, 1920)])
def test_cache_fill_bitexact(dtype, B, M, k, d):
    bf = dtype == "bf16"
    Cm = wl.activations_iid(B, M, d, seed=81, bf16=bf)
    yk = wl.activations_iid(B, max(k, 1), d, seed=82, bf16=bf)[:, :k]
    rng = np.random.default_rng(M + k)
    keep = np.stack([np.sort(rng.choice(M, k, replace=False)) for _ in range(B)]).astype(np.int32).reshape(B, k)
    drop = np.stack([np.setdiff1d(np.arange(M), keep[b]) for b in range(B)]).astype(np.int32).reshape(B, M - k)
    ctx = _ctx(d, dtype)
    kd, dd = torch.from_numpy(keep).cuda(), torch.from_numpy(drop).cuda()
    ykd, Cd = to_dev(yk, dtype), to_dev(Cm, dtype)
    y = torch.full((B, M, d), float("nan"), dtype=tdtype(dtype), device="cuda")
    fv.fvar_cache_fill(ctx, ykd if k else None, kd if k else None, dd if k < M else None, B, M, k,
                       Cd if k < M else None, y)
    # in place: the cache buffer itself receives the kept rows
    Cin = Cd.clone()
    fv.fvar_cache_fill(ctx, ykd if k else None, kd if k else None, dd if k < M else None, B, M, k,
                       Cin, Cin)
    torch.cuda.synchronize()
    for b in range(B):
        ref = rp_path.cache_fill(yk[b], keep[b], Cm[b])
        assert np.array_equal(to_np(y[b]), ref)
        assert np.array_equal(to_np(Cin[b]), ref)


# ----------------------------------------------------------------------------- factors
@pytest.mark.parametrize("dtype,B,M,d,r,rank,noise,per_sample", [
    ("bf16", 2, 72, 128, 8, 24, 0.1, True),
    ("bf16", 1, 200, 192, 40, 60, 0.1, False),       # r not a multiple of 32, ragged row block
    ("bf16", 2, 576, 1920, 64, 102, 0.1, False),     # depth-30 geometry, scale 24
    ("bf16", 1, 256, 256, 128, 200, 0.1, False),     # largest rank
    ("bf16", 1, 64, 64, 16, 16, 0.0, False),         # exactly rank r: lossless
    ("f32", 2, 36, 64, 8, 12, 0.1, True),
    ("f32", 1, 256, 1024, 32, 32, 0.05, False),      # the fp32 configuration
])
def test_cache_factors_parity(dtype, B, M, d, r, rank, noise, per_sample):
    bf = dtype == "bf16"
    Cm = wl.cached_feature(B, M, d, rank, seed=90 + M, noise=noise)
    if bf:
        Cm = wl.round_to_bf16(Cm)
    Q = _q(B, M, r, 91 + M, dtype, per_sample)
    ctx = _ctx(d, dtype)
    Cd = to_dev(Cm, dtype)
    w_c = torch.full((B, M, r), float("nan"), dtype=tdtype(dtype), device="cuda")
    g_c = torch.full((B, r, d), float("nan"), dtype=tdtype(dtype), device="cuda")
    ws = torch.empty(fv.fvar_factors_workspace_bytes(ctx, B, M, r), dtype=torch.uint8, device="cuda")
    fv.fvar_cache_factors(ctx, Cd, _qt_dev(Q, dtype), per_sample, B, M, r, 0.0, w_c, g_c, ws)
    torch.cuda.synchronize()
    Wg, Gg = to_np(w_c), to_np(g_c)
    for b in range(B):
        Wo, Go = factors.stored_factors(Cm[b], Q[b if per_sample else 0], bf16=bf)
        assert rel_err(Gg[b], Go) <= TOL[dtype], ("G", b, rel_err(Gg[b], Go))
        assert rel_err(Wg[b], Wo) <= TOL[dtype], ("W", b, rel_err(Wg[b], Wo))
        # the restoration the factors exist for: as close to C as the oracle's
        C64 = Cm[b].astype(np.float64)
        res_g = np.linalg.norm(Wg[b].astype(np.float64) @ Gg[b].astype(np.float64) - C64)
        res_o = np.linalg.norm(Wo.astype(np.float64) @ Go.astype(np.float64) - C64)
        assert res_g <= res_o * 1.02 + (4e-3 if bf else 1e-6) * np.linalg.norm(C64)
        if noise == 0.0:       # rank r exactly (up to the bf16 rounding of C, W and G themselves)
            assert res_g <= (2e-2 if bf else 1e-5) * np.linalg.norm(C64)


def test_cache_factors_feed_the_fill():
    # factors built on the GPU, used by the rank-r fill, against the oracle's fill of its factors
    dtype, B, M, d, r, k = "bf16", 2, 144, 256, 32, 58
    Cm = wl.round_to_bf16(wl.cached_feature(B, M, d, 40, seed=95, noise=0.05))
    Q = _q(B, M, r, 96, dtype, False)
    ctx = _ctx(d, dtype)
    w_c = torch.empty((B, M, r), dtype=torch.bfloat16, device="cuda")
    g_c = torch.empty((B, r, d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(fv.fvar_factors_workspace_bytes(ctx, B, M, r), dtype=torch.uint8, device="cuda")
    fv.fvar_cache_factors(ctx, to_dev(Cm, dtype), _qt_dev(Q, dtype), False, B, M, r, 0.0, w_c, g_c, ws)
    rng = np.random.default_rng(1)
    keep = np.stack([np.sort(rng.choice(M, k, replace=False)) for _ in range(B)]).astype(np.int32)
    drop = np.stack([np.setdiff1d(np.arange(M), keep[b]) for b in range(B)]).astype(np.int32)
    yk = wl.activations_iid(B, k, d, seed=97, bf16=True)
    y = torch.empty((B, M, d), dtype=torch.bfloat16, device="cuda")
    fv.fvar_lowrank_fill(ctx, to_dev(yk, dtype), torch.from_numpy(keep).cuda(), torch.from_numpy(drop).cuda(),
                         B, M, k, r, w_c, g_c, y)
    torch.cuda.synchronize()
    for b in range(B):
        Wo, Go = factors.stored_factors(Cm[b], Q[0], bf16=True)
        ref = oracle.lowrank_fill(yk[b], keep[b], drop[b], M, Wo, Go)
        assert rel_err(to_np(y[b]), ref) <= TOL[dtype]


# ----------------------------------------------------------------------------- whole RP step
def _rp_case(dtype, B, M, r, d, H, Lp, seed):
    bf = dtype == "bf16"
    x = wl.activations_lowrank(B, M, d, seed=seed, bf16=bf)
    w = wl.block_weights(d, 4 * d, seed=seed + 1, bf16=bf, std=0.8 / np.sqrt(d))
    Kp, Vp = wl.kv_prefix(B, Lp, H, d // H, seed=seed + 2, bf16=bf)
    Cm = wl.cached_feature(B, M, d, max(8, r), seed=seed + 3, noise=0.05)
    if bf:
        Cm = wl.round_to_bf16(Cm)
    Q = _q(B, M, r, seed + 4, dtype, False)
    return x, w, Kp, Vp, Cm, Q


@pytest.mark.parametrize("dtype,B,M,r,d,H,Lp", [
    ("bf16", 2, 144, 58, 256, 4, 100),
    ("bf16", 1, 200, 64, 256, 2, 77),        # head_dim 128
    ("f32", 1, 64, 16, 128, 2, 40),
    ("f32", 1, 256, 128, 1024, 16, 424),     # the fp32 configuration with the projected input
])
def test_rp_step_parity(dtype, B, M, r, d, H, Lp):
    x, w, Kp, Vp, Cm, Q = _rp_case(dtype, B, M, r, d, H, Lp, seed=300 + M)
    blk = GpuBlock(d, H, 4 * d, dtype, w, Kp, Vp, Lp + r)
    xd = to_dev(x, dtype)
    f_r = torch.empty((B, r, d), dtype=tdtype(dtype), device="cuda")
    fv.fvar_rp_project(blk.ctx, _qt_dev(Q, dtype), False, xd, B, M, r, f_r)
    y_keep = blk.dense(f_r)                                  # the r projected rows are the block's tokens
    s, keep, drop = blk.score_select(xd, r)
    y = torch.full((B, M, d), float("nan"), dtype=tdtype(dtype), device="cuda")
    fv.fvar_cache_fill(blk.ctx, y_keep, keep, drop, B, M, r, to_dev(Cm, dtype), y)
    torch.cuda.synchronize()
    ow = oracle.BlockWeights(**w)
    for b in range(B):
        Kc = np.zeros((Lp + r, H, d // H), np.float32); Vc = np.zeros_like(Kc)
        Kc[:Lp], Vc[:Lp] = Kp[b], Vp[b]
        ref = rp_path.rp_step(x[b], Q[0], Cm[b], ow, H, Kc, Vc, Lp, bf16=dtype == "bf16")
        assert rel_err(to_np(f_r[b]), ref["f_r"]) <= TOL[dtype]
        assert np.array_equal(keep[b].cpu().numpy(), ref["idx_keep"])
        assert np.array_equal(drop[b].cpu().numpy(), ref["idx_drop"])
        assert rel_err(to_np(y_keep[b]), ref["y_keep"]) <= TOL[dtype], rel_err(to_np(y_keep[b]), ref["y_keep"])
        assert rel_err(to_np(blk.K[b, Lp:]), Kc[Lp:]) <= TOL[dtype]
        assert rel_err(to_np(blk.V[b, Lp:]), Vc[Lp:]) <= TOL[dtype]
        yg = to_np(y[b])
        assert np.array_equal(yg[ref["idx_drop"]], Cm[b][ref["idx_drop"]])
        assert np.array_equal(yg[ref["idx_keep"]], to_np(y_keep[b]))


def test_rp_project_depth30_launch_shape_sampled():
    # the shape the benchmark times (batch 8, scale 32, 410 of 1024 rows): sampled output rows
    W = wl.WORKLOADS["var_d30_512_bf16"]
    B, M, d = W.batch, W.tokens(32), W.hidden
    r = W.keep(32)
    x = wl.activations_lowrank(B, M, d, seed=1002, bf16=True)
    Q = _q(B, M, r, 4002, "bf16", False)
    ctx = _ctx(d, "bf16", H=W.heads)
    out = torch.empty((B, r, d), dtype=torch.bfloat16, device="cuda")
    fv.fvar_rp_project(ctx, _qt_dev(Q, "bf16"), False, to_dev(x, "bf16"), B, M, r, out)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    for b in (0, 3, 7):
        rows = np.concatenate([[0, r - 1, 127, 128, 383, 384], rng.integers(0, r, 10)])
        ref = Q[0][:, rows].astype(np.float64).T @ x[b].astype(np.float64)
        assert rel_err(to_np(out[b])[rows], factors.round_bf16(ref)) <= TOL["bf16"]


# ----------------------------------------------------------------------------- cache up-sampling
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,hs,ws,hd,wd,c", [(2, 3, 3, 4, 4, 8), (1, 24, 24, 32, 32, 64), (2, 5, 7, 8, 9, 24),
                                              (1, 4, 4, 4, 4, 16), (1, 6, 6, 3, 3, 8), (1, 1, 1, 5, 5, 8),
                                              (1, 18, 18, 24, 24, 1920)])
def test_upsample_tokens_parity(dtype, B, hs, ws, hd, wd, c):
    from oracle import upsample
    bf = dtype == "bf16"
    src = wl.activations_iid(B, hs * ws, c, seed=110 + hs, bf16=bf)
    ctx = _ctx(64, dtype)
    dst = torch.full((B, hd * wd, c), float("nan"), dtype=tdtype(dtype), device="cuda")
    fv.fvar_upsample_tokens(ctx, to_dev(src, dtype), B, hs, ws, c, hd, wd, dst)
    torch.cuda.synchronize()
    for b in range(B):
        ref = upsample.upsample_tokens(src[b], hs, ws, hd, wd)
        assert rel_err(to_np(dst[b]), ref) <= (2.0 ** -8 if bf else 1e-6)
    if (hs, ws) == (hd, wd):
        assert np.array_equal(to_np(dst), src)


@pytest.mark.parametrize("hs,hd,d,r,nblk,B,k", [(8, 12, 256, 32, 1, 2, 58),
                                               (24, 32, 1920, 64, 3, 2, 410),     # depth-30 shape, 24 -> 32
                                               (40, 48, 2048, 64, 2, 2, 692)])    # Infinity-2B shape, 40 -> 48
def test_factored_cache_handed_from_scale_to_scale(hs, hd, d, r, nblk, B, k):
    """The cached counterpart features stay in factored form between two scales: the outputs of
    all blocks at the previous scale are factored in ONE call (batch = blocks x samples), only the
    thin factor W_c is up-sampled to the next grid (Up(W_c G_c) = Up(W_c) G_c), and the next
    scale's restoration multiplies it with the unchanged G_c.  Against the oracle's chain
    stored_factors -> upsample_tokens -> lowrank_fill: every stage meets the bar on identical
    inputs (the oracle continues from the factors the GPU stored); the whole chain, in which the
    two sides may round a stored factor element to different bf16 neighbours before the rank-r sum
    amplifies the difference, is held to 2.5 x the bar, like the unrounded statement below."""
    from oracle import upsample
    dtype = "bf16"
    Ms, M, n = hs * hs, hd * hd, nblk * B
    Cm = wl.round_to_bf16(wl.cached_feature(n, Ms, d, max(r, 40), seed=120 + hs, noise=0.05))
    Q = _q(1, Ms, r, 121 + hs, dtype, False)
    ctx = _ctx(d, dtype)
    w_s = torch.empty((n, Ms, r), dtype=torch.bfloat16, device="cuda")
    g_c = torch.empty((n, r, d), dtype=torch.bfloat16, device="cuda")
    ws_ = torch.empty(fv.fvar_factors_workspace_bytes(ctx, n, Ms, r), dtype=torch.uint8, device="cuda")
    fv.fvar_cache_factors(ctx, to_dev(Cm, dtype), _qt_dev(Q, dtype), False, n, Ms, r, 0.0, w_s, g_c, ws_)
    w_up = torch.empty((n, M, r), dtype=torch.bfloat16, device="cuda")
    fv.fvar_upsample_tokens(ctx, w_s, n, hs, hs, r, hd, hd, w_up)
    rng = np.random.default_rng(2)
    keep = np.stack([np.sort(rng.choice(M, k, replace=False)) for _ in range(B)]).astype(np.int32)
    drop = np.stack([np.setdiff1d(np.arange(M), keep[b]) for b in range(B)]).astype(np.int32)
    yk = wl.activations_iid(B, k, d, seed=122, bf16=True)
    ykd, kd, dd = to_dev(yk, dtype), torch.from_numpy(keep).cuda(), torch.from_numpy(drop).cuda()
    torch.cuda.synchronize()
    Wg, Gg, Wupg = to_np(w_s), to_np(g_c), to_np(w_up)
    for i in range(n):                            # stage 1 and 2 against the oracle
        Wo, Go = factors.stored_factors(Cm[i], Q[0], bf16=True)
        assert rel_err(Gg[i], Go) <= TOL[dtype] and rel_err(Wg[i], Wo) <= TOL[dtype]
        assert rel_err(Wupg[i], upsample.upsample_tokens(Wg[i], hs, hs, hd, hd)) <= 2.0 ** -8
    for blk in range(nblk):                       # block blk of the next scale uses slice blk*B .. of the factors
        sl = slice(blk * B, (blk + 1) * B)
        y = torch.empty((B, M, d), dtype=torch.bfloat16, device="cuda")
        fv.fvar_lowrank_fill(ctx, ykd, kd, dd, B, M, k, r, w_up[sl].contiguous(), g_c[sl].contiguous(), y)
        torch.cuda.synchronize()
        for b in range(B):
            Wo, Go = factors.stored_factors(Cm[blk * B + b], Q[0], bf16=True)
            Wup = factors.round_bf16(upsample.upsample_tokens(Wo, hs, hs, hd, hd))
            ref = oracle.lowrank_fill(yk[b], keep[b], drop[b], M, Wup, Go)
            assert rel_err(to_np(y[b]), ref) <= 2.5 * TOL[dtype]                     # whole chain
            ref_stage = oracle.lowrank_fill(yk[b], keep[b], drop[b], M, Wupg[blk * B + b], Gg[blk * B + b])
            assert rel_err(to_np(y[b]), ref_stage) <= TOL[dtype]                    # stage 3 alone
            if blk == 0 and b == 0:
                # that restoration is the up-sampled restored cache itself; against this unrounded
                # statement the bf16 storage of Up(W_c) and of the output both count, hence the
                # wider bound
                full = upsample.upsample_tokens(Wo.astype(np.float64) @ Go.astype(np.float64), hs, hs, hd, hd)
                assert rel_err(to_np(y[b])[drop[b]], full[drop[b]]) <= 2.5 * TOL[dtype]


# ----------------------------------------------------------------------------- one selection per chunk
@pytest.mark.parametrize("dtype,B,M,k,d,H,Lp,r,nblk", [
    ("bf16", 2, 144, 58, 256, 4, 100, 16, 3),
    ("f32", 1, 64, 20, 128, 2, 40, 8, 2),
])
def test_block_chunk_with_one_selection(dtype, B, M, k, d, H, Lp, r, nblk):
    """Select once, gather once, run the chunk's blocks on the compact rows, fill once: the
    existing entry points chained (pruned call for the first block, the dense call on k rows for
    the others) against the oracle's chunk."""
    bf = dtype == "bf16"
    x = wl.activations_lowrank(B, M, d, seed=400, bf16=bf)
    ws = [wl.block_weights(d, 4 * d, seed=401 + i, bf16=bf, std=0.8 / np.sqrt(d)) for i in range(nblk)]
    kvs = [wl.kv_prefix(B, Lp, H, d // H, seed=420 + i, bf16=bf) for i in range(nblk)]
    Cm = wl.cached_feature(B, M, d, r, seed=430, noise=0.05)
    z = wl.normal_draws(B, M, r, seed=431)
    Wc = np.empty((B, M, r), np.float32); Gc = np.empty((B, r, d), np.float32)
    for b in range(B):
        Wc[b], Gc[b] = factors.cache_factors(Cm[b], z[b])
    if bf:
        Wc, Gc = wl.round_to_bf16(Wc), wl.round_to_bf16(Gc)
    blks = [GpuBlock(d, H, 4 * d, dtype, ws[i], kvs[i][0], kvs[i][1], Lp + k) for i in range(nblk)]
    xd = to_dev(x, dtype)
    s, keep, drop = blks[0].score_select(xd, k)
    rows = blks[0].pruned(xd, keep, k)
    for blk in blks[1:]:
        rows = blk.dense(rows)
    y = blks[0].fill(rows, keep, drop, M, to_dev(Wc, dtype), to_dev(Gc, dtype))
    torch.cuda.synchronize()
    for b in range(B):
        caches = []
        for i in range(nblk):
            Kc = np.zeros((Lp + k, H, d // H), np.float32); Vc = np.zeros_like(Kc)
            Kc[:Lp], Vc[:Lp] = kvs[i][0][b], kvs[i][1][b]
            caches.append((Kc, Vc))
        ref = oracle.pruned_chunk(x[b], k, [oracle.BlockWeights(**w) for w in ws], H, caches, Lp,
                                  Wc[b], Gc[b])
        assert np.array_equal(keep[b].cpu().numpy(), ref["idx_keep"])
        assert np.array_equal(drop[b].cpu().numpy(), ref["idx_drop"])
        assert rel_err(to_np(rows[b]), ref["y_keep"]) <= TOL[dtype], rel_err(to_np(rows[b]), ref["y_keep"])
        assert rel_err(to_np(y[b]), ref["y"]) <= TOL[dtype]
        for i in range(nblk):
            assert rel_err(to_np(blks[i].K[b, Lp:]), caches[i][0][Lp:]) <= TOL[dtype]
            assert rel_err(to_np(blks[i].V[b, Lp:]), caches[i][1][Lp:]) <= TOL[dtype]


def test_cache_factors_depth30_launch_shape():
    # the shape the benchmark times (batch 8, scale 32, rank 64): two samples against the oracle
    W = wl.WORKLOADS["var_d30_512_bf16"]
    B, M, d, r = W.batch, W.tokens(32), W.hidden, W.rank
    Cm = wl.round_to_bf16(wl.cached_feature(B, M, d, 180, seed=4100, noise=0.1))
    Q = _q(B, M, r, 4101, "bf16", False)
    ctx = _ctx(d, "bf16", H=W.heads)
    w_c = torch.empty((B, M, r), dtype=torch.bfloat16, device="cuda")
    g_c = torch.empty((B, r, d), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(fv.fvar_factors_workspace_bytes(ctx, B, M, r), dtype=torch.uint8, device="cuda")
    fv.fvar_cache_factors(ctx, to_dev(Cm, "bf16"), _qt_dev(Q, "bf16"), False, B, M, r, 0.0, w_c, g_c, ws)
    torch.cuda.synchronize()
    for b in (0, 7):
        Wo, Go = factors.stored_factors(Cm[b], Q[0], bf16=True)
        assert rel_err(to_np(g_c[b]), Go) <= TOL["bf16"]
        assert rel_err(to_np(w_c[b]), Wo) <= TOL["bf16"]


@pytest.mark.parametrize("B,M,d,r", [(200, 256, 512, 64), (192, 304, 448, 72), (96, 512, 1024, 128)])
def test_cache_factors_many_samples(B, M, d, r):
    """The caches of all blocks of a scale in one call (hundreds of samples): the projection
    G_c = Q^T C and the product T = C G_c^T then run on the tiled MFMA kernel of the linear
    layers (k-major operand / batched fp32 output).  Three samples against the oracle."""
    Cm = wl.round_to_bf16(wl.cached_feature(B, M, d, max(8, r // 2), seed=4300 + r, noise=0.1))
    Q = _q(B, M, r, 4301 + r, "bf16", False)
    ctx = _ctx(d, "bf16")
    w_c = torch.full((B, M, r), float("nan"), dtype=torch.bfloat16, device="cuda")
    g_c = torch.full((B, r, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(fv.fvar_factors_workspace_bytes(ctx, B, M, r), dtype=torch.uint8, device="cuda")
    fv.fvar_cache_factors(ctx, to_dev(Cm, "bf16"), _qt_dev(Q, "bf16"), False, B, M, r, 0.0, w_c, g_c, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(w_c.float()).all() and torch.isfinite(g_c.float()).all()
    for b in (0, B // 3, B - 1):
        Wo, Go = factors.stored_factors(Cm[b], Q[0], bf16=True)
        assert rel_err(to_np(g_c[b]), Go) <= TOL["bf16"], (b, rel_err(to_np(g_c[b]), Go))
        assert rel_err(to_np(w_c[b]), Wo) <= TOL["bf16"], (b, rel_err(to_np(w_c[b]), Wo))
