"""GPU parity at the geometry each bf16 workload is named for: the late scales 48 and 64 of the
Infinity-2B-shaped model at batch 1 (long caches: the key axis of the attention and the
contraction axis of the O / FC2 layers are divided between workgroups), the same model at
batch 32 with the keep-ratio and rank sweep and on its larger scales, the 80x80 scale of the
4096-hidden shape at batch 4, and the STAR-shaped stand-in at its late scale.  The GPU runs the
benchmark's launch configuration (full batch); the oracle computes one or two samples element by
element, the other samples are checked through properties that hold at any size.  Bars as everywhere: indices bit-exact, bf16 outputs within 2e-2."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

from gpu_util import (GpuBlock, check_map, check_scores_and_indices, first_clean_seed, oracle_dense,  # noqa: E402
                      oracle_pruned, rel_err, report, to_dev, to_np)

BAR = 2e-2


def draw_inputs(W, side, B, seed):
    d, H, F = W.hidden, W.heads, W.ffn_hidden
    M, Lp = W.tokens(side), W.prev_len(side)
    draw = lambda sd: wl.activations_lowrank(B, M, d, seed=sd, bf16=True)
    x = draw(first_clean_seed(draw, "bf16", seed))
    w = wl.block_weights(d, F, seed=seed + 1000, bf16=True)
    Kp, Vp = wl.kv_prefix(B, Lp, H, d // H, seed=seed + 2000, bf16=True)
    return x, w, Kp, Vp


def check_other_samples(samples, s, keep_h, drop_h, y_h, yk_h, x, k, Wc, Gc, rng):
    """Properties that need no oracle block: exact selection from the GPU's own scores, kept rows
    of the map are the rows of y_keep, sampled restored rows equal the plain product."""
    for b in samples:
        check_scores_and_indices(to_np(s[b]), keep_h[b], drop_h[b], x[b], k)
        assert np.array_equal(y_h[b][keep_h[b]], yk_h[b])
        if drop_h.shape[1]:
            rows = rng.choice(drop_h[b], min(16, drop_h.shape[1]), replace=False)
            ref_rows = Wc[b][rows].astype(np.float64) @ Gc[b].astype(np.float64)
            assert rel_err(y_h[b][rows], ref_rows) <= BAR


def compare_sample(tag, b, blk, Lp, k, x, w, H, Kp, Vp, Wc, Gc, keep_h, drop_h, yk_h, y_h, whole=True):
    ref = oracle_pruned(x[b:b + 1], k, w, H, Kp[b:b + 1], Vp[b:b + 1], Wc[b:b + 1], Gc[b:b + 1])
    assert np.array_equal(keep_h[b], ref["idx_keep"][0])
    assert np.array_equal(drop_h[b], ref["idx_drop"][0])
    errs = dict(K_new=rel_err(to_np(blk.K[b, Lp:Lp + k]), ref["K_new"][0]),
                V_new=rel_err(to_np(blk.V[b, Lp:Lp + k]), ref["V_new"][0]),
                y_keep=rel_err(yk_h[b], ref["y_keep"][0]))
    report(f"{tag} sample {b}", **errs)
    for name, e in errs.items():
        assert e <= BAR, (tag, b, name, e)
    check_map(f"{tag} sample {b}", y_h[b], yk_h[b], keep_h[b], drop_h[b], ref["y"][0], BAR, whole=whole)


@pytest.mark.parametrize("side", [48, 64])
def test_infinity2b_late_scales_batch1(side):
    """Infinity-2B shape, batch 1, keep 0.3, rank 64: 692 / 1229 kept rows against 4121 / 6425
    cached rows.  Every output compared with the oracle; the dense control too at scale 48."""
    W = wl.WORKLOADS["infinity2b_1024_bf16"]
    B, d, H, F, r = 1, W.hidden, W.heads, W.ffn_hidden, W.rank
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    x, w, Kp, Vp = draw_inputs(W, side, B, 1100 + side)
    Wc, Gc = wl.direct_factors(B, M, r, d, seed=4100 + side, bf16=True)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, W.total_len(), scales=W.scales)
    xd = to_dev(x, "bf16")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
    torch.cuda.synchronize()
    keep_h, drop_h, y_h, yk_h = keep.cpu().numpy(), drop.cpu().numpy(), to_np(y), to_np(y_keep)
    check_other_samples([0], s, keep_h, drop_h, y_h, yk_h, x, k, Wc, Gc, np.random.default_rng(side))
    compare_sample(f"infinity2b s{side}", 0, blk, Lp, k, x, w, H, Kp, Vp, Wc, Gc, keep_h, drop_h,
                   yk_h, y_h)
    if side == 48:
        yo, Kn, Vn = oracle_dense(x, w, H, Kp, Vp)
        yd = blk.dense(xd)
        torch.cuda.synchronize()
        errs = dict(K_new=rel_err(to_np(blk.K[:, Lp:Lp + M]), Kn), y=rel_err(to_np(yd), yo))
        report(f"infinity2b s{side} dense", **errs)
        assert max(errs.values()) <= BAR


def test_infinity2b_batch32_keep_and_rank_sweep():
    """Infinity-2B shape at batch 16 x 2 (classifier-free-guidance doubling) on the 40x40 scale:
    keep ratio 1.0 / 0.5 / 0.3 / 0.2 at the benchmark's launch shape, one sample per ratio (two at
    0.3) against the oracle; keep 1.0 must also equal the dense call bit for bit; ranks 16 and
    128 of the fill at keep 0.3."""
    W = wl.WORKLOADS["infinity2b_1024_b32_bf16"]
    side = 40
    B, d, H, F = W.batch, W.hidden, W.heads, W.ffn_hidden
    M, Lp = W.tokens(side), W.prev_len(side)
    x, w, Kp, Vp = draw_inputs(W, side, B, 1200)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, Lp + M)
    xd = to_dev(x, "bf16")
    rng = np.random.default_rng(40)
    y_dense = blk.dense(xd)
    K_dense = blk.K.clone()
    torch.cuda.synchronize()
    for num, den, samples, r in [(1, 1, [3], 64), (1, 2, [9], 64), (3, 10, [0, 31], 64),
                                 (1, 5, [17], 64), (3, 10, [], 16), (3, 10, [], 128)]:
        k = max(1, -((-M * num) // den))
        Wc, Gc = wl.direct_factors(B, M, r, d, seed=4200 + r, bf16=True)
        s, keep, drop = blk.score_select(xd, k)
        y_keep = blk.pruned(xd, keep, k)
        y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
        torch.cuda.synchronize()
        keep_h, drop_h, y_h, yk_h = keep.cpu().numpy(), drop.cpu().numpy(), to_np(y), to_np(y_keep)
        assert np.isfinite(y_h).all()
        check_other_samples(range(B), s, keep_h, drop_h, y_h, yk_h, x, k, Wc, Gc, rng)
        for b in samples:
            compare_sample(f"infinity2b b32 s40 keep {num}/{den} r{r}", b, blk, Lp, k, x, w, H, Kp, Vp,
                           Wc, Gc, keep_h, drop_h, yk_h, y_h)
        if k == M:
            assert torch.equal(y, y_dense) and torch.equal(y_keep, y_dense)
            assert torch.equal(blk.K, K_dense)


@pytest.mark.parametrize("side", [48, 64])
def test_infinity2b_batch32_late_scales(side):
    """Infinity-2B shape at batch 32 on the 48x48 and 64x64 scales (22 144 / 39 328 rows through
    the linear layers, 4813 / 7654 keys): the benchmark's launch shape, one sample against the
    oracle, every sample through the properties that hold at any size."""
    W = wl.WORKLOADS["infinity2b_1024_b32_bf16"]
    B, d, H, F, r = W.batch, W.hidden, W.heads, W.ffn_hidden, W.rank
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    x, w, Kp, Vp = draw_inputs(W, side, B, 1400 + side)
    Wc, Gc = wl.direct_factors(B, M, r, d, seed=4400 + side, bf16=True)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, Lp + M)
    xd = to_dev(x, "bf16")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
    torch.cuda.synchronize()
    keep_h, drop_h, y_h, yk_h = keep.cpu().numpy(), drop.cpu().numpy(), to_np(y), to_np(y_keep)
    assert np.isfinite(y_h).all()
    check_other_samples(range(B), s, keep_h, drop_h, y_h, yk_h, x, k, Wc, Gc, np.random.default_rng(side))
    compare_sample(f"infinity2b b32 s{side}", 17, blk, Lp, k, x, w, H, Kp, Vp, Wc, Gc, keep_h, drop_h,
                   yk_h, y_h)


def test_star_shaped_scale64_batch4():
    """The STAR-shaped stand-in (hidden 2048, keep 22/125, rank 64) at its late scale, batch 4:
    721 kept rows of 4096 against 6425 cached rows, one sample against the oracle."""
    W = wl.WORKLOADS["star_shaped_1024_bf16"]
    side = 64
    B, d, H, F, r = W.batch, W.hidden, W.heads, W.ffn_hidden, W.rank
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    assert (M, k) == (4096, 721)
    x, w, Kp, Vp = draw_inputs(W, side, B, 1500)
    Wc, Gc = wl.direct_factors(B, M, r, d, seed=4500, bf16=True)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, W.total_len(), scales=W.scales)
    xd = to_dev(x, "bf16")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
    torch.cuda.synchronize()
    keep_h, drop_h, y_h, yk_h = keep.cpu().numpy(), drop.cpu().numpy(), to_np(y), to_np(y_keep)
    check_other_samples(range(B), s, keep_h, drop_h, y_h, yk_h, x, k, Wc, Gc, np.random.default_rng(64))
    compare_sample("star-shaped s64", 1, blk, Lp, k, x, w, H, Kp, Vp, Wc, Gc, keep_h, drop_h, yk_h, y_h)


def test_large_shape_scale80_batch4():
    """Hidden 4096, 32 heads of 128, rank 128, batch 4 at the 80x80 scale: 1600 kept rows of 6400
    against 10521 cached rows (12121 keys).  One sample against the oracle."""
    W = wl.WORKLOADS["large_1280_bf16"]
    side = 80
    B, d, H, F, r = W.batch, W.hidden, W.heads, W.ffn_hidden, W.rank
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    assert (M, Lp, k) == (6400, 10521, 1600)
    x, w, Kp, Vp = draw_inputs(W, side, B, 1300)
    Wc, Gc = wl.direct_factors(B, M, r, d, seed=4300, bf16=True)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, W.total_len(), scales=W.scales)
    xd = to_dev(x, "bf16")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
    torch.cuda.synchronize()
    keep_h, drop_h, y_h, yk_h = keep.cpu().numpy(), drop.cpu().numpy(), to_np(y), to_np(y_keep)
    check_other_samples(range(B), s, keep_h, drop_h, y_h, yk_h, x, k, Wc, Gc, np.random.default_rng(80))
    compare_sample("large s80", 2, blk, Lp, k, x, w, H, Kp, Vp, Wc, Gc, keep_h, drop_h, yk_h, y_h,
                   whole=False)
