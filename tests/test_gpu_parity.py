"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same seeded inputs.

Bars: indices bit-exact; bf16 outputs within 2e-2, fp32 outputs within 1e-4, both measured as
max_i |g_i - o_i| / max(|o_i|, rms(o))."""
import numpy as np
import pytest
import torch

import oracle
from oracle import factors
import workloads as wl

pytestmark = pytest.mark.gpu

from gpu_util import (TOL, GpuBlock, check_scores_and_indices, check_map, check_scores_of_map,  # noqa: E402
                      fill_scored, first_clean_seed,
                      oracle_dense, oracle_pruned, rel_err, report, tdtype, to_dev, to_np)


def same_scores(s, keep, drop, x, k, ref):
    """Scores bit-identical to the oracle's (the case's seed was chosen for that, see
    first_clean_seed) and the selection exact."""
    for b in range(x.shape[0]):
        check_scores_and_indices(to_np(s[b]), keep[b].cpu().numpy(), drop[b].cpu().numpy(), x[b], k)
    assert np.array_equal(to_np(s), ref["scores"])


def make_case(dtype, B, M, d, H, F, Lp, r, seed, std=None, bias=False, affine=False, noise=0.05,
              iid=False):
    """Inputs of one block step.  Small hidden sizes scale the weight std as 0.8/sqrt(d), which
    keeps the per-layer gain of the real workloads (0.02 * sqrt(1024..4096) = 0.64..1.28).
    The activations take the first seed (seed, seed+7919, ...) for which the GPU stores the same
    fp32 scores as the oracle; every other tensor is drawn from `seed` itself."""
    bf = dtype == "bf16"
    if std is None:
        std = 0.8 / np.sqrt(d)
    draw = lambda sd: (wl.activations_iid if iid else wl.activations_lowrank)(B, M, d, seed=sd, bf16=bf)
    x = draw(first_clean_seed(draw, dtype, seed))
    w = wl.block_weights(d, F, seed=seed + 1, bf16=bf, std=std, with_bias=bias, with_affine=affine)
    Kp, Vp = wl.kv_prefix(B, Lp, H, d // H, seed=seed + 2, bf16=bf)
    Cm = wl.cached_feature(B, M, d, r, seed=seed + 3, noise=noise)
    z = wl.normal_draws(B, M, r, seed=seed + 4)
    Wc = np.empty((B, M, r), np.float32)
    Gc = np.empty((B, r, d), np.float32)
    for b in range(B):
        Wc[b], Gc[b] = factors.cache_factors(Cm[b], z[b])
    if bf:
        Wc, Gc = wl.round_to_bf16(Wc), wl.round_to_bf16(Gc)
    return x, w, Kp, Vp, Wc, Gc


# ----------------------------------------------------------------------------- score + select
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,M,d", [(1, 1, 64), (2, 63, 128), (3, 257, 1920), (2, 1024, 2048),
                                   (1, 1600, 4096)])
def test_scores_and_indices_bitexact(dtype, B, M, d):
    x = wl.activations_lowrank(B, M, d, seed=17 + M, bf16=dtype == "bf16")
    blk = GpuBlock(d, d // 64, 64 * 4, dtype, {}, np.zeros((B, 0, d // 64, 64), np.float32),
                   np.zeros((B, 0, d // 64, 64), np.float32), 1)
    xd = to_dev(x, dtype)
    for k in sorted({1, max(1, M // 3), M}):
        s, keep, drop = blk.score_select(xd, k)
        torch.cuda.synchronize()
        for b in range(B):
            check_scores_and_indices(to_np(s[b]), keep[b].cpu().numpy(), drop[b].cpu().numpy(), x[b], k)


@pytest.mark.parametrize("M", [1, 2, 64, 65, 1000, 1024, 1025, 6400, 12288, 13001])
def test_select_on_given_scores(M):
    rng = np.random.default_rng(M)
    blk = GpuBlock(64, 1, 64, "f32", {}, np.zeros((1, 0, 1, 64), np.float32),
                   np.zeros((1, 0, 1, 64), np.float32), 1)
    cases = [rng.standard_normal(M).astype(np.float32) ** 2,
             np.full(M, 3.25, np.float32),                                  # all equal
             np.round(rng.standard_normal(M) * 2).astype(np.float32),       # heavy ties, negatives, +-0
             np.arange(M, dtype=np.float32),                                # ascending
             -np.arange(M, dtype=np.float32),                               # descending
             (rng.integers(0, 3, M) * 1e-30).astype(np.float32)]            # tiny values, many ties
    cases[2][::7] = -0.0
    S = np.stack(cases)
    B = S.shape[0]
    sd = torch.from_numpy(S).cuda()
    for k in sorted({1, 2, M // 2, M - 1, M} - {0}):
        if k > M:
            continue
        _, keep, drop = blk.score_select(torch.empty((B, M, 64), device="cuda"), k, scores_in=sd)
        torch.cuda.synchronize()
        for b in range(B):
            ko, do = oracle.topk(S[b], k)
            assert np.array_equal(keep[b].cpu().numpy(), ko), (M, k, b)
            assert np.array_equal(drop[b].cpu().numpy(), do), (M, k, b)


# ----------------------------------------------------------------------------- fill
@pytest.mark.parametrize("dtype,r", [("bf16", 8), ("bf16", 64), ("bf16", 72), ("bf16", 128),
                                     ("bf16", 256), ("f32", 4), ("f32", 32), ("f32", 100)])
@pytest.mark.parametrize("M,d,k", [(300, 1920, 120), (64, 128, 1), (129, 256, 129), (130, 192, 0)])
def test_lowrank_fill(dtype, r, M, d, k):
    bf = dtype == "bf16"
    B = 2
    rng = np.random.default_rng(r + M)
    Wc = rng.standard_normal((B, M, r)).astype(np.float32)
    Gc = (rng.standard_normal((B, r, d)) / np.sqrt(r)).astype(np.float32)
    yk = rng.standard_normal((B, k, d)).astype(np.float32)
    if bf:
        Wc, Gc, yk = wl.round_to_bf16(Wc), wl.round_to_bf16(Gc), wl.round_to_bf16(yk)
    keep = np.stack([np.sort(rng.permutation(M)[:k]) for _ in range(B)]).astype(np.int32).reshape(B, k)
    drop = np.stack([np.setdiff1d(np.arange(M), keep[b]) for b in range(B)]).astype(np.int32)
    blk = GpuBlock(d, d // 64, 256, dtype, {}, np.zeros((B, 0, d // 64, 64), np.float32),
                   np.zeros((B, 0, d // 64, 64), np.float32), 1)
    y = blk.fill(to_dev(yk, dtype), torch.from_numpy(keep).cuda(), torch.from_numpy(drop).cuda(), M,
                 to_dev(Wc, dtype), to_dev(Gc, dtype))
    torch.cuda.synchronize()
    y = to_np(y)
    assert np.isfinite(y).all(), "some row was never written"
    for b in range(B):
        ref = oracle.lowrank_fill(yk[b], keep[b], drop[b], M, Wc[b], Gc[b])
        assert np.array_equal(y[b][keep[b]], yk[b])                       # kept rows are copies
        assert rel_err(y[b], ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype,r,M,d,k", [("bf16", 64, 300, 1920, 120), ("bf16", 128, 700, 4096, 200),
                                           ("bf16", 8, 129, 256, 129), ("bf16", 24, 130, 192, 0),
                                           ("bf16", 200, 97, 320, 5), ("f32", 32, 200, 1024, 77),
                                           ("f32", 4, 64, 128, 64)])
def test_lowrank_fill_scored(dtype, r, M, d, k):
    """The restoration that also reports the row energies of the map it writes: same map as the
    plain call bit for bit, and scores equal to the oracle's scores of that stored map."""
    bf = dtype == "bf16"
    B = 3
    rng = np.random.default_rng(7 * r + M)
    Wc = rng.standard_normal((B, M, r)).astype(np.float32)
    Gc = (rng.standard_normal((B, r, d)) / np.sqrt(r)).astype(np.float32)
    yk = (rng.standard_normal((B, k, d)) * np.exp(rng.standard_normal((B, k, 1)))).astype(np.float32)
    if bf:
        Wc, Gc, yk = wl.round_to_bf16(Wc), wl.round_to_bf16(Gc), wl.round_to_bf16(yk)
    keep = np.stack([np.sort(rng.permutation(M)[:k]) for _ in range(B)]).astype(np.int32).reshape(B, k)
    drop = np.stack([np.setdiff1d(np.arange(M), keep[b]) for b in range(B)]).astype(np.int32)
    blk = GpuBlock(d, d // 64, 256, dtype, {}, np.zeros((B, 0, d // 64, 64), np.float32),
                   np.zeros((B, 0, d // 64, 64), np.float32), 1)
    args = (to_dev(yk, dtype), torch.from_numpy(keep).cuda(), torch.from_numpy(drop).cuda(), M,
            to_dev(Wc, dtype), to_dev(Gc, dtype))
    y_plain = blk.fill(*args)
    y, scores = fill_scored(blk, *args)
    torch.cuda.synchronize()
    assert torch.equal(y, y_plain)
    yh, sh = to_np(y), to_np(scores)
    assert np.isfinite(sh).all()
    for b in range(B):
        check_scores_of_map(sh[b], yh[b])
        ref = oracle.lowrank_fill(yk[b], keep[b], drop[b], M, Wc[b], Gc[b])
        assert rel_err(yh[b], ref) <= TOL[dtype]
    # the next block's selection from these scores is the oracle's selection on the stored map
    kk = max(1, M // 3)
    s2, keep2, drop2 = blk.score_select(y, kk)
    _, keep3, drop3 = blk.score_select(y, kk, scores_in=scores)
    torch.cuda.synchronize()
    for b in range(B):
        ko, do = oracle.topk(sh[b], kk)
        assert np.array_equal(keep3[b].cpu().numpy(), ko) and np.array_equal(drop3[b].cpu().numpy(), do)
        so = oracle.scores(yh[b])
        if np.array_equal(so, sh[b]):
            k2, d2 = oracle.topk(so, kk)
            assert np.array_equal(ko, k2) and np.array_equal(do, d2)
    if np.array_equal(to_np(s2), sh):
        assert torch.equal(keep2, keep3) and torch.equal(drop2, drop3)


# ----------------------------------------------------------------------------- block, small shapes
SMALL = [  # dtype, B, M, d, H, F, Lp, k, r
    ("bf16", 2, 96, 128, 2, 256, 37, 40, 16),
    ("bf16", 1, 300, 256, 2, 512, 129, 131, 32),     # head_dim 128, ragged tiles
    ("bf16", 3, 70, 256, 4, 320, 1, 1, 8),           # one kept row, one cached key
    ("bf16", 1, 200, 384, 6, 768, 500, 200, 24),     # keep everything
    ("f32", 2, 96, 128, 2, 256, 37, 40, 16),
    ("f32", 1, 150, 256, 2, 512, 65, 33, 8),         # head_dim 128
    ("bf16", 2, 130, 192, 3, 448, 0, 67, 16),        # empty cache prefix: only the new rows are keys
    ("bf16", 3, 520, 256, 2, 1024, 300, 257, 64),    # head_dim 128, several samples, k just over a tile
    ("f32", 1, 64, 64, 1, 64, 0, 64, 4),             # smallest geometry, nothing cached, keep all
    ("bf16", 1, 160, 256, 2, 512, 1500, 64, 16),     # batch 1, long cache: key axis split 5 ways (head_dim 128)
    ("bf16", 1, 300, 128, 2, 256, 1000, 150, 16),    # the same with head_dim 64 and two query blocks per wavefront
    ("bf16", 1, 256, 1024, 16, 4096, 424, 128, 32),  # few tiles, long contraction: linear layers split along k
    # many rows, wide MLP, contraction of one, two and three 64-wide k-tiles: the big-tile GEMM
    # configurations with a pipeline shorter than their ring of stages
    ("bf16", 2, 1600, 64, 1, 2048, 10, 1500, 8),
    ("bf16", 2, 1600, 128, 1, 3072, 10, 1500, 8),
    ("bf16", 2, 1400, 192, 3, 2304, 70, 1300, 8),
]


@pytest.mark.parametrize("dtype,B,M,d,H,F,Lp,k,r", SMALL)
@pytest.mark.parametrize("extras", [False, True])
def test_pruned_path_small(dtype, B, M, d, H, F, Lp, k, r, extras):
    x, w, Kp, Vp, Wc, Gc = make_case(dtype, B, M, d, H, F, Lp, r, seed=100 + M,
                                     bias=extras, affine=extras)
    ref = oracle_pruned(x, k, w, H, Kp, Vp, Wc, Gc)
    blk = GpuBlock(d, H, F, dtype, w, Kp, Vp, Lp + M)
    xd = to_dev(x, dtype)
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, dtype), to_dev(Gc, dtype))
    torch.cuda.synchronize()
    same_scores(s, keep, drop, x, k, ref)
    assert np.array_equal(keep.cpu().numpy(), ref["idx_keep"])
    assert np.array_equal(drop.cpu().numpy(), ref["idx_drop"])
    tol = TOL[dtype]
    assert rel_err(to_np(blk.K[:, Lp:Lp + k]), ref["K_new"]) <= tol
    assert rel_err(to_np(blk.V[:, Lp:Lp + k]), ref["V_new"]) <= tol
    assert rel_err(to_np(y_keep), ref["y_keep"]) <= tol
    for b in range(B):
        check_map(f"b{b}", to_np(y[b]), to_np(y_keep[b]), ref["idx_keep"][b], ref["idx_drop"][b],
                  ref["y"][b], tol)
    assert np.array_equal(to_np(blk.K[:, :Lp]), Kp)                        # prefix untouched


@pytest.mark.parametrize("dtype,B,M,d,H,F,Lp,k,r", SMALL[:2] + SMALL[4:5])
def test_dense_block_small_and_keep_all(dtype, B, M, d, H, F, Lp, k, r):
    x, w, Kp, Vp, Wc, Gc = make_case(dtype, B, M, d, H, F, Lp, r, seed=300 + M, bias=True)
    yo, Kn, Vn = oracle_dense(x, w, H, Kp, Vp)
    blk = GpuBlock(d, H, F, dtype, w, Kp, Vp, Lp + M)
    xd = to_dev(x, dtype)
    y = blk.dense(xd)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_err(to_np(y), yo) <= tol
    assert rel_err(to_np(blk.K[:, Lp:]), Kn) <= tol and rel_err(to_np(blk.V[:, Lp:]), Vn) <= tol
    # keep ratio 1.0: the pruned entry point with every row kept gives the dense result bit for bit
    blk2 = GpuBlock(d, H, F, dtype, w, Kp, Vp, Lp + M)
    _, keep, drop = blk2.score_select(xd, M)
    assert np.array_equal(keep.cpu().numpy(), np.tile(np.arange(M, dtype=np.int32), (B, 1)))
    y2 = blk2.pruned(xd, keep, M)
    y3 = blk2.fill(y2, keep, drop, M, None, None)
    torch.cuda.synchronize()
    assert torch.equal(y2, y) and torch.equal(y3, y)
    assert torch.equal(blk2.K, blk.K) and torch.equal(blk2.V, blk.V)


@pytest.mark.parametrize("case", [1, 9, 11])     # plain; key axis of the attention split; linear layers split along k
def test_runs_are_deterministic(case):
    dtype, B, M, d, H, F, Lp, k, r = SMALL[case]
    x, w, Kp, Vp, Wc, Gc = make_case(dtype, B, M, d, H, F, Lp, r, seed=7)
    outs = []
    for _ in range(2):
        blk = GpuBlock(d, H, F, dtype, w, Kp, Vp, Lp + M)
        xd = to_dev(x, dtype)
        _, keep, drop = blk.score_select(xd, k)
        y = blk.fill(blk.pruned(xd, keep, k), keep, drop, M, to_dev(Wc, dtype), to_dev(Gc, dtype))
        torch.cuda.synchronize()
        outs.append((y.clone(), blk.K.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("H,k", [(4, 4200), (4, 4300), (2, 4200)])
def test_attention_last_round_divided_between_workgroups(H, k):
    """Many (query block, head, sample) triples whose count is just above a multiple of what the
    chip holds at once: the triples of the last round of workgroups are divided along the key
    axis and merged.  Three kernel variants (head_dim 64 with one and two query blocks per
    wavefront, head_dim 128); every sample is compared with the oracle, the divided triples are
    those of the last sample."""
    dtype, B, d, F, Lp, r = "bf16", 8, 256, 256, 2100, 8
    M = k + 50
    x, w, Kp, Vp, Wc, Gc = make_case(dtype, B, M, d, H, F, Lp, r, seed=900 + k + H)
    ref = oracle_pruned(x, k, w, H, Kp, Vp, Wc, Gc)
    blk = GpuBlock(d, H, F, dtype, w, Kp, Vp, Lp + M)
    xd = to_dev(x, dtype)
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    torch.cuda.synchronize()
    same_scores(s, keep, drop, x, k, ref)
    for b in range(B):
        e = rel_err(to_np(y_keep[b]), ref["y_keep"][b])
        assert e <= TOL[dtype], (b, e)
    assert rel_err(to_np(blk.K[:, Lp:Lp + k]), ref["K_new"]) <= TOL[dtype]


# ----------------------------------------------------------------------------- real shapes
def test_var_d16_last_scale_fp32_full():
    """The fp32 configuration at its full size: 256 tokens, 424 cached rows, keep 0.5, r = 32."""
    W = wl.WORKLOADS["var_d16_s16_f32"]
    side = 16
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    x, w, Kp, Vp, Wc, Gc = make_case("f32", 1, M, W.hidden, W.heads, W.ffn_hidden, Lp, W.rank,
                                     seed=1000, std=0.02, iid=True)
    ref = oracle_pruned(x, k, w, W.heads, Kp, Vp, Wc, Gc)
    blk = GpuBlock(W.hidden, W.heads, W.ffn_hidden, "f32", w, Kp, Vp, W.total_len(), scales=W.scales)
    xd = to_dev(x, "f32")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "f32"), to_dev(Gc, "f32"))
    torch.cuda.synchronize()
    same_scores(s, keep, drop, x, k, ref)
    assert np.array_equal(keep.cpu().numpy(), ref["idx_keep"])
    assert np.array_equal(drop.cpu().numpy(), ref["idx_drop"])
    assert rel_err(to_np(y_keep), ref["y_keep"]) <= 1e-4
    check_map("var_d16 fp32", to_np(y[0]), to_np(y_keep[0]), ref["idx_keep"][0], ref["idx_drop"][0],
              ref["y"][0], 1e-4)
    yd, _, _ = oracle_dense(x, w, W.heads, Kp, Vp)
    blkd = GpuBlock(W.hidden, W.heads, W.ffn_hidden, "f32", w, Kp, Vp, W.total_len())
    assert rel_err(to_np(blkd.dense(xd)), yd) <= 1e-4


@pytest.mark.parametrize("side", [24, 32])
def test_var_d30_full_batch_launch_shape(side):
    """The benchmark's launch configuration (batch 8, hidden 1920, 30 heads).  One sample is
    compared element by element with the oracle; the others through properties that hold at any
    size (partition, scatter copies, fill rows against the plain product)."""
    W = wl.WORKLOADS["var_d30_512_bf16"]
    B, d, H, F, r = W.batch, W.hidden, W.heads, W.ffn_hidden, W.rank
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    bf = True
    x = wl.activations_lowrank(B, M, d, seed=1002, bf16=bf)
    w = wl.block_weights(d, F, seed=2000, bf16=bf)
    Kp, Vp = wl.kv_prefix(B, Lp, H, d // H, seed=3000, bf16=bf)
    Wc, Gc = wl.direct_factors(B, M, r, d, seed=4000, bf16=bf)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, W.total_len(), scales=W.scales)
    xd = to_dev(x, "bf16")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
    torch.cuda.synchronize()
    keep_h, drop_h, y_h, yk_h = keep.cpu().numpy(), drop.cpu().numpy(), to_np(y), to_np(y_keep)
    rng = np.random.default_rng(side)
    for b in range(B):
        check_scores_and_indices(to_np(s[b]), keep_h[b], drop_h[b], x[b], k)
        assert np.array_equal(y_h[b][keep_h[b]], yk_h[b])
        rows = rng.choice(drop_h[b], 16, replace=False)
        ref_rows = Wc[b][rows].astype(np.float64) @ Gc[b].astype(np.float64)
        assert rel_err(y_h[b][rows], ref_rows) <= 2e-2
    b = 5
    ref = oracle_pruned(x[b:b + 1], k, w, H, Kp[b:b + 1], Vp[b:b + 1], Wc[b:b + 1], Gc[b:b + 1])
    assert rel_err(to_np(blk.K[b, Lp:Lp + k]), ref["K_new"][0]) <= 2e-2
    assert rel_err(yk_h[b], ref["y_keep"][0]) <= 2e-2
    check_map(f"var_d30 s{side}", y_h[b], yk_h[b], ref["idx_keep"][0], ref["idx_drop"][0], ref["y"][0], 2e-2)


@pytest.mark.parametrize("name,side,B", [("infinity2b_1024_bf16", 40, 1), ("large_1280_bf16", 40, 1)])
def test_head_dim_128_workloads_real_shape(name, side, B):
    """Infinity-2B-shaped (hidden 2048, 16 heads of 128) and large-model-shaped (hidden 4096,
    32 heads of 128, rank 128) blocks at the 40x40 scale with their real cache prefix (2521 rows):
    one sample, every output compared with the oracle."""
    W = wl.WORKLOADS[name]
    d, H, F, r = W.hidden, W.heads, W.ffn_hidden, W.rank
    M, Lp, k = W.tokens(side), W.prev_len(side), W.keep(side)
    draw = lambda sd: wl.activations_lowrank(B, M, d, seed=sd, bf16=True)
    x = draw(first_clean_seed(draw, "bf16", 1003))
    w = wl.block_weights(d, F, seed=2003, bf16=True)
    Kp, Vp = wl.kv_prefix(B, Lp, H, d // H, seed=3003, bf16=True)
    Wc, Gc = wl.direct_factors(B, M, r, d, seed=4003, bf16=True)
    blk = GpuBlock(d, H, F, "bf16", w, Kp, Vp, Lp + M)
    xd = to_dev(x, "bf16")
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, "bf16"), to_dev(Gc, "bf16"))
    torch.cuda.synchronize()
    ref = oracle_pruned(x, k, w, H, Kp, Vp, Wc, Gc)
    same_scores(s, keep, drop, x, k, ref)
    assert np.array_equal(keep.cpu().numpy(), ref["idx_keep"])
    assert rel_err(to_np(blk.K[:, Lp:Lp + k]), ref["K_new"]) <= 2e-2
    assert rel_err(to_np(blk.V[:, Lp:Lp + k]), ref["V_new"]) <= 2e-2
    report(f"{name} s{side}", K_new=rel_err(to_np(blk.K[:, Lp:Lp + k]), ref["K_new"]),
           V_new=rel_err(to_np(blk.V[:, Lp:Lp + k]), ref["V_new"]),
           y_keep=rel_err(to_np(y_keep), ref["y_keep"]))
    assert rel_err(to_np(y_keep), ref["y_keep"]) <= 2e-2
    for b in range(B):
        check_map(f"{name} s{side}", to_np(y[b]), to_np(y_keep[b]), ref["idx_keep"][b], ref["idx_drop"][b],
                  ref["y"][b], 2e-2, whole=W.hidden < 4096)


# ----------------------------------------------------------------------------- random geometry
@pytest.mark.parametrize("seed", range(12))
def test_pruned_path_random_geometry(seed):
    """Seeded random geometry inside the documented limits (head_dim 64 or 128, 1-4 heads, ragged
    token counts, cache prefixes around the 64-key tile edges, any keep count): same bar."""
    rng = np.random.default_rng(5000 + seed)
    dtype = "bf16" if seed % 4 else "f32"
    Dh, H = int(rng.choice([64, 128])), int(rng.integers(1, 5))
    d = H * Dh
    F = int(rng.choice([64, 128, 192, 256, 512])) * int(rng.integers(1, 4))
    r = int(rng.choice([4, 8, 12, 32])) if dtype == "f32" else int(rng.choice([8, 16, 24, 64]))
    B, M = int(rng.integers(1, 4)), max(r, int(rng.integers(1, 400)))
    k = int(rng.integers(1, M + 1))
    Lp = int(rng.choice([0, 1, 63, 64, 65, 200, 700, 1300]))
    x, w, Kp, Vp, Wc, Gc = make_case(dtype, B, M, d, H, F, Lp, r, seed=6000 + seed,
                                     bias=bool(seed & 1), affine=bool(seed & 2))
    ref = oracle_pruned(x, k, w, H, Kp, Vp, Wc, Gc)
    blk = GpuBlock(d, H, F, dtype, w, Kp, Vp, Lp + M)
    xd = to_dev(x, dtype)
    s, keep, drop = blk.score_select(xd, k)
    y_keep = blk.pruned(xd, keep, k)
    y = blk.fill(y_keep, keep, drop, M, to_dev(Wc, dtype), to_dev(Gc, dtype))
    torch.cuda.synchronize()
    same_scores(s, keep, drop, x, k, ref)
    assert np.array_equal(keep.cpu().numpy(), ref["idx_keep"])
    assert np.array_equal(drop.cpu().numpy(), ref["idx_drop"])
    tol = TOL[dtype]
    assert rel_err(to_np(blk.K[:, Lp:Lp + k]), ref["K_new"]) <= tol
    assert rel_err(to_np(blk.V[:, Lp:Lp + k]), ref["V_new"]) <= tol
    assert rel_err(to_np(y_keep), ref["y_keep"]) <= tol
    for b in range(B):
        check_map(f"b{b}", to_np(y[b]), to_np(y_keep[b]), ref["idx_keep"][b], ref["idx_drop"][b],
                  ref["y"][b], tol)
