"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only)."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import factors
import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


# ----------------------------------------------------------------------------- schedules
def _golden():
    sched, keeps = {}, []
    for line in open(os.path.join(HERE, "golden", "scale_schedules.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [t.strip() for t in line.split(";")]
        if f[0] == "keep":
            num, den = f[2].split("/")
            keeps.append((int(f[1]), int(num), int(den), int(f[3])))
        else:
            sched[f[0]] = (tuple(int(s) for s in f[1].split(",")), int(f[2]),
                           {int(a.split(":")[0]): int(a.split(":")[1]) for a in f[3].split(",")})
    return sched, keeps


def test_scale_schedules_and_keep_counts():
    sched, keeps = _golden()
    names = {"infinity_1024": "infinity2b_1024_bf16", "var_d16_256": "var_d16_s16_f32",
             "var_d30_512": "var_d30_512_bf16", "large_1280": "large_1280_bf16"}
    for g, n in names.items():
        sides, total, prev = sched[g]
        w = wl.WORKLOADS[n]
        assert w.scales == sides and w.total_len() == total
        for side, lp in prev.items():
            assert w.prev_len(side) == lp
    for M, num, den, k in keeps:
        assert oracle.keep_count(M, num, den) == k
    # a float ceil of 0.3f * 1600 would give 481; the rational form must not
    assert oracle.keep_count(1600, 3, 10) == 480
    assert oracle.keep_count(10, 0, 1) == 1 and oracle.keep_count(10, 5, 1) == 10
    for w in wl.WORKLOADS.values():
        for s in w.late_scales:
            assert w.keep(s) == oracle.keep_count(s * s, w.keep_num, w.keep_den)


# ----------------------------------------------------------------------------- scores
def test_scores_closed_forms():
    d = 96
    x = np.zeros((5, d), np.float32)
    x[0, 3] = 1.0                       # one-hot -> 1
    x[1, :] = 0.5                       # constant c -> d c^2
    x[2, :] = -2.0
    x[3, 7] = 3.0; x[3, 8] = 4.0        # 3-4-5
    s = oracle.scores(x)
    assert s.tolist() == [1.0, d * 0.25, d * 4.0, 25.0, 0.0]


def test_scores_are_correctly_rounded_and_order_free():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((64, 1000)).astype(np.float32)
    # math.fsum gives the exactly rounded sum of the (exact) fp64 products
    import math
    s = oracle.scores(x)
    for i in range(64):
        ex = np.float32(math.fsum(float(v) * float(v) for v in x[i]))
        assert s[i] == ex
    perm = rng.permutation(1000)
    assert np.array_equal(oracle.scores(x[:, perm]), s)


def test_importance_is_a_distribution():
    x = wl.activations_lowrank(1, 200, 64, seed=3)[0]
    s = oracle.scores(x)
    P = oracle.importance(s)
    assert np.all(P >= 0) and abs(float(P.astype(np.float64).sum()) - 1.0) < 1e-6
    # proportional to the row energy: same ordering as the scores
    assert np.array_equal(np.argsort(-P, kind="stable"), np.argsort(-s, kind="stable"))


# ----------------------------------------------------------------------------- top-k
def _brute_topk(s, k):
    order = sorted(range(len(s)), key=lambda i: (-float(s[i]), i))
    keep = sorted(order[:k])
    drop = sorted(order[k:])
    return np.array(keep, np.int32), np.array(drop, np.int32)


@pytest.mark.parametrize("M", [1, 2, 7, 33, 64])
def test_topk_bruteforce(M):
    rng = np.random.default_rng(M)
    for trial in range(20):
        s = rng.standard_normal(M).astype(np.float32) ** 2
        if trial % 3 == 1:                                   # heavy ties
            s = np.round(s * 2).astype(np.float32)
        if trial % 3 == 2:                                   # duplicated values
            s[rng.integers(0, M, M // 2 + 1)] = s[0]
        for k in sorted({0, 1, M // 2, max(M - 1, 0), M}):
            keep, drop = oracle.topk(s, k)
            bk, bd = _brute_topk(s, k)
            assert np.array_equal(keep, bk) and np.array_equal(drop, bd)


def test_topk_special_cases():
    s = np.full(16, 2.5, np.float32)
    keep, drop = oracle.topk(s, 5)                           # all equal -> lowest indices
    assert keep.tolist() == [0, 1, 2, 3, 4] and drop.tolist() == list(range(5, 16))
    s = np.array([1, 9, 3, 9, 2], np.float32)
    assert oracle.topk(s, 1)[0].tolist() == [1]              # argmax, lowest index among ties
    assert oracle.topk(s, 5)[0].tolist() == [0, 1, 2, 3, 4]
    keep, drop = oracle.topk(s, 3)
    assert keep.tolist() == [1, 2, 3] and drop.tolist() == [0, 4]
    z = np.array([0.0, -0.0, 0.0], np.float32)               # signed zeros tie
    assert oracle.topk(z, 2)[0].tolist() == [0, 1]


# ----------------------------------------------------------------------------- block pieces
def test_layernorm_moments_and_affine():
    rng = np.random.default_rng(1)
    x = (3.0 + 2.0 * rng.standard_normal((9, 512))).astype(np.float32)
    eps = 1e-6
    u = oracle.layernorm(x, eps=eps).astype(np.float64)
    var = x.astype(np.float64).var(axis=1)
    assert np.abs(u.mean(axis=1)).max() < 1e-7
    assert np.allclose(u.var(axis=1), var / (var + eps), rtol=1e-6)
    g = rng.standard_normal(512).astype(np.float32)
    b = rng.standard_normal(512).astype(np.float32)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (512,),
                                         torch.from_numpy(g).double(),
                                         torch.from_numpy(b).double(), eps).numpy()
    assert np.abs(oracle.layernorm(x, g, b, eps) - ref).max() < 1e-6
    # eps matters when the variance is tiny
    c = np.full((1, 64), 5.0, np.float32); c[0, 0] += 1e-3
    v = c.astype(np.float64).var()
    assert np.allclose(oracle.layernorm(c, eps=1e-6).astype(np.float64).var(), v / (v + 1e-6), rtol=1e-3)


def test_linear_matches_fp64_matmul_and_layout():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 33)).astype(np.float32)
    W = rng.standard_normal((19, 33)).astype(np.float32)      # [out,in]
    b = rng.standard_normal(19).astype(np.float32)
    ref = x.astype(np.float64) @ W.astype(np.float64).T + b
    y = oracle.linear(x, W, b)
    assert y.shape == (7, 19) and np.abs(y - ref).max() <= 1e-6 * np.abs(ref).max()
    e = np.zeros((1, 33), np.float32); e[0, 4] = 1.0          # picks column 4 of W
    assert np.array_equal(oracle.linear(e, W)[0], W[:, 4])


def test_gelu_tanh_values():
    x = np.array([0.0, 1.0, -1.0, 6.0, -6.0, 0.5], np.float32)
    y = oracle.gelu_tanh(x)
    ref = torch.nn.functional.gelu(torch.from_numpy(x).double(), approximate="tanh").numpy()
    assert np.abs(y - ref).max() < 1e-7
    assert y[0] == 0.0 and abs(y[3] - 6.0) < 1e-6 and abs(y[4]) < 1e-6
    assert abs(y[1] - 0.841192) < 1e-6                        # textbook value of the tanh form at 1


# ----------------------------------------------------------------------------- attention
def _rand_qkv(n, L, H, Dh, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, H, Dh)).astype(np.float32),
            rng.standard_normal((L, H, Dh)).astype(np.float32),
            rng.standard_normal((L, H, Dh)).astype(np.float32))


def test_attention_rows_sum_to_one_and_special_caches():
    q, K, V = _rand_qkv(5, 37, 3, 16, 0)
    o, lse, ps = oracle.attention(q, K, V, want_stats=True)
    assert np.abs(ps - 1.0).max() <= 1e-6 * 37
    # a single cached key: output is its value row
    o1 = oracle.attention(q, K[:1], V[:1])
    assert np.abs(o1 - V[:1]).max() < 1e-7
    # all keys equal: output is the mean of the values
    Ke = np.repeat(K[:1], 37, axis=0)
    oe = oracle.attention(q, Ke, V)
    assert np.abs(oe - V.astype(np.float64).mean(axis=0)[None]).max() < 1e-6
    # adding a constant vector to every key shifts every logit of a row equally
    shift = np.random.default_rng(5).standard_normal((1, 3, 16)).astype(np.float32)
    os_ = oracle.attention(q, K + shift, V)
    assert np.abs(os_ - o).max() < 2e-5


def test_attention_matches_fp64_library_routine():
    q, K, V = _rand_qkv(11, 53, 4, 32, 1)
    tq, tK, tV = (torch.from_numpy(a).double().permute(1, 0, 2) for a in (q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(tq[None], tK[None], tV[None])[0]
    ref = ref.permute(1, 0, 2).numpy()
    o = oracle.attention(q, K, V)
    assert np.abs(o - ref).max() < 1e-6
    o2 = oracle.attention(q, K, V, scale=0.3)
    ref2 = torch.nn.functional.scaled_dot_product_attention(tq[None], tK[None], tV[None], scale=0.3)[0]
    assert np.abs(o2 - ref2.permute(1, 0, 2).numpy()).max() < 1e-6


def test_split_kv_merge_by_lse():
    q, K, V = _rand_qkv(6, 80, 2, 16, 2)
    o, lse, _ = oracle.attention(q, K, V, want_stats=True)
    oa, la, _ = oracle.attention(q, K[:30], V[:30], want_stats=True)
    ob, lb, _ = oracle.attention(q, K[30:], V[30:], want_stats=True)
    m = np.maximum(la, lb).astype(np.float64)
    wa, wb = np.exp(la - m), np.exp(lb - m)
    merged = (wa[..., None] * oa + wb[..., None] * ob) / (wa + wb)[..., None]
    assert np.abs(merged - o).max() < 1e-5
    assert np.abs((m + np.log(wa + wb)) - lse).max() < 1e-5


def _torch_block(x, w, H, Kp, Vp, eps=1e-6):
    """Independent fp64 statement of the block with library routines (cross-check only)."""
    F = torch.nn.functional
    t = lambda a: None if a is None else torch.from_numpy(np.asarray(a)).double()
    x = t(x); n, d = x.shape; Dh = d // H
    u = F.layer_norm(x, (d,), t(w.ln1_g), t(w.ln1_b), eps)
    qkv = F.linear(u, t(w.w_qkv), t(w.b_qkv))
    q, kk, v = qkv.split(d, dim=1)
    Kall = torch.cat([t(Kp).reshape(-1, d), kk]).reshape(-1, H, Dh)
    Vall = torch.cat([t(Vp).reshape(-1, d), v]).reshape(-1, H, Dh)
    o = F.scaled_dot_product_attention(q.reshape(n, H, Dh).permute(1, 0, 2)[None],
                                       Kall.permute(1, 0, 2)[None], Vall.permute(1, 0, 2)[None])[0]
    o = o.permute(1, 0, 2).reshape(n, d)
    h1 = x + F.linear(o, t(w.w_o), t(w.b_o))
    u2 = F.layer_norm(h1, (d,), t(w.ln2_g), t(w.ln2_b), eps)
    y = h1 + F.linear(F.gelu(F.linear(u2, t(w.w_fc1), t(w.b_fc1)), approximate="tanh"),
                      t(w.w_fc2), t(w.b_fc2))
    return y.numpy(), kk.numpy(), v.numpy()


@pytest.mark.parametrize("full", [False, True])
def test_dense_block_matches_fp64_framework(full):
    if full:      # the fp32 parity configuration at its real shape (dense: all 256 rows)
        w_ = wl.WORKLOADS["var_d16_s16_f32"]
        d, H, Fh, n, Lp = w_.hidden, w_.heads, w_.ffn_hidden, 256, w_.prev_len(16)
        wd = wl.block_weights(d, Fh, seed=2000)
    else:         # small, with biases and LayerNorm affine switched on
        d, H, Fh, n, Lp = 64, 4, 160, 9, 13
        wd = wl.block_weights(d, Fh, seed=7, with_bias=True, with_affine=True, std=0.2)
    w = oracle.BlockWeights(**wd)
    x = wl.activations_iid(1, n, d, seed=1000)[0]
    Kp, Vp = wl.kv_prefix(1, Lp, H, d // H, seed=3000)
    Kc = np.zeros((Lp + n, H, d // H), np.float32); Vc = np.zeros_like(Kc)
    Kc[:Lp], Vc[:Lp] = Kp[0], Vp[0]
    y = oracle.block_forward(x, w, H, Kc, Vc, Lp)
    ref, kk, v = _torch_block(x, w, H, Kp[0], Vp[0])
    scale = max(np.abs(ref).max(), 1.0)
    assert np.abs(y - ref).max() / scale < 2e-6
    assert np.abs(Kc[Lp:].reshape(n, d) - kk).max() < 1e-5
    assert np.abs(Vc[Lp:].reshape(n, d) - v).max() < 1e-5
    assert np.array_equal(Kc[:Lp], Kp[0])                     # prefix untouched


def test_block_causal_mask_equals_incremental_cache():
    """Teacher-forced scales 1..3 in one sequence under the mask scale(q) >= scale(kv) give the
    same attention rows as scale-by-scale calls that see the growing cache."""
    sides = (1, 2, 3)
    H, Dh = 2, 8
    L = sum(s * s for s in sides)
    q, K, V = _rand_qkv(L, L, H, Dh, 4)
    sc = np.concatenate([np.full(s * s, i) for i, s in enumerate(sides)])
    mask = (sc[:, None] >= sc[None, :]).astype(np.uint8)
    o_mask = oracle.attention(q, K, V, mask=mask)
    start = 0
    for s in sides:
        end = start + s * s
        o_inc = oracle.attention(q[start:end], K[:end], V[:end])
        assert np.array_equal(o_inc, o_mask[start:end])
        start = end


# ----------------------------------------------------------------------------- pruned path
def _small_case(seed=0, M=24, d=32, H=4, Fh=80, Lp=10, r=6, noise=0.0):
    x = wl.activations_lowrank(1, M, d, seed=seed)[0]
    w = oracle.BlockWeights(**wl.block_weights(d, Fh, seed=seed + 1, std=0.2, with_bias=True))
    Kp, Vp = wl.kv_prefix(1, Lp, H, d // H, seed=seed + 2)
    Cm = wl.cached_feature(1, M, d, r, seed=seed + 3, noise=noise)[0]
    z = wl.normal_draws(1, M, r, seed=seed + 4)[0]
    Wc, Gc = factors.cache_factors(Cm, z)
    return x, w, H, Kp[0], Vp[0], Cm, Wc, Gc


def _cache(Kp, Vp, extra):
    Lp, H, Dh = Kp.shape
    Kc = np.zeros((Lp + extra, H, Dh), np.float32); Vc = np.zeros_like(Kc)
    Kc[:Lp], Vc[:Lp] = Kp, Vp
    return Kc, Vc


def test_keep_all_reproduces_dense_exactly():
    x, w, H, Kp, Vp, Cm, Wc, Gc = _small_case()
    M = x.shape[0]; Lp = Kp.shape[0]
    Kd, Vd = _cache(Kp, Vp, M)
    dense = oracle.block_forward(x, w, H, Kd, Vd, Lp)
    Kq, Vq = _cache(Kp, Vp, M)
    out = oracle.pruned_step(x, M, w, H, Kq, Vq, Lp, Wc, Gc)
    assert np.array_equal(out["y"], dense) and np.array_equal(out["y_keep"], dense)
    assert out["idx_keep"].tolist() == list(range(M)) and out["idx_drop"].size == 0
    assert np.array_equal(Kq, Kd) and np.array_equal(Vq, Vd)


def test_pruned_step_composition():
    x, w, H, Kp, Vp, Cm, Wc, Gc = _small_case(seed=5, noise=0.05)
    M, d = x.shape; Lp = Kp.shape[0]; k = 9
    Kq, Vq = _cache(Kp, Vp, k)
    out = oracle.pruned_step(x, k, w, H, Kq, Vq, Lp, Wc, Gc)
    keep, drop = out["idx_keep"], out["idx_drop"]
    # partition of [0,M), both ascending
    assert sorted(keep.tolist() + drop.tolist()) == list(range(M))
    assert np.all(np.diff(keep) > 0) and np.all(np.diff(drop) > 0)
    bk, bd = _brute_topk(oracle.scores(x), k)
    assert np.array_equal(keep, bk) and np.array_equal(drop, bd)
    # kept rows: the block on exactly those rows, independently through the fp64 framework
    ref, kk, v = _torch_block(x[keep], w, H, Kp, Vp)
    assert np.abs(out["y_keep"] - ref).max() < 1e-5
    assert np.array_equal(out["y"][keep], out["y_keep"])
    # appended cache rows follow idx_keep order
    assert np.abs(Kq[Lp:].reshape(k, d) - kk).max() < 1e-5
    # pruned rows: the rank-r restoration of the cached feature
    fill = Wc.astype(np.float64) @ Gc.astype(np.float64)
    assert np.abs(out["y"][drop] - fill[drop]).max() < 1e-5


def test_single_kept_row_equals_one_query_dense_block():
    x, w, H, Kp, Vp, Cm, Wc, Gc = _small_case(seed=9)
    Lp = Kp.shape[0]
    Kq, Vq = _cache(Kp, Vp, 1)
    out = oracle.pruned_step(x, 1, w, H, Kq, Vq, Lp, Wc, Gc)
    i = int(out["idx_keep"][0])
    assert i == int(np.argmax(oracle.scores(x)))
    Kd, Vd = _cache(Kp, Vp, 1)
    one = oracle.block_forward(x[i:i + 1], w, H, Kd, Vd, Lp)
    assert np.array_equal(out["y_keep"], one)


# ----------------------------------------------------------------------------- factors & fill
def test_fill_lossless_on_exact_rank_r_cache():
    M, d, r = 40, 48, 8
    Cm = wl.cached_feature(1, M, d, r, seed=11)[0]
    z = wl.normal_draws(1, M, r, seed=12)[0]
    Wc, Gc = factors.cache_factors(Cm, z)
    keep = np.array([3, 17], np.int32)
    drop = np.array([i for i in range(M) if i not in (3, 17)], np.int32)
    yk = np.ones((2, d), np.float32)
    Y = oracle.lowrank_fill(yk, keep, drop, M, Wc, Gc)
    rel = np.linalg.norm(Y[drop] - Cm[drop]) / np.linalg.norm(Cm[drop])
    assert rel < 1e-5
    assert np.array_equal(Y[keep], yk)


def test_full_rank_fill_equals_raw_cached_rows():
    # r = rank(C) = min(M,d): the restoration returns the cached rows themselves, i.e. the
    # representative-token restoration of Eq. "redefine" with the raw cache.
    M, d = 12, 20
    Cm = wl.cached_feature(1, M, d, M, seed=13, noise=0.3)[0]
    z = wl.normal_draws(1, M, M, seed=14)[0]
    Wc, Gc = factors.cache_factors(Cm, z)
    drop = np.arange(M, dtype=np.int32)
    Y = oracle.lowrank_fill(np.zeros((0, d), np.float32), np.zeros(0, np.int32), drop, M, Wc, Gc)
    assert np.linalg.norm(Y - Cm) / np.linalg.norm(Cm) < 1e-4


def test_factors_normal_equations_and_eckart_young():
    M, d, r = 60, 40, 6
    Cm = wl.cached_feature(1, M, d, 20, seed=15, noise=0.2)[0].astype(np.float64)
    z = wl.normal_draws(1, M, r, seed=16)[0]
    Q = factors.random_projection_matrix(z, r)
    G = factors.project(Q, Cm)
    W = factors.restoration_matrix(G, Cm)
    resid = Cm - W @ G
    assert np.abs(resid @ G.T).max() < 1e-8 * np.abs(Cm).max() * np.abs(G).max() * d
    sv = np.linalg.svd(Cm, compute_uv=False)
    assert np.linalg.norm(resid) >= np.sqrt((sv[r:] ** 2).sum()) * (1 - 1e-12)
    # any other W does worse
    rng = np.random.default_rng(0)
    assert np.linalg.norm(Cm - (W + 1e-3 * rng.standard_normal(W.shape)) @ G) > np.linalg.norm(resid)
    # energy ratio: monotone thresholds, alpha -> 1 needs the full rank
    ranks = [factors.energy_rank(Cm, a) for a in (0.5, 0.9, 0.96, 0.99, 1.0)]
    assert ranks == sorted(ranks) and ranks[-1] == min(M, d)
    exact = wl.cached_feature(1, M, d, 5, seed=17)[0]
    assert factors.energy_rank(exact, 0.999999) == 5


def test_random_projection_preserves_norm_in_expectation():
    M, r, trials = 50, 16, 400
    xv = np.random.default_rng(1).standard_normal(M)
    vals = []
    for t in range(trials):
        Q = factors.random_projection_matrix(wl.normal_draws(1, M, r, seed=100 + t)[0], r)
        vals.append(np.sum((Q.T @ xv) ** 2))
    vals = np.array(vals) / np.sum(xv ** 2)
    # E = 1, Var = 2/r for a chi-square with r degrees of freedom scaled by 1/r
    assert abs(vals.mean() - 1.0) < 3 * np.sqrt(2.0 / r / trials)
    Q = factors.random_projection_matrix(wl.normal_draws(1, 4000, r, seed=5)[0], r)
    assert abs(Q.var() * r - 1.0) < 0.02


# ----------------------------------------------------------------------------- RP input path
def test_round_bf16_matches_library_cast():
    rng = np.random.default_rng(3)
    a = (rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.00390625, 1.01171875]      # the last two sit exactly between neighbours
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(factors.round_bf16(a), ref)
    assert factors.round_bf16(a[2:4]).tolist() == [1.0, 1.015625]      # ties go to the even mantissa


def test_rp_input_is_qt_times_x():
    from oracle import rp_path
    M, d, r = 23, 16, 5
    rng = np.random.default_rng(4)
    X = rng.standard_normal((M, d)); Y = rng.standard_normal((M, d))
    Q = factors.random_projection_matrix(wl.normal_draws(1, M, r, seed=21)[0], r)
    F = rp_path.rp_input(Q, X)
    assert F.shape == (r, d) and F.dtype == np.float32
    # written out element by element: F[t,j] = sum_i Q[i,t] X[i,j]  (catches a transposed operand)
    brute = np.array([[sum(Q[i, t] * X[i, j] for i in range(M)) for j in range(d)] for t in range(r)])
    assert np.abs(F - brute).max() < 1e-6
    # linear in X
    lin = rp_path.rp_input(Q, 2.0 * X - 3.0 * Y)
    assert np.abs(lin - (2.0 * F - 3.0 * rp_path.rp_input(Q, Y))).max() < 1e-5
    # a column-selection Q turns the projection into the row gather of the token-selection path
    idx = np.array([2, 7, 11, 19, 22])
    S = np.zeros((M, r)); S[idx, np.arange(r)] = 1.0
    assert np.array_equal(rp_path.rp_input(S, X), X[idx].astype(np.float32))
    # storage rounding
    assert np.array_equal(rp_path.rp_input(Q, X, bf16=True), factors.round_bf16(F64 := factors.project(Q, X)))
    assert np.abs(rp_path.rp_input(Q, X, bf16=True) - F64).max() <= np.abs(F64).max() * 2.0 ** -8


def test_cache_fill_is_eq_redefine():
    from oracle import rp_path
    M, d = 9, 4
    Cm = np.arange(M * d, dtype=np.float32).reshape(M, d)
    keep = np.array([1, 4, 8], np.int32)
    yk = -np.ones((3, d), np.float32) * np.array([[1.0], [2.0], [3.0]], np.float32)
    Y = rp_path.cache_fill(yk, keep, Cm)
    for i in range(M):
        if i in keep.tolist():
            assert np.array_equal(Y[i], yk[keep.tolist().index(i)])
        else:
            assert np.array_equal(Y[i], Cm[i])
    assert np.array_equal(rp_path.cache_fill(np.zeros((0, d), np.float32), np.zeros(0, np.int32), Cm), Cm)
    full = np.arange(M, dtype=np.int32)
    assert np.array_equal(rp_path.cache_fill(2 * Cm, full, Cm), 2 * Cm)
    # the rank-r fill at full rank restores exactly these rows (Eq. "redefine" with the raw cache)
    C2 = wl.cached_feature(1, 12, 20, 12, seed=13, noise=0.3)[0]
    Wc, Gc = factors.cache_factors(C2, wl.normal_draws(1, 12, 12, seed=14)[0])
    keep2 = np.array([0, 5], np.int32); drop2 = np.array([i for i in range(12) if i not in (0, 5)], np.int32)
    yk2 = np.ones((2, 20), np.float32)
    a = oracle.lowrank_fill(yk2, keep2, drop2, 12, Wc, Gc)
    b = rp_path.cache_fill(yk2, keep2, C2)
    assert np.abs(a - b).max() < 1e-4 * np.abs(C2).max()


def test_rp_step_with_selection_matrix_equals_token_selection_path():
    from oracle import rp_path
    x, w, H, Kp, Vp, Cm, Wc, Gc = _small_case(seed=7, noise=0.05)
    M, d = x.shape; Lp = Kp.shape[0]; r = 6
    keep, drop = oracle.topk(oracle.scores(x), r)
    S = np.zeros((M, r)); S[keep, np.arange(r)] = 1.0
    Kq, Vq = _cache(Kp, Vp, r)
    ref = oracle.pruned_step(x, r, w, H, Kq, Vq, Lp, Wc, Gc)
    Kr, Vr = _cache(Kp, Vp, r)
    out = rp_path.rp_step(x, S, Cm, w, H, Kr, Vr, Lp)
    assert np.array_equal(out["idx_keep"], ref["idx_keep"]) and np.array_equal(out["idx_drop"], ref["idx_drop"])
    assert np.array_equal(out["y_keep"], ref["y_keep"])
    assert np.array_equal(Kr, Kq) and np.array_equal(Vr, Vq)
    assert np.array_equal(out["y"][keep], ref["y_keep"]) and np.array_equal(out["y"][drop], Cm[drop])
    # a Gaussian Q: the block sees r mixed rows; the output keeps the cached rows elsewhere
    Q = factors.random_projection_matrix(wl.normal_draws(1, M, r, seed=31)[0], r)
    Kg, Vg = _cache(Kp, Vp, r)
    g = rp_path.rp_step(x, Q, Cm, w, H, Kg, Vg, Lp)
    Kd, Vd = _cache(Kp, Vp, r)
    direct = oracle.block_forward(rp_path.rp_input(Q, x), w, H, Kd, Vd, Lp)
    assert np.array_equal(g["y_keep"], direct) and np.array_equal(g["y"][drop], Cm[drop])
    assert np.array_equal(g["y"][keep], direct)


def test_stored_factors_solve_against_the_stored_g():
    M, d, r = 60, 40, 6
    Cm = wl.cached_feature(1, M, d, 20, seed=15, noise=0.2)[0]
    Q = factors.random_projection_matrix(wl.normal_draws(1, M, r, seed=16)[0], r)
    W0, G0 = factors.cache_factors(Cm, wl.normal_draws(1, M, r, seed=16)[0])
    W1, G1 = factors.stored_factors(Cm, Q)
    assert np.array_equal(G1, G0) and np.abs(W1 - W0).max() < 1e-5 * np.abs(W0).max()
    # bf16 storage: G is a bf16 value, and W satisfies the normal equations of THAT G
    Wb, Gb = factors.stored_factors(Cm, Q, bf16=True)
    assert np.array_equal(Gb, factors.round_bf16(Gb)) and np.array_equal(Wb, factors.round_bf16(Wb))
    assert np.abs(Gb - G0).max() <= 2.0 ** -8 * np.abs(G0).max()
    Wex = factors.restoration_matrix(Gb, Cm)
    G64 = Gb.astype(np.float64)
    scale = np.abs(Cm).max() * np.abs(G64).max() * d
    assert np.abs((Cm - Wex @ G64) @ G64.T).max() < 1e-9 * scale
    assert np.abs(Wb - Wex).max() <= 2.0 ** -8 * np.abs(Wex).max()
    # solving against the unrounded product instead leaves a visible normal-equation residual
    Wwrong = factors.restoration_matrix(factors.project(Q, Cm), Cm)
    assert np.abs((Cm - Wwrong @ G64) @ G64.T).max() > 1e-6 * scale


# ----------------------------------------------------------------------------- cache up-sampling
def test_upsample_matches_library_bilinear_and_is_linear_on_tokens():
    from oracle import upsample
    rng = np.random.default_rng(8)
    for (hs, ws, hd, wd) in [(3, 3, 4, 4), (24, 24, 32, 32), (5, 7, 8, 9), (4, 4, 4, 4), (6, 6, 3, 3), (1, 1, 5, 5)]:
        c = 6
        src = rng.standard_normal((hs * ws, c))
        got = upsample.upsample_tokens(src, hs, ws, hd, wd)
        t = torch.from_numpy(src.reshape(hs, ws, c)).permute(2, 0, 1)[None]
        ref = torch.nn.functional.interpolate(t, size=(hd, wd), mode="bilinear", align_corners=False)
        ref = ref[0].permute(1, 2, 0).reshape(hd * wd, c).numpy()
        assert np.abs(got - ref).max() < 1e-12, (hs, ws, hd, wd)
    # hand case: 2 -> 4 along one axis gives weights (1, 3/4|1/4, 1/4|3/4, 1)
    one = upsample.upsample_tokens(np.array([[0.0], [4.0]]), 2, 1, 4, 1)[:, 0]
    assert one.tolist() == [0.0, 1.0, 3.0, 4.0]
    # same size is the identity; a constant map stays constant
    a = rng.standard_normal((20, 3))
    assert np.array_equal(upsample.upsample_tokens(a, 4, 5, 4, 5), a)
    assert np.allclose(upsample.upsample_tokens(np.full((9, 2), 2.5), 3, 3, 7, 5), 2.5, rtol=0, atol=1e-15)
    # linear on the token axis: Up(W G) = Up(W) G  (the thin-factor form of Eq. "upcache")
    Wm = rng.standard_normal((6 * 6, 4)); G = rng.standard_normal((4, 10))
    lhs = upsample.upsample_tokens(Wm @ G, 6, 6, 8, 8)
    rhs = upsample.upsample_tokens(Wm, 6, 6, 8, 8) @ G
    assert np.abs(lhs - rhs).max() < 1e-12


# ----------------------------------------------------------------------------- block chunks
def test_pruned_chunk_of_one_block_is_the_pruned_step_and_chunks_compose():
    x, w, H, Kp, Vp, Cm, Wc, Gc = _small_case(seed=21, noise=0.05)
    M, d = x.shape; Lp = Kp.shape[0]; k = 7
    Ka, Va = _cache(Kp, Vp, k)
    ref = oracle.pruned_step(x, k, w, H, Ka, Va, Lp, Wc, Gc)
    Kb, Vb = _cache(Kp, Vp, k)
    one = oracle.pruned_chunk(x, k, [w], H, [(Kb, Vb)], Lp, Wc, Gc)
    for key in ("scores", "idx_keep", "idx_drop", "y_keep", "y"):
        assert np.array_equal(one[key], ref[key]), key
    assert np.array_equal(Kb, Ka) and np.array_equal(Vb, Va)
    # two blocks: the second sees the first one's compact output, checked through the independent
    # fp64 statement of the block
    w2 = oracle.BlockWeights(**wl.block_weights(d, w.w_fc1.shape[0], seed=77, std=0.8 / np.sqrt(d)))
    Kp2, Vp2 = wl.kv_prefix(1, Lp, H, d // H, seed=78)
    K1, V1 = _cache(Kp, Vp, k); K2, V2 = _cache(Kp2[0], Vp2[0], k)
    two = oracle.pruned_chunk(x, k, [w, w2], H, [(K1, V1), (K2, V2)], Lp, Wc, Gc)
    assert np.array_equal(two["idx_keep"], ref["idx_keep"])
    mid, _, _ = _torch_block(x[ref["idx_keep"]], w, H, Kp, Vp)
    out, kk2, _ = _torch_block(mid, w2, H, Kp2[0], Vp2[0])
    assert np.abs(two["y_keep"] - out).max() < 2e-5
    assert np.abs(K2[Lp:].reshape(k, d) - kk2).max() < 2e-5
    assert np.array_equal(two["y"][two["idx_keep"]], two["y_keep"])
    fill = Wc.astype(np.float64) @ Gc.astype(np.float64)
    assert np.abs(two["y"][two["idx_drop"]] - fill[two["idx_drop"]]).max() < 1e-5


def test_oracle_c_clean_under_address_and_ub_sanitizers(tmp_path):
    """oracle/fvar_oracle.c compiled with -fsanitize=address,undefined (runtimes linked
    statically, so nothing has to be preloaded) and run by tests/oracle_sanitize_driver.c on
    ragged shapes with exactly-sized buffers: no out-of-bounds access, no undefined arithmetic,
    no leak in any oracle function."""
    import shutil
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    src = [os.path.join(here, "oracle_sanitize_driver.c"),
           os.path.join(here, "..", "oracle", "fvar_oracle.c")]
    exe = str(tmp_path / "oracle_san")
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    cc = subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined",
                         "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan",
                         "-static-libubsan", "-o", exe] + src + ["-lm"], capture_output=True, text=True)
    if cc.returncode != 0 and "asan" in cc.stderr.lower():
        pytest.skip("static sanitizer runtimes not installed")
    assert cc.returncode == 0, cc.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "checksum" in run.stdout and "ERROR" not in run.stderr
