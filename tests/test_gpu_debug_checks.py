"""Debug checks of the library: with fvar_debug_checks on, index arrays that break the contract
(out of range, not ascending, a token in both lists) are rejected from the host before anything
is launched, and the block call guards its workspace with a canary."""
import numpy as np
import pytest
import torch

import paper_2512_16483_amd as fv
import workloads as wl

pytestmark = pytest.mark.gpu


def _setup(B=2, M=40, d=128, k=12, r=8):
    ctx = fv.Context(hidden=d, heads=2, head_dim=64, ffn_hidden=256, dtype="bf16")
    fv.fvar_debug_checks(ctx, True)
    keep = np.stack([np.sort(np.random.default_rng(b).permutation(M)[:k]) for b in range(B)]).astype(np.int32)
    drop = np.stack([np.setdiff1d(np.arange(M), keep[b]) for b in range(B)]).astype(np.int32)
    bf = lambda *s: torch.randn(*s, device="cuda").to(torch.bfloat16)
    return ctx, keep, drop, bf(B, k, d), bf(B, M, r), bf(B, r, d), torch.empty((B, M, d), dtype=torch.bfloat16, device="cuda")


def test_fill_rejects_broken_index_arrays():
    B, M, k, r = 2, 40, 12, 8
    ctx, keep, drop, yk, Wc, Gc, y = _setup(B, M, 128, k, r)
    cu = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    fv.fvar_lowrank_fill(ctx, yk, cu(keep), cu(drop), B, M, k, r, Wc, Gc, y)       # the contract holds
    torch.cuda.synchronize()
    bad = []
    a = keep.copy(); a[1, 3] = M; bad.append((a, drop, b"outside"))                # out of range
    a = keep.copy(); a[0, 5] = -1; bad.append((a, drop, b"outside"))
    a = keep.copy(); a[0, [2, 3]] = a[0, [3, 2]]; bad.append((a, drop, b"ascending"))   # order
    a = keep.copy(); a[1, 4] = a[1, 3]; bad.append((a, drop, b"ascending"))        # duplicate
    a = drop.copy(); a[0, 0], a[0, 1] = a[0, 1], a[0, 0]; bad.append((keep, a, b"ascending"))
    # a token in both lists (and another one in neither): every list still ascending and in range
    a = drop.copy()
    j = int(np.searchsorted(a[1], keep[1, 6]))
    j = min(max(j, 0), a.shape[1] - 1)
    a[1, j] = keep[1, 6]
    if (np.diff(a[1]) > 0).all():
        bad.append((keep, a, b"idx_keep and idx_drop"))
    for kk, dd, word in bad:
        with pytest.raises(fv.FvarError) as e:
            fv.fvar_lowrank_fill(ctx, yk, cu(kk), cu(dd), B, M, k, r, Wc, Gc, y)
        assert e.value.status == fv.FVAR_ERR_INVALID_ARG and word in str(e.value).encode()
    fv.fvar_debug_checks(ctx, False)                                                # off: not looked at
    fv.fvar_lowrank_fill(ctx, yk, cu(keep), cu(drop), B, M, k, r, Wc, Gc, y)
    torch.cuda.synchronize()


def test_block_call_checks_indices_and_guards_its_workspace():
    B, M, d, H, F, Lp, k = 1, 96, 128, 2, 256, 10, 32
    ctx = fv.Context(hidden=d, heads=H, head_dim=64, ffn_hidden=F, dtype="bf16")
    w = {n: torch.from_numpy(v).cuda().to(torch.bfloat16).contiguous()
         for n, v in wl.block_weights(d, F, seed=5, bf16=True, std=0.05).items()}
    x = torch.randn((B, M, d), device="cuda").to(torch.bfloat16)
    K = torch.zeros((B, Lp + M, H, 64), dtype=torch.bfloat16, device="cuda")
    V = torch.zeros_like(K)
    keep = torch.arange(0, 2 * k, 2, dtype=torch.int32, device="cuda").reshape(B, k).contiguous()
    yk = torch.empty((B, k, d), dtype=torch.bfloat16, device="cuda")
    plain = fv.fvar_block_workspace_bytes(ctx, B, k)
    fv.fvar_debug_checks(ctx, True)
    guarded = fv.fvar_block_workspace_bytes(ctx, B, k)
    assert guarded == plain + 256
    ws = torch.empty(guarded, dtype=torch.uint8, device="cuda")
    fv.fvar_block_forward_pruned(ctx, w, x, B, M, keep, k, K, V, Lp + M, Lp, yk, ws)   # canary intact
    assert bool((ws[plain:] == 0xA5).all())
    with pytest.raises(fv.FvarError) as e:                                              # too small now
        fv.fvar_block_forward_pruned(ctx, w, x, B, M, keep, k, K, V, Lp + M, Lp, yk, ws[:plain])
    assert e.value.status == fv.FVAR_ERR_WORKSPACE
    bad = keep.clone(); bad[0, 7] = M + 3
    with pytest.raises(fv.FvarError) as e:
        fv.fvar_block_forward_pruned(ctx, w, x, B, M, bad, k, K, V, Lp + M, Lp, yk, ws)
    assert e.value.status == fv.FVAR_ERR_INVALID_ARG
