#!/usr/bin/env python3
"""Benchmark of the late-scale pruned block path on one MI355X.

A step = every late scale of the workload through all of its blocks; every block runs score ->
select -> pruned block (gather, LN, QKV, attention over the multi-scale cache, O, LN, MLP) ->
low-rank fill + scatter, and its output token map is the next block's input.  The default
workload is the largest single-GPU shape: hidden 4096, 32 heads of 128, 40 blocks, the 80x80
scale (6400 tokens, 1600 kept, 12121 keys), rank 128, batch 4; `--workload` selects the other
shapes and `--sweep` runs the keep-ratio x rank x scale table of the batch-32 Infinity-2B shape.
Inputs are synthetic and resident in HBM.  Prints one JSON line."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
WORKLOAD = "large_1280_bf16"
# HBM-side bytes per GEMM launch of a workload (FETCH_SIZE + WRITE_SIZE of two rocprofv3 --pmc runs,
# each scaled by what the same counter reads for a device copy of known size; the summary file
# under profiles/ is named in the entry).  An entry is dropped (traffic: null) whenever gemm.hip
# changes, until the counters are taken again.
GEMM_TRAFFIC = {
    "large_1280_bf16": {"bytes_per_launch": 1.333e9,
                        "source": "profiles/pruned_chain_large_1280_bf16_hbm_counters.txt"},
    "infinity2b_1024_b32_bf16": {"bytes_per_launch": 1.769e9,
                                 "source": "profiles/pruned_chain_infinity2b_1024_b32_bf16_hbm_counters.txt"},
}
SWEEP_WORKLOAD = "infinity2b_1024_b32_bf16"


class Chain:
    """Device state of one workload and the launch sequence of one step."""

    def __init__(self, W, fv, torch):
        import workloads as wl
        self.W, self.fv, self.torch = W, fv, torch
        self.ctx = fv.Context(hidden=W.hidden, heads=W.heads, head_dim=W.head_dim,
                              ffn_hidden=W.ffn_hidden, scales=W.scales, dtype=W.dtype)
        self.blocks = wl.device_block_state(W)
        self.cap = W.total_len()
        self.set_reduction(W)

    def set_reduction(self, W):
        """(Re)build the per-scale state for W's keep ratio and rank; weights and caches stay."""
        import workloads as wl
        fv, torch = self.fv, self.torch
        self.W = W
        self.scale = {}
        dt = torch.bfloat16 if W.dtype == "bf16" else torch.float32
        B, d = W.batch, W.hidden
        for side in W.late_scales:
            M, k = W.tokens(side), W.keep(side)
            x0, Wc, Gc = wl.device_workload(W, side)
            self.scale[side] = dict(
                M=M, k=k, Lp=W.prev_len(side), x0=x0, Wc=Wc, Gc=Gc,
                bufs=[torch.empty((B, M, d), dtype=dt, device="cuda") for _ in range(2)],
                y_keep=torch.empty((B, k, d), dtype=dt, device="cuda"),
                keep=torch.empty((B, k), dtype=torch.int32, device="cuda"),
                drop=torch.empty((B, M - k), dtype=torch.int32, device="cuda"))
        maxM = max(s["M"] for s in self.scale.values())
        self.sel_ws = torch.empty(fv.fvar_select_workspace_bytes(self.ctx, B, maxM),
                                  dtype=torch.uint8, device="cuda")
        self.ws = torch.empty(fv.fvar_block_workspace_bytes(self.ctx, B, maxM), dtype=torch.uint8,
                              device="cuda")

    def pruned_scale(self, side):
        fv, W, s = self.fv, self.W, self.scale[side]
        B, M, k, r = W.batch, s["M"], s["k"], W.rank
        x = s["x0"]
        for i, (w, K, V) in enumerate(self.blocks):
            y = s["bufs"][i & 1]
            fv.fvar_score_select(self.ctx, x, B, M, k, s["keep"], s["drop"], ws=self.sel_ws)
            fv.fvar_block_forward_pruned(self.ctx, w, x, B, M, s["keep"], k, K, V, self.cap, s["Lp"],
                                         s["y_keep"], self.ws)
            fv.fvar_lowrank_fill(self.ctx, s["y_keep"], s["keep"], s["drop"], B, M, k, r,
                                 s["Wc"][i], s["Gc"][i], y)
            x = y
        return x

    def dense_scale(self, side):
        fv, W, s = self.fv, self.W, self.scale[side]
        B, M = W.batch, s["M"]
        x = s["x0"]
        for i, (w, K, V) in enumerate(self.blocks):
            y = s["bufs"][i & 1]
            fv.fvar_block_forward_dense(self.ctx, w, x, B, M, K, V, self.cap, s["Lp"], y, self.ws)
            x = y
        return x

    def scored_scale(self, side):
        """The same chain with the scores of block i+1 produced by the kernels that write block
        i's output map (fvar_lowrank_fill_scored): only the first block of the scale reads its
        input to score it."""
        fv, W, s = self.fv, self.W, self.scale[side]
        B, M, k, r = W.batch, s["M"], s["k"], W.rank
        if "scores" not in s:
            s["scores"] = self.torch.empty((B, M), dtype=self.torch.float32, device="cuda")
            s["fill_ws"] = self.torch.empty(fv.fvar_fill_scored_workspace_bytes(self.ctx, B, M),
                                            dtype=self.torch.uint8, device="cuda")
        x = s["x0"]
        for i, (w, K, V) in enumerate(self.blocks):
            y = s["bufs"][i & 1]
            fv.fvar_score_select(self.ctx, x, B, M, k, s["keep"], s["drop"], ws=self.sel_ws,
                                 scores_in=s["scores"] if i else None)
            fv.fvar_block_forward_pruned(self.ctx, w, x, B, M, s["keep"], k, K, V, self.cap, s["Lp"],
                                         s["y_keep"], self.ws)
            fv.fvar_lowrank_fill_scored(self.ctx, s["y_keep"], s["keep"], s["drop"], B, M, k, r,
                                        s["Wc"][i], s["Gc"][i], y, s["scores"], s["fill_ws"])
            x = y
        return x

    def rp_state(self, side):
        """Extra device state of the random-projection input variant and of the factor
        construction: Q^T [k,M] and [r,M] with N(0,1/rows) entries, and a cached counterpart
        feature C (same recipe as the block input, other seed)."""
        import workloads as wl
        s, W, torch = self.scale[side], self.W, self.torch
        if "Qt" not in s:
            g = torch.Generator(device="cuda").manual_seed(4100 + side)
            dt = s["x0"].dtype
            for name, rows in (("Qt", s["k"]), ("Qt_r", W.rank)):
                s[name] = (torch.randn((rows, s["M"]), generator=g, device="cuda") /
                           rows ** 0.5).to(dt)
            s["C"] = wl.device_workload(W, side, seed=5000)[0]
            s["f_r"] = torch.empty_like(s["y_keep"])
            s["Wf"], s["Gf"] = torch.empty_like(s["Wc"][0]), torch.empty_like(s["Gc"][0])
        return s

    def rp_scale(self, side):
        """The fidelity stage as the paper's algorithm prints it: the block runs on the k rows
        Q^T x, its outputs go to the selected positions and the raw cached rows to the others."""
        fv, W, s = self.fv, self.W, self.rp_state(side)
        B, M, k = W.batch, s["M"], s["k"]
        x = s["x0"]
        for i, (w, K, V) in enumerate(self.blocks):
            y = s["bufs"][i & 1]
            fv.fvar_score_select(self.ctx, x, B, M, k, s["keep"], s["drop"], ws=self.sel_ws)
            fv.fvar_rp_project(self.ctx, s["Qt"], False, x, B, M, k, s["f_r"])
            fv.fvar_block_forward_dense(self.ctx, w, s["f_r"], B, k, K, V, self.cap, s["Lp"],
                                        s["y_keep"], self.ws)
            fv.fvar_cache_fill(self.ctx, s["y_keep"], s["keep"], s["drop"], B, M, k, s["C"], y)
            x = y
        return x

    def chunked_scale(self, side, chunk=4):
        """One selection per chunk of `chunk` blocks (the granularity the paper applies its
        reduction at): score/select/gather at the chunk's first block, the other blocks run on
        the compact rows, one fill at the chunk's end."""
        fv, W, s = self.fv, self.W, self.scale[side]
        B, M, k, r = W.batch, s["M"], s["k"], W.rank
        if "rows2" not in s:
            s["rows2"] = self.torch.empty_like(s["y_keep"])
        x = s["x0"]
        nb = len(self.blocks)
        for c0 in range(0, nb, chunk):
            y = s["bufs"][(c0 // chunk) & 1]
            fv.fvar_score_select(self.ctx, x, B, M, k, s["keep"], s["drop"], ws=self.sel_ws)
            rows, other = s["y_keep"], s["rows2"]
            for i in range(c0, min(c0 + chunk, nb)):
                w, K, V = self.blocks[i]
                if i == c0:
                    fv.fvar_block_forward_pruned(self.ctx, w, x, B, M, s["keep"], k, K, V, self.cap,
                                                 s["Lp"], rows, self.ws)
                else:
                    fv.fvar_block_forward_dense(self.ctx, w, rows, B, k, K, V, self.cap, s["Lp"],
                                                other, self.ws)
                    rows, other = other, rows
            fv.fvar_lowrank_fill(self.ctx, rows, s["keep"], s["drop"], B, M, k, r, s["Wc"][c0],
                                 s["Gc"][c0], y)
            x = y
        return x

    def factors(self, side):
        """W_c, G_c of the cached counterpart feature of one block at one scale."""
        fv, W, s = self.fv, self.W, self.rp_state(side)
        B, M, r = W.batch, s["M"], W.rank
        if "fws" not in s:
            s["fws"] = self.torch.empty(fv.fvar_factors_workspace_bytes(self.ctx, B, M, r),
                                        dtype=self.torch.uint8, device="cuda")
        fv.fvar_cache_factors(self.ctx, s["C"], s["Qt_r"], False, B, M, r, 0.0, s["Wf"], s["Gf"],
                              s["fws"])

    def factors_all_blocks(self, side):
        """The same construction for the cached features of all blocks of the scale in one call
        (they are all known once the previous scale is finished): batch = blocks x B."""
        fv, W, s = self.fv, self.W, self.rp_state(side)
        n, M, r, torch = W.batch * W.blocks, s["M"], W.rank, self.torch
        if "C_all" not in s:
            s["C_all"] = s["C"].repeat(W.blocks, 1, 1).contiguous()
            s["W_all"] = torch.empty((n, M, r), dtype=s["C"].dtype, device="cuda")
            s["G_all"] = torch.empty((n, r, W.hidden), dtype=s["C"].dtype, device="cuda")
            s["fws_all"] = torch.empty(fv.fvar_factors_workspace_bytes(self.ctx, n, M, r),
                                       dtype=torch.uint8, device="cuda")
        fv.fvar_cache_factors(self.ctx, s["C_all"], s["Qt_r"], False, n, M, r, 0.0, s["W_all"],
                              s["G_all"], s["fws_all"])

    def factored_handover(self, side):
        """What hands the cached counterpart features to scale `side` in factored form: the
        outputs of all blocks at the previous scale are factored in one call (batch = blocks x B)
        and the thin factors are up-sampled to this scale's grid.  Returns the previous side."""
        import workloads as wl
        fv, W, torch = self.fv, self.W, self.torch
        prev = W.scales[W.scales.index(side) - 1]
        s = self.scale[side]
        n, Mp, M, r, d = W.batch * W.blocks, prev * prev, side * side, W.rank, W.hidden
        if "ho" not in s:
            dt = s["x0"].dtype
            g = torch.Generator(device="cuda").manual_seed(4200 + side)
            Wd = __import__("dataclasses").replace(W, batch=n, blocks=0)
            ho = {"C": wl.device_workload(Wd, prev, seed=5100)[0],
                  "Qt": (torch.randn((r, Mp), generator=g, device="cuda") / r ** 0.5).to(dt),
                  "Ws": torch.empty((n, Mp, r), dtype=dt, device="cuda"),
                  "G": torch.empty((n, r, d), dtype=dt, device="cuda"),
                  "Wup": torch.empty((n, M, r), dtype=dt, device="cuda"),
                  "ws": torch.empty(fv.fvar_factors_workspace_bytes(self.ctx, n, Mp, r), dtype=torch.uint8,
                                    device="cuda")}
            s["ho"] = ho
        ho = s["ho"]
        fv.fvar_cache_factors(self.ctx, ho["C"], ho["Qt"], False, n, Mp, r, 0.0, ho["Ws"], ho["G"], ho["ws"])
        fv.fvar_upsample_tokens(self.ctx, ho["Ws"], n, prev, prev, r, side, side, ho["Wup"])
        return prev

    def step(self, dense=False, events=None):
        for side in self.W.late_scales:
            if events is not None:
                e0 = self.torch.cuda.Event(enable_timing=True)
                e1 = self.torch.cuda.Event(enable_timing=True)
                e0.record()
            (self.dense_scale if dense else self.pruned_scale)(side)
            if events is not None:
                e1.record()
                events.setdefault(side, []).append((e0, e1))


def gemm_flops(W, side, dense=False):
    """Algorithmic flops of the four linear layers of one block launch set: 24 * rows * d^2."""
    rows = W.batch * (W.tokens(side) if dense else W.keep(side))
    d, F = W.hidden, W.ffn_hidden
    return {"gemm_qkv": 2.0 * rows * 3 * d * d, "gemm_o": 2.0 * rows * d * d,
            "gemm_fc1": 2.0 * rows * F * d, "gemm_fc2": 2.0 * rows * d * F}


def kernel_work(W, side):
    """Algorithmic work of one launch of every kernel label at scale `side` (pruned path):
    (kind, amount) with kind 'flop' or 'byte'."""
    es = 2 if W.dtype == "bf16" else 4
    B, M, k, d, r = W.batch, W.tokens(side), W.keep(side), W.hidden, W.rank
    L = W.prev_len(side) + k
    out = {lab: ("flop", v) for lab, v in gemm_flops(W, side).items()}
    out["attention"] = ("flop", 4.0 * B * k * L * d)
    out["score"] = ("byte", B * M * (d * es + 4.0))
    out["select"] = ("byte", B * M * 8.0)
    out["gather_ln1"] = ("byte", B * k * (3.0 * d * es + 4))
    out["ln2"] = ("byte", B * k * d * (4.0 + es))       # reads the fp32 residual stream
    out["fill"] = ("byte", B * (M * d * es + k * d * es + (M - k) * r * es + r * d * es))
    # random-projection input variant and factor construction
    out["rp_project"] = ("flop", 2.0 * B * k * M * d)
    out["cache_fill"] = ("byte", 2.0 * B * M * d * es)
    out["factor_project"] = ("flop", 2.0 * B * r * M * d)
    out["factor_t"] = ("byte", B * (M * d * es + r * d * es + M * r * 4.0))
    out["factor_gram"] = ("flop", 2.0 * B * r * r * d)
    out["factor_inverse"] = ("flop", B * (r ** 3) * (1.0 / 3 + 1.0 / 3 + 2.0 / 3))
    out["factor_w"] = ("flop", 2.0 * B * M * r * r)
    return out


def handover(chain, W, fv, torch):
    """Per late scale: time of the factored hand-over of the cached features from the previous
    scale (factor build of all blocks in one call + up-sampling of the thin factors), per block."""
    es = 2 if W.dtype == "bf16" else 4
    rep = {}
    for side in W.late_scales:
        if W.scales.index(side) == 0:
            continue
        prev = chain.factored_handover(side)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            chain.factored_handover(side)
        torch.cuda.synchronize()
        wall_us = (time.perf_counter() - t0) * 1e6 / 3
        fv.fvar_profile_enable(chain.ctx, True)
        chain.factored_handover(side)
        torch.cuda.synchronize()
        prof = fv.fvar_profile_read(chain.ctx)
        fv.fvar_profile_enable(chain.ctx, False)
        n = W.batch * W.blocks
        up_us = prof["upsample"][1] * 1e3
        up_bytes = n * (prev * prev + side * side) * W.rank * es
        rep[str(side)] = {"from_scale": prev, "us_per_block": round(wall_us / W.blocks, 1),
                          "factor_kernels_us_per_block": {l: round(v[1] * 1e3 / W.blocks, 2)
                                                          for l, v in prof.items() if l != "upsample"},
                          "upsample": {"us_all_blocks": round(up_us, 2), "GB/s": round(up_bytes / up_us / 1e3, 1),
                                       "bytes": up_bytes}}
        chain.scale[side].pop("ho")
    return rep


def rates(prof, work):
    """{label: avg_us and achieved rate} from a profile read and the per-launch work table."""
    rep = {}
    for lab, (launches, total_ms) in prof.items():
        kind, amount = work[lab]
        rate = amount * launches / (total_ms * 1e-3)
        rep[lab] = {"avg_us": round(total_ms * 1e3 / launches, 2)}
        rep[lab]["TFLOP/s" if kind == "flop" else "GB/s"] = round(rate / (1e12 if kind == "flop" else 1e9), 2)
    return rep


def variants(chain, W, fv, torch, steps):
    """The random-projection input variant of the same chain, and the construction of the cache
    factors, measured the same way (not part of `value`)."""
    tokens = W.batch * sum(W.tokens(s) for s in W.late_scales)
    for side in W.late_scales:
        chain.rp_scale(side)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for side in W.late_scales:
            chain.rp_scale(side)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for side in W.late_scales:
        chain.chunked_scale(side)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for side in W.late_scales:
            chain.chunked_scale(side)
    torch.cuda.synchronize()
    ms_chunk = (time.perf_counter() - t0) * 1e3 / steps
    for side in W.late_scales:
        chain.scored_scale(side)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for side in W.late_scales:
            chain.scored_scale(side)
    torch.cuda.synchronize()
    ms_scored = (time.perf_counter() - t0) * 1e3 / steps
    fv.fvar_profile_enable(chain.ctx, True)
    for side in W.late_scales:
        chain.scored_scale(side)
    torch.cuda.synchronize()
    scored_k = {l: round(v[1] * 1e3 / v[0], 2) for l, v in fv.fvar_profile_read(chain.ctx).items()
                if l in ("score", "select", "fill")}
    fv.fvar_profile_enable(chain.ctx, False)
    fv.fvar_profile_enable(chain.ctx, True)
    rp_k, fac = {}, {}
    for side in W.late_scales:
        chain.rp_scale(side)
        torch.cuda.synchronize()
        prof = fv.fvar_profile_read(chain.ctx)
        rp_k[str(side)] = rates({l: v for l, v in prof.items() if l in ("rp_project", "cache_fill")},
                                kernel_work(W, side))
        for _ in range(5):
            chain.factors(side)
        torch.cuda.synchronize()
        prof = fv.fvar_profile_read(chain.ctx)
        fac[str(side)] = {"kernels": rates(prof, kernel_work(W, side)),
                          "us_per_call_kernels": round(sum(v[1] for v in prof.values()) * 1e3 / 5, 1)}
    fv.fvar_profile_enable(chain.ctx, False)
    for side in W.late_scales:                       # wall time of the factor call, launch gaps included
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            chain.factors(side)
        torch.cuda.synchronize()
        fac[str(side)]["us_per_call"] = round((time.perf_counter() - t0) * 1e6 / 20, 1)
        chain.factors_all_blocks(side)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            chain.factors_all_blocks(side)
        torch.cuda.synchronize()
        fac[str(side)]["us_per_block_when_all_blocks_batched"] = round(
            (time.perf_counter() - t0) * 1e6 / 5 / W.blocks, 1)
        fv.fvar_profile_enable(chain.ctx, True)
        chain.factors_all_blocks(side)
        torch.cuda.synchronize()
        fac[str(side)]["batched_kernels_us_per_block"] = {
            l: round(v[1] * 1e3 / W.blocks, 2) for l, v in fv.fvar_profile_read(chain.ctx).items()}
        fv.fvar_profile_enable(chain.ctx, False)
        for k in ("C_all", "W_all", "G_all", "fws_all"):
            chain.scale[side].pop(k)
    return {"selection_per_chunk_of_4_blocks": {"ms_per_step": ms_chunk,
                                                "tokens_per_s": tokens / (ms_chunk * 1e-3)},
            "scores_from_the_fill": {"ms_per_step": ms_scored, "tokens_per_s": tokens / (ms_scored * 1e-3),
                                     "avg_us": scored_k},
            "rp_input_path": {"ms_per_step": ms, "tokens_per_s": tokens / (ms * 1e-3), "kernels": rp_k},
            "cache_factors": fac,
            "factored_cache_handover": handover(chain, W, fv, torch)}


def cpu_baseline(W, scales=None, samples=1, budget_gflop=300.0):
    """The CPU oracle on a bounded sample: one block, `samples` batch elements, the late scales
    (or the given subset of them).  When one sample's pruned step exceeds `budget_gflop` (about
    20 s on the host cores) the oracle runs with a quarter (or a sixteenth ...) of the kept rows
    and the time is scaled back up: all but a few per cent of the oracle's work is per kept row."""
    import numpy as np
    import oracle
    import workloads as wl
    d, H, F, r = W.hidden, W.heads, W.ffn_hidden, W.rank
    w = oracle.BlockWeights(**wl.block_weights(d, F, seed=2000, bf16=True))
    tokens, secs, notes = 0, 0.0, []
    scales = tuple(scales or W.late_scales)
    samples = max(1, min(samples, W.batch))
    for side in scales:
        M, k, Lp = W.tokens(side), W.keep(side), W.prev_len(side)
        div = 1
        while (24.0 * d * d + 4.0 * (Lp + k) * d) * (k / div) > budget_gflop * 1e9 and k // (div * 4) >= 1:
            div *= 4
        ks = max(1, k // div)
        if div > 1:
            notes.append(f"scale {side}: oracle run with {ks} of the {k} kept rows, time x {k / ks:.3g}")
        x = wl.activations_lowrank(samples, M, d, seed=1000 + side, bf16=True)
        Kp, Vp = wl.kv_prefix(samples, Lp, H, d // H, seed=3000, bf16=True)
        Wc, Gc = wl.direct_factors(samples, M, r, d, seed=4000, bf16=True)
        for b in range(samples):
            Kc = np.zeros((Lp + ks, H, d // H), np.float32)
            Vc = np.zeros_like(Kc)
            Kc[:Lp], Vc[:Lp] = Kp[b], Vp[b]
            t0 = time.perf_counter()
            oracle.pruned_step(x[b], ks, w, H, Kc, Vc, Lp, Wc[b], Gc[b])
            secs += (time.perf_counter() - t0) * (k / ks)
            tokens += M
    return {"value": tokens / (secs * W.blocks), "unit": "tokens/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"1 of {W.blocks} blocks x {samples} of {W.batch} samples, scales "
                      f"{'+'.join(str(s) for s in scales)} ({secs:.2f} s"
                      f"{' after scaling' if notes else ' measured'}); value = sample tokens / "
                      f"(sample time x {W.blocks} blocks), i.e. extrapolated to the full depth"
                      + ("; " + "; ".join(notes) if notes else "")}


def measure(chain, W, fv, torch, steps, warmup, with_dense=True, dense_steps=None):
    """Times `steps` steps of the pruned chain (and the dense control), then reads the per-kernel
    durations of one more pass.  Returns the pieces of the JSON line."""
    for _ in range(warmup):
        chain.step()
    torch.cuda.synchronize()
    events = {}
    t0 = time.perf_counter()
    for _ in range(steps):
        chain.step(events=events)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    tokens = W.batch * sum(W.tokens(s) for s in W.late_scales)
    ms_scale = {str(s): sum(a.elapsed_time(b) for a, b in ev) / len(ev) for s, ev in events.items()}

    # dense control, same chain without the reduction
    dense = None
    if with_dense:
        chain.step(dense=True)
        torch.cuda.synchronize()
        dev = {}
        n = dense_steps or max(2, steps // 3)
        t0 = time.perf_counter()
        for _ in range(n):
            chain.step(dense=True, events=dev)
        torch.cuda.synchronize()
        d_ms = (time.perf_counter() - t0) * 1e3 / n
        dense = {"ms_per_step": d_ms, "tokens_per_s": tokens / (d_ms * 1e-3),
                 "ms_per_scale": {str(s): sum(a.elapsed_time(b) for a, b in ev) / len(ev)
                                  for s, ev in dev.items()}}

    # per-kernel durations: HIP event pairs recorded by the library on the launch stream
    prof_steps = 2
    per_scale = {}
    fv.fvar_profile_enable(chain.ctx, True)
    for side in W.late_scales:
        for _ in range(prof_steps):
            chain.pruned_scale(side)
        torch.cuda.synchronize()
        per_scale[side] = fv.fvar_profile_read(chain.ctx)
    fv.fvar_profile_enable(chain.ctx, False)

    kernels = {}
    for side, prof in per_scale.items():
        work = kernel_work(W, side)
        for lab, (launches, total_ms) in prof.items():
            kind, amount = work[lab]
            e = kernels.setdefault(lab, {"launches": 0, "total_ms": 0.0, "work": 0.0, "kind": kind})
            e["launches"] += launches
            e["total_ms"] += total_ms
            e["work"] += amount * launches
    report = {}
    for lab, e in kernels.items():
        avg_us = e["total_ms"] * 1e3 / e["launches"]
        rate = e["work"] / (e["total_ms"] * 1e-3)
        if e["kind"] == "flop":
            report[lab] = {"avg_us": round(avg_us, 2), "TFLOP/s": round(rate / 1e12, 1),
                           "frac_of_mfma_peak": round(rate / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
        else:
            report[lab] = {"avg_us": round(avg_us, 2), "GB/s": round(rate / 1e9, 1),
                           "frac_of_hbm_peak": round(rate / 1e9 / HBM_PEAK_GBS, 4)}
    # the four linear layers are one kernel (same code, four shapes): the dominant one
    gl = [l for l in kernels if l.startswith("gemm_")]
    g_ms = sum(kernels[l]["total_ms"] for l in gl)
    g_flop = sum(kernels[l]["work"] for l in gl)
    g_launch = sum(kernels[l]["launches"] for l in gl)
    total_ms = sum(e["total_ms"] for e in kernels.values())
    achieved = g_flop / (g_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_bf16_kernel (qkv, o, fc1, fc2 launches)",
                "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "avg_launch_us": round(g_ms * 1e3 / g_launch, 2),
                "flop_per_launch": g_flop / g_launch,
                "share_of_kernel_time": round(g_ms / total_ms, 3)}
    return {"ms_per_step": ms_per_step, "tokens": tokens, "ms_per_scale": ms_scale, "dense": dense,
            "roofline": roofline, "kernels": report}


def sweep(fv, torch, wl, steps, warmup):
    """Keep ratio {1, 1/2, 3/10, 1/5} x rank {16, 64, 128} on the late scales {40, 48, 64} of the
    Infinity-2B shape at batch 16 x 2, the dense chain as control: one row per combination with the
    time per late scale.  The rank only enters the fill, so the ranks other than the workload's
    own are timed at the workload's keep ratio."""
    import dataclasses
    W0 = wl.WORKLOADS[SWEEP_WORKLOAD]
    chain = Chain(W0, fv, torch)
    rows, dense = [], None
    combos = [(1, 1, W0.rank), (1, 2, W0.rank), (3, 10, W0.rank), (1, 5, W0.rank), (3, 10, 16), (3, 10, 128)]
    for num, den, r in combos:
        W = dataclasses.replace(W0, keep_num=num, keep_den=den, rank=r)
        chain.set_reduction(W)
        m = measure(chain, W, fv, torch, steps, warmup, with_dense=dense is None, dense_steps=2)
        dense = dense or m["dense"]
        rows.append({"keep": f"{num}/{den}", "rank": r,
                     "k": {str(s): W.keep(s) for s in W.late_scales},
                     "ms_per_step": round(m["ms_per_step"], 2),
                     "ms_per_scale": {k: round(v, 2) for k, v in m["ms_per_scale"].items()},
                     "speedup_vs_dense": round(dense["ms_per_step"] / m["ms_per_step"], 3),
                     "tokens_per_s": m["tokens"] / (m["ms_per_step"] * 1e-3),
                     "gemm_frac_of_mfma_peak": m["roofline"]["frac"],
                     "attention": m["kernels"].get("attention"), "fill": m["kernels"].get("fill"),
                     "score": m["kernels"].get("score")})
    return W0, rows, dense


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the random-projection input variant and the factor construction")
    ap.add_argument("--workload", default=WORKLOAD, choices=None,
                    help="another shape of workloads.WORKLOADS (default: the largest one, hidden "
                         "4096 at the 80x80 scale, which the headline figure is quoted on)")
    ap.add_argument("--keep", default=None, metavar="NUM/DEN",
                    help="keep ratio instead of the workload's (e.g. 3/10); 1/1 runs every row")
    ap.add_argument("--rank", type=int, default=None, help="fill rank instead of the workload's")
    ap.add_argument("--sweep", action="store_true",
                    help=f"keep-ratio x rank x scale table of {SWEEP_WORKLOAD} instead of one workload")
    ap.add_argument("--constant-operands", action="store_true",
                    help="overwrite every input, weight, cache and factor with the constant 1.0 "
                         "before timing: same launches and flop counts on operands that toggle no "
                         "bits, which shows how much of the step time is the chip's clock governor "
                         "(the line says data: constant and is no throughput figure)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB device copy (reference for scaling HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path has no multi-GPU part (run with --gpus 1)")

    import torch
    import paper_2512_16483_amd as fv
    import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.sweep:
        W, rows, dense = sweep(fv, torch, wl, max(2, args.steps // 3), max(1, args.warmup // 2))
        ref = next(r for r in rows if r["keep"] == f"{W.keep_num}/{W.keep_den}" and r["rank"] == W.rank)
        print(json.dumps({
            "metric": "late-scale pruned block throughput (tokens/s; ms per late scale in ms_per_scale)",
            "value": ref["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": max(2, args.steps // 3),
            "warmup": max(1, args.warmup // 2), "ms_per_step": ref["ms_per_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": W.dtype,
            "data": "synthetic",
            "config": {"workload": SWEEP_WORKLOAD + " (keep x rank sweep)", "hidden": W.hidden,
                       "heads": W.heads, "head_dim": W.head_dim, "blocks": W.blocks, "batch": W.batch,
                       "late_scales": list(W.late_scales), "kv_tokens": W.total_len()},
            "dense_control": dense, "sweep": rows}))
        return

    if args.workload not in wl.WORKLOADS:
        sys.exit(f"unknown workload {args.workload}; known: {', '.join(wl.WORKLOADS)}")
    default_wl = args.workload == WORKLOAD
    W = wl.WORKLOADS[args.workload]
    if W.dtype != "bf16":
        sys.exit("bench.py times the bf16 shapes; the fp32 shape is a parity configuration")
    if args.keep or args.rank:
        import dataclasses
        num, den = (int(t) for t in args.keep.split("/")) if args.keep else (W.keep_num, W.keep_den)
        W = dataclasses.replace(W, keep_num=num, keep_den=den, rank=args.rank or W.rank)
        default_wl = False
    chain = Chain(W, fv, torch)
    if args.constant_operands:
        default_wl = False
        for w, K, V in chain.blocks:
            for t in list(w.values()) + [K, V]:
                t.fill_(1.0)
        for s in chain.scale.values():
            for t in [s["x0"]] + list(s["Wc"]) + list(s["Gc"]):
                t.fill_(1.0)

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    m = measure(chain, W, fv, torch, args.steps, args.warmup, with_dense=not args.no_dense)
    ms_per_step, tokens, dense = m["ms_per_step"], m["tokens"], m["dense"]
    traffic = GEMM_TRAFFIC.get(args.workload) if not (args.keep or args.rank) else None
    if args.constant_operands:
        traffic = None
    if traffic:
        m["roofline"]["traffic"] = traffic["bytes_per_launch"]
        m["roofline"]["traffic_source"] = traffic["source"]

    out = {
        "metric": "late-scale pruned block throughput (tokens/s; ms per late scale in ms_per_scale)",
        "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": W.dtype,
        "data": "constant" if args.constant_operands else "synthetic",
        "config": {"workload": args.workload, "hidden": W.hidden, "heads": W.heads,
                   "head_dim": W.head_dim, "blocks": W.blocks, "batch": W.batch,
                   "late_scales": list(W.late_scales), "keep_ratio": W.keep_num / W.keep_den,
                   "rank": W.rank, "kv_tokens": W.total_len()},
        "ms_per_scale": m["ms_per_scale"],
        "dense_control": dense,
        "speedup_vs_dense": (dense["ms_per_step"] / ms_per_step) if dense else None,
        "roofline": m["roofline"],
        "kernels": m["kernels"],
    }
    if not args.no_variants and default_wl:
        out["variants"] = variants(chain, W, fv, torch, max(2, args.steps // 3))
    if not args.no_cpu_baseline:
        # bounded sample: one block, one sample, the first late scale
        out["cpu_baseline"] = cpu_baseline(W, W.late_scales[:1])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
