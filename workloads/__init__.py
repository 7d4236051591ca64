"""Workload shapes and seeded synthetic inputs.

Shared by the CPU oracle's tests and the GPU path's tests / benchmark.  Holds no
arithmetic of the method itself: only shapes, scale schedules and random tensors.
All tensors come out as fp32 numpy arrays; with `bf16=True` the values are first
rounded to the nearest bf16 (ties to even) so that both sides start from exactly
the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    hidden: int
    heads: int
    head_dim: int
    ffn_hidden: int
    scales: Tuple[int, ...]            # side length of each (square) scale
    late_scales: Tuple[int, ...]       # the scales run through the reduced block
    keep_num: int                      # keep ratio = keep_num / keep_den
    keep_den: int
    rank: int
    batch: int
    blocks: int
    dtype: str                         # "f32" | "bf16"

    def tokens(self, side: int) -> int:
        return side * side

    def prev_len(self, side: int) -> int:
        """L_prev: number of cached tokens of all scales before `side`."""
        i = self.scales.index(side)
        return sum(s * s for s in self.scales[:i])

    def total_len(self) -> int:
        return sum(s * s for s in self.scales)

    def keep(self, side: int) -> int:
        """k = ceil(M * num / den) in integer arithmetic, clamped to [1, M]."""
        M = side * side
        k = -((-M * self.keep_num) // self.keep_den)
        return max(1, min(M, k))


_INF = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)

WORKLOADS: Dict[str, Workload] = {
    # single VAR-d16-shaped block at the last scale, fp32 parity case
    "var_d16_s16_f32": Workload("var_d16_s16_f32", 1024, 16, 64, 4096,
                                (1, 2, 3, 4, 5, 6, 8, 10, 13, 16), (16,), 1, 2, 32, 1, 1, "f32"),
    # VAR-d30-shaped late scales at 512 px: the configuration the benchmark times
    "var_d30_512_bf16": Workload("var_d30_512_bf16", 1920, 30, 64, 7680,
                                 (1, 2, 3, 4, 6, 9, 13, 18, 24, 32), (24, 32), 2, 5, 64, 8, 30,
                                 "bf16"),
    # Infinity-2B-shaped 1024 px, batch 1
    "infinity2b_1024_bf16": Workload("infinity2b_1024_bf16", 2048, 16, 128, 8192, _INF,
                                     (40, 48, 64), 3, 10, 64, 1, 32, "bf16"),
    # same, batch 16 with classifier-free-guidance doubling (effective batch 32)
    "infinity2b_1024_b32_bf16": Workload("infinity2b_1024_b32_bf16", 2048, 16, 128, 8192, _INF,
                                         (40, 48, 64), 3, 10, 64, 32, 32, "bf16"),
    # STAR-1.7B-shaped: 30 blocks, the reduction applied at the 64x64 scale only (the paper's
    # setting for that model); block geometry assumed from the parameter count (1.7e9 / 30 blocks
    # / 12 d^2 gives d close to 2048), keep ratio = the paper's mean rank fraction 17.6 %
    "star_shaped_1024_bf16": Workload("star_shaped_1024_bf16", 2048, 16, 128, 8192, _INF,
                                      (64,), 22, 125, 64, 4, 30, "bf16"),
    # large-model shape with an extra 80x80 final scale
    "large_1280_bf16": Workload("large_1280_bf16", 4096, 32, 128, 16384, _INF + (80,),
                                (80,), 1, 4, 128, 4, 40, "bf16"),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of fp32 values onto the bf16 grid (result still fp32)."""
    a = np.ascontiguousarray(a, np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _q(a: np.ndarray, bf16: bool) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if bf16 else a


def activations_iid(B: int, M: int, d: int, seed: int = 1000, bf16: bool = False) -> np.ndarray:
    """x[B,M,d] ~ N(0,1) i.i.d."""
    return _q(_rng(seed, 0).standard_normal((B, M, d)), bf16)


def activations_lowrank(B: int, M: int, d: int, seed: int = 1000, rank_frac: float = 0.176,
                        noise: float = 0.1, bf16: bool = False) -> np.ndarray:
    """x = diag(a) (A B^T / sqrt(rho) + noise * E): low-rank with heterogeneous row energies.

    rho = ceil(rank_frac * min(M,d)); a_i ~ LogNormal(0, 0.5).  A stand-in for the interpolated
    late-scale input features, which the paper reports to be low rank (17.6 % mean rank fraction
    at 96 % energy) and whose rows are sampled by energy."""
    g = _rng(seed, 1)
    rho = int(np.ceil(rank_frac * min(M, d)))
    out = np.empty((B, M, d), np.float32)
    for b in range(B):
        A = g.standard_normal((M, rho), dtype=np.float32)
        Bm = g.standard_normal((d, rho), dtype=np.float32)
        E = g.standard_normal((M, d), dtype=np.float32)
        a = np.exp(0.5 * g.standard_normal(M)).astype(np.float32)
        out[b] = a[:, None] * (A @ Bm.T / np.float32(np.sqrt(rho)) + np.float32(noise) * E)
    return _q(out, bf16)


def block_weights(d: int, F: int, seed: int = 2000, bf16: bool = False, std: float = 0.02,
                  with_bias: bool = False, with_affine: bool = False) -> Dict[str, np.ndarray]:
    """Weights of one block, `out,in` layout, N(0, std^2); optional biases / LayerNorm affine."""
    g = _rng(seed, 2)
    w = {
        "w_qkv": _q(std * g.standard_normal((3 * d, d)), bf16),
        "w_o": _q(std * g.standard_normal((d, d)), bf16),
        "w_fc1": _q(std * g.standard_normal((F, d)), bf16),
        "w_fc2": _q(std * g.standard_normal((d, F)), bf16),
    }
    if with_bias:
        w["b_qkv"] = _q(std * g.standard_normal(3 * d), bf16)
        w["b_o"] = _q(std * g.standard_normal(d), bf16)
        w["b_fc1"] = _q(std * g.standard_normal(F), bf16)
        w["b_fc2"] = _q(std * g.standard_normal(d), bf16)
    if with_affine:
        w["ln1_g"] = _q(1.0 + 0.1 * g.standard_normal(d), bf16)
        w["ln1_b"] = _q(0.1 * g.standard_normal(d), bf16)
        w["ln2_g"] = _q(1.0 + 0.1 * g.standard_normal(d), bf16)
        w["ln2_b"] = _q(0.1 * g.standard_normal(d), bf16)
    return w


def kv_prefix(B: int, L: int, H: int, Dh: int, seed: int = 3000, bf16: bool = False):
    """Cached keys and values of the earlier scales, each [B,L,H,Dh] ~ N(0,1)."""
    g = _rng(seed, 3)
    K = _q(g.standard_normal((B, L, H, Dh)), bf16)
    V = _q(g.standard_normal((B, L, H, Dh)), bf16)
    return K, V


def cached_feature(B: int, M: int, d: int, rank: int, seed: int = 4000, noise: float = 0.0,
                   bf16: bool = False) -> np.ndarray:
    """Cached counterpart feature C[B,M,d] = A B^T / sqrt(rank) (+ noise * E): rank `rank` exactly
    when noise == 0."""
    g = _rng(seed, 4)
    A = g.standard_normal((B, M, rank))
    Bm = g.standard_normal((B, d, rank))
    Cm = np.einsum("bmr,bdr->bmd", A, Bm) / np.sqrt(rank)
    if noise:
        Cm = Cm + noise * g.standard_normal((B, M, d))
    return _q(Cm, bf16)


def normal_draws(B: int, M: int, r: int, seed: int = 4000) -> np.ndarray:
    """Standard-normal draws z[B,M,r] for the random-projection matrix (fp64)."""
    return _rng(seed, 5).standard_normal((B, M, r))


def direct_factors(B: int, M: int, r: int, d: int, seed: int = 4000, bf16: bool = False):
    """Throughput-only stand-ins for the cache factors: W_c[B,M,r] ~ N(0,1),
    G_c[B,r,d] ~ N(0,1/r).  Same shapes and magnitudes as real factors, no solve involved."""
    g = _rng(seed, 6)
    W = _q(g.standard_normal((B, M, r)), bf16)
    G = _q(g.standard_normal((B, r, d)) / np.sqrt(r), bf16)
    return W, G


# --------------------------------------------------------------------------- device-side generators
# Same recipes as above, drawn with torch's seeded generator directly in GPU memory: the
# throughput workloads hold gigabytes of weights and caches, too much to draw on the host.
def device_workload(W: Workload, side: int, seed: int = 1000, device: str = "cuda"):
    """Synthetic device tensors of one late scale of workload W (torch tensors, W.dtype):
    x0[B,M,d] (low rank + noise, log-normal row scales), per block factors W_c[B,M,r], G_c[B,r,d]."""
    import torch
    dt = torch.bfloat16 if W.dtype == "bf16" else torch.float32
    g = torch.Generator(device=device)
    g.manual_seed(seed + side)
    B, M, d, r = W.batch, side * side, W.hidden, W.rank
    rho = int(np.ceil(0.176 * min(M, d)))
    A = torch.randn((B, M, rho), generator=g, device=device)
    Bm = torch.randn((B, d, rho), generator=g, device=device)
    E = torch.randn((B, M, d), generator=g, device=device)
    a = torch.exp(0.5 * torch.randn((B, M, 1), generator=g, device=device))
    x0 = (a * (A @ Bm.transpose(1, 2) / rho ** 0.5 + 0.1 * E)).to(dt).contiguous()
    Wc = [torch.randn((B, M, r), generator=g, device=device).to(dt) for _ in range(W.blocks)]
    Gc = [(torch.randn((B, r, d), generator=g, device=device) / r ** 0.5).to(dt)
          for _ in range(W.blocks)]
    return x0, Wc, Gc


def device_block_state(W: Workload, seed: int = 2000, device: str = "cuda"):
    """Per block: weights N(0, 0.02^2) (`out,in`, no bias, no affine) and a KV cache
    [B, total_len, H, Dh] ~ N(0,1) that stands for the keys/values of the earlier scales."""
    import torch
    dt = torch.bfloat16 if W.dtype == "bf16" else torch.float32
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    d, F, B, L = W.hidden, W.ffn_hidden, W.batch, W.total_len()
    blocks = []
    for _ in range(W.blocks):
        w = {"w_qkv": (0.02 * torch.randn((3 * d, d), generator=g, device=device)).to(dt),
             "w_o": (0.02 * torch.randn((d, d), generator=g, device=device)).to(dt),
             "w_fc1": (0.02 * torch.randn((F, d), generator=g, device=device)).to(dt),
             "w_fc2": (0.02 * torch.randn((d, F), generator=g, device=device)).to(dt)}
        K = torch.randn((B, L, W.heads, W.head_dim), generator=g, device=device).to(dt)
        V = torch.randn((B, L, W.heads, W.head_dim), generator=g, device=device).to(dt)
        blocks.append((w, K, V))
    return blocks
