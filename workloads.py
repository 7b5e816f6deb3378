"""Seeded synthetic workloads: shapes and random tensors only.

This module serves both the CPU oracle's tests and the HIP path's tests/bench.
It holds none of the method's arithmetic (no entropy, selection, attention,
interpolation): only the five workload shapes, the keep-count table and
counter-based (Philox) random tensors, so that both sides see identical bytes.

Every tensor is a pure function of (seed, tensor id, block index, scale grid).
Values are drawn in float32 on the host and rounded once to the workload's
storage dtype (float32 or bfloat16).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np
import torch


# ----------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Scale:
    """One pruned next-scale step: current grid, prior grid, cached KV rows."""
    grid: int          # h = w of the current scale
    prev_grid: int     # hp = wp of the prior scale (source of the residual cache)
    kv_len: int        # P: rows already in the KV cache (all prior scales)

    @property
    def N(self) -> int:
        return self.grid * self.grid


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16" (storage of activations/weights)
    B: int
    C: int
    heads: int
    L: int                     # transformer blocks
    V: int                     # codebook size
    keep_hi: float             # keep ratio at block 0
    keep_lo: float             # keep ratio at block L-1
    scales: Tuple[Scale, ...]  # pruned scales, last one is the headline step
    seed: int = 0
    ffn_mult: int = 4

    @property
    def last(self) -> Scale:
        return self.scales[-1]

    @property
    def dh(self) -> int:
        return self.C // self.heads

    @property
    def F(self) -> int:
        return self.ffn_mult * self.C

    def keep_ratio(self, j: int) -> float:
        if self.L == 1:
            return self.keep_hi
        return self.keep_hi + (self.keep_lo - self.keep_hi) * j / (self.L - 1)

    def k(self, j: int, scale: Scale | None = None) -> int:
        """Kept tokens per batch row at block j: ceil(keep_j * N), never pruning
        more than the ratio asks for; clamped to [0, N]."""
        s = scale or self.last
        return keep_count(self.keep_ratio(j), s.N)

    def k_table(self, scale: Scale | None = None) -> List[int]:
        return [self.k(j, scale) for j in range(self.L)]

    def kv_capacity(self, scale: Scale | None = None) -> int:
        """Rows allocated per KV cache: P + N rounded up to a multiple of 64."""
        s = scale or self.last
        return (s.kv_len + s.N + 63) // 64 * 64


def keep_count(keep: float, N: int) -> int:
    k = int(math.ceil(keep * N - 1e-9))
    return max(0, min(N, k))


def _prefix(grids: List[int], upto: int) -> int:
    return sum(g * g for g in grids[:upto])


_G256 = [1, 2, 3, 4, 5, 6, 8, 10, 13, 16]
_G512 = [1, 2, 3, 4, 6, 9, 13, 18, 24, 32]
_G1024 = [1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64]


def _scales(grids: List[int], first_pruned: int) -> Tuple[Scale, ...]:
    out = []
    for t, g in enumerate(grids):
        if g >= first_pruned:
            out.append(Scale(grid=g, prev_grid=grids[t - 1], kv_len=_prefix(grids, t)))
    return tuple(out)


def grid_list(wl: "Workload") -> List[int]:
    """The full list of scale grids the workload's pruned scales belong to."""
    last = wl.scales[-1]
    for grids in (_G256, _G512, _G1024):
        if last.grid in grids and last.kv_len == _prefix(grids, grids.index(last.grid)):
            return list(grids)
    raise ValueError("the workload's scales match no known grid list")


WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1-tiny-f32", "f32", B=1, C=64, heads=4, L=1, V=512,
                     keep_hi=0.5, keep_lo=0.5, scales=_scales(_G256, 16)),
    "cfg2": Workload("cfg2-var-d16", "bf16", B=8, C=1024, heads=16, L=16, V=4096,
                     keep_hi=0.8, keep_lo=0.4, scales=_scales(_G256, 16)),
    "cfg3": Workload("cfg3-var-d30", "bf16", B=16, C=1920, heads=30, L=30, V=4096,
                     keep_hi=0.7, keep_lo=0.3, scales=_scales(_G256, 13)),
    "cfg4": Workload("cfg4-512px", "bf16", B=8, C=2304, heads=36, L=36, V=4096,
                     keep_hi=0.5, keep_lo=0.5, scales=_scales(_G512, 18)),
    "cfg5": Workload("cfg5-1024px", "bf16", B=2, C=2048, heads=16, L=32, V=4096,
                     keep_hi=0.6, keep_lo=0.2, scales=_scales(_G1024, 32)),
}


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
_TENSOR_IDS = {
    "logits": 1, "temperature": 2, "x": 3, "k_cache": 4, "v_cache": 5, "cache_prev": 6,
    "w_qkv": 10, "b_qkv": 11, "w_o": 12, "b_o": 13, "w_fc1": 14, "b_fc1": 15,
    "w_fc2": 16, "b_fc2": 17, "ada": 20, "qk_scale": 21,
    "w_cq": 22, "b_cq": 23, "w_co": 24, "b_co": 25, "k_text": 26, "v_text": 27,
}


def _rng(seed: int, name: str, block: int, grid: int) -> np.random.Generator:
    key = (np.uint64(seed) << np.uint64(32)) | np.uint64(_TENSOR_IDS[name])
    ctr = [np.uint64(block), np.uint64(grid), np.uint64(0), np.uint64(0)]
    return np.random.Generator(np.random.Philox(key=[key, np.uint64(0x4E4F5641)], counter=ctr))


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def _normal(seed, name, block, grid, shape, std, dtype) -> torch.Tensor:
    g = _rng(seed, name, block, grid)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return torch.from_numpy(a).to(torch_dtype(dtype))


def make_logits(wl: Workload, block: int, scale: Scale | None = None,
                dtype: str | None = None, B: int | None = None) -> torch.Tensor:
    """[B, N, V] codebook logits: N(0, s_t^2), one temperature s_t per token,
    log-uniform in [0.1, 10]."""
    s = scale or wl.last
    B = wl.B if B is None else B
    gt = _rng(wl.seed, "temperature", block, s.grid)
    temp = np.exp(gt.uniform(math.log(0.1), math.log(10.0), size=(B, s.N, 1))).astype(np.float32)
    g = _rng(wl.seed, "logits", block, s.grid)
    a = g.standard_normal(size=(B, s.N, wl.V), dtype=np.float32)
    a *= temp
    return torch.from_numpy(a).to(torch_dtype(dtype or wl.dtype))


def make_x(wl: Workload, scale: Scale | None = None) -> torch.Tensor:
    s = scale or wl.last
    return _normal(wl.seed, "x", 0, s.grid, (wl.B, s.N, wl.C), 1.0, wl.dtype)


def make_cache_prev(wl: Workload, block: int, scale: Scale | None = None) -> torch.Tensor:
    """Prior-scale residual cache on the prior grid: [B, hp*wp, C], N(0,1)."""
    s = scale or wl.last
    return _normal(wl.seed, "cache_prev", block, s.grid,
                   (wl.B, s.prev_grid * s.prev_grid, wl.C), 1.0, wl.dtype)


def make_kv_prior(wl: Workload, block: int, scale: Scale | None = None
                  ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Prior-scale keys and values in the logical layout [B, P, C], N(0,1)."""
    s = scale or wl.last
    kc = _normal(wl.seed, "k_cache", block, s.grid, (wl.B, s.kv_len, wl.C), 1.0, wl.dtype)
    vc = _normal(wl.seed, "v_cache", block, s.grid, (wl.B, s.kv_len, wl.C), 1.0, wl.dtype)
    return kc, vc


def make_weights(wl: Workload, block: int) -> Dict[str, torch.Tensor]:
    """Block weights, N(0, 0.02^2), stored out-feature major ([out, in]) so that
    a projection is y = u @ W.T + b."""
    C, F = wl.C, wl.F
    shapes = {
        "w_qkv": (3 * C, C), "b_qkv": (3 * C,), "w_o": (C, C), "b_o": (C,),
        "w_fc1": (F, C), "b_fc1": (F,), "w_fc2": (C, F), "b_fc2": (C,),
    }
    return {n: _normal(wl.seed, n, block, 0, shp, 0.02, wl.dtype) for n, shp in shapes.items()}


def make_block_variant(wl: Workload, block: int, text_len: int = 77) -> Dict[str, torch.Tensor]:
    """Inputs of the block variants: per-image conditioning vectors `ada` [B, 6, C] (shift1, scale1,
    gate1, shift2, scale2, gate2; shifts and scales N(0, 0.2^2), gates 1 + N(0, 0.2^2)) in the
    workload's dtype, the per-head score multiplier `qk_scale` [heads] fp32, uniform in [4, 16], and a
    cross-attention sub-layer: projections N(0, 0.02^2) like the other weights, projected keys / values
    of `text_len` condition tokens [B, text_len, C], N(0, 1)."""
    g = _rng(wl.seed, "ada", block, 0)
    ada = g.standard_normal(size=(wl.B, 6, wl.C), dtype=np.float32) * np.float32(0.2)
    ada[:, 2] += np.float32(1.0)
    ada[:, 5] += np.float32(1.0)
    gs = _rng(wl.seed, "qk_scale", block, 0)
    qk_scale = gs.uniform(4.0, 16.0, size=(wl.heads,)).astype(np.float32)
    C = wl.C
    cross = {n: _normal(wl.seed, n, block, 0, shp, 0.02, wl.dtype)
             for n, shp in {"w_cq": (C, C), "b_cq": (C,), "w_co": (C, C), "b_co": (C,)}.items()}
    cross["k_text"] = _normal(wl.seed, "k_text", block, 0, (wl.B, text_len, C), 1.0, wl.dtype)
    cross["v_text"] = _normal(wl.seed, "v_text", block, 0, (wl.B, text_len, C), 1.0, wl.dtype)
    return {"ada": torch.from_numpy(ada).to(torch_dtype(wl.dtype)), "qk_scale": torch.from_numpy(qk_scale),
            "cross": cross}


def small_variant(wl: Workload, B: int | None = None, L: int | None = None) -> Workload:
    """Same widths, fewer batch rows / blocks (used to bound oracle time)."""
    from dataclasses import replace
    return replace(wl, B=wl.B if B is None else B, L=wl.L if L is None else L)
