"""All scales of one batch of images through L blocks: a sequence of C-ABI calls.

Scales up to and including the activation scale t* run dense: every token is kept, which
builds each block's K/V cache and, from t* on, its residual cache (Sec. 3.3, "Residual Cache
Reuse": the cache is active for t >= t*).  Later scales run the entropy-pruned path of
:mod:`paper_2602_01345_amd.step`; a block's new residual cache becomes its prior cache at the
next scale, and only the kept tokens' K/V rows are appended, so the blocks' cache lengths drift
apart.  This module owns device buffers and call order only; every step runs in the library.

A scale whose keep counts are known on the host beforehand (dense scales, table-driven pruned
scales) can be planned: :meth:`ImageRunner.plan_image` lays out static buffers for every scale and
:meth:`ScalePlan.capture` records the scale's launches into a HIP graph, so the many small launches of
the early scales are replayed with one call instead of being issued one by one from Python.

Keep counts at a pruned scale come either from a table (host integers) or from the layer-linkage
controller (``nova_layer_ratio`` on the device).  In controller mode every image has its own count
per block and the counts never leave the device: selection, block and merge take them as a device
array (``nova_select`` / ``nova_pruned_block_rows`` / ``nova_merge_cache_rows``) with the row pitch
N, and each block's per-image cache lengths are kept in a device array that the block call itself
advances.  Nothing on that path synchronises with the host.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import torch

from .binding import NOVA_BF16, NOVA_F32, BlockShape, BlockVariant, Nova


@dataclass
class ScaleResult:
    """What one scale produced (device tensors are views of the runner's buffers of that scale)."""
    out: torch.Tensor                     # [B, N, C] output of the last block
    k: List[object]                       # per block: the keep count (int), or in controller mode a [B] int32
                                          # device tensor with every image's own count
    mean_entropy: Optional[torch.Tensor]  # [B] scale mean entropy of the last block's logits, if logits were given
    block_out: List[torch.Tensor]         # per block [B, N, C] (kept for inspection)
    block_cache: List[torch.Tensor]       # per block residual cache [B, N, C]
    block_entropy: List[torch.Tensor]     # with inspect=True: per block [B, N] fp32 token entropies (pruned scales)
    block_idx: List[torch.Tensor]         # with inspect=True: per block [B, k] kept indices


@dataclass
class ScalePlan:
    """Static buffers and launch parameters of one scale of a planned image (table-driven counts)."""
    t: int
    grid: int
    prev_grid: int
    k: List[int]                          # keep count per block
    kv_len: List[int]                     # rows in each block's K/V cache before this scale
    x: torch.Tensor                       # [B, N, C] input buffer (the caller copies the scale's input here)
    logits: Optional[List[torch.Tensor]]  # per block [B, N, V] for a pruned scale
    entropy: Optional[torch.Tensor]
    idx: List[torch.Tensor]               # per block [B, k] (dense: one shared identity)
    mask: List[torch.Tensor]              # per block [B, N]
    y: List[torch.Tensor]
    out: List[torch.Tensor]
    cache_new: List[Optional[torch.Tensor]]
    cache_prev: List[Optional[torch.Tensor]]
    graph: Optional[torch.cuda.CUDAGraph] = None


class ImageRunner:
    def __init__(self, nova: Nova, *, B: int, C: int, heads: int, grids: Sequence[int], dtype: torch.dtype,
                 weights: List[Dict[str, torch.Tensor]], ffn_mult: int = 4, device: str = "cuda",
                 variants: Optional[List[Optional[BlockVariant]]] = None, interp: int = 0):
        """variants: per block, the block variations (nova_pruned_block_variant) or None; interp: the cache
        interpolation kernel of nova_merge_cache_interp (0 bilinear, 1 nearest, 2 bicubic)."""
        self.nova = nova
        self.variants = variants if variants is not None else [None] * len(weights)
        self.interp = interp
        self.B, self.C, self.heads, self.ffn_mult = B, C, heads, ffn_mult
        self.grids = list(grids)
        self.dtype = dtype
        self.code = NOVA_BF16 if dtype == torch.bfloat16 else NOVA_F32
        self.weights = weights
        self.L = len(weights)
        self.device = device
        dh = C // heads
        self.cap = (sum(g * g for g in self.grids) + 63) // 64 * 64
        self.k_cache = [torch.zeros((B, heads, self.cap, dh), dtype=dtype, device=device) for _ in range(self.L)]
        self.v_cache = [torch.zeros((B, heads, dh, self.cap), dtype=dtype, device=device) for _ in range(self.L)]
        self.kv_len = [0] * self.L                      # rows appended so far, per block
        self.cache: List[Optional[torch.Tensor]] = [None] * self.L     # residual cache of the previous scale
        self.cache_grid: Optional[int] = None
        self._workspace: Optional[torch.Tensor] = None
        self._state = torch.zeros(B, dtype=torch.float32, device=device)      # layer-ratio running sums
        self._ratio_tj = torch.empty(B, dtype=torch.float32, device=device)
        self._k_row = torch.empty(B, dtype=torch.int32, device=device)
        # per-image cache lengths of every block (device): exact once images keep different numbers of tokens;
        # kv_len then holds the host's upper bound
        self.kv_rows = [torch.zeros(B, dtype=torch.int32, device=device) for _ in range(self.L)]

    def reset(self):
        """Forget the previous image: cache lengths back to zero, no residual cache (buffers are reused)."""
        self.kv_len = [0] * self.L
        self.cache = [None] * self.L
        self.cache_grid = None
        for t in self.kv_rows:
            t.zero_()

    def _shape(self, N: int, j: int, k: int) -> BlockShape:
        return BlockShape(self.code, self.B, N, self.C, self.heads, self.kv_len[j], self.cap, k, self.ffn_mult)

    def _ensure_workspace(self, shape: BlockShape):
        need = self.nova.workspace_bytes(shape)
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)

    # -- planned (allocation-free, graph-capturable) execution -----------------------------------
    def plan_image(self, k_tables: Dict[int, Sequence[int]], logits: Dict[int, List[torch.Tensor]],
                   first_cache_scale: int) -> List[ScalePlan]:
        """Plans every scale in order.  k_tables[t] gives the keep counts of a pruned scale t (scales
        without an entry run dense); residual caches are kept from scale first_cache_scale on."""
        B, C, dev = self.B, self.C, self.device
        plans: List[ScalePlan] = []
        kv = [0] * self.L
        prev_cache: List[Optional[torch.Tensor]] = [None] * self.L
        prev_grid = None
        need = 0
        for t, g in enumerate(self.grids):
            N = g * g
            dense = t not in k_tables
            ks = [N] * self.L if dense else [int(k) for k in k_tables[t]]
            keep = t >= first_cache_scale
            if dense:
                ident = torch.arange(N, dtype=torch.int32, device=dev).expand(B, N).contiguous()
                ones = torch.ones((B, N), dtype=torch.uint8, device=dev)
                idx, mask = [ident] * self.L, [ones] * self.L
            else:
                idx = [torch.empty((B, max(k, 1)), dtype=torch.int32, device=dev) for k in ks]
                mask = [torch.empty((B, N), dtype=torch.uint8, device=dev) for _ in ks]
            plan = ScalePlan(
                t=t, grid=g, prev_grid=prev_grid if prev_cache[0] is not None else g, k=ks, kv_len=list(kv),
                x=torch.empty((B, N, C), dtype=self.dtype, device=dev),
                logits=None if dense else logits[t],
                entropy=None if dense else torch.empty((B, N), dtype=torch.float32, device=dev),
                idx=idx, mask=mask,
                y=[torch.empty((B, max(k, 1), C), dtype=self.dtype, device=dev) for k in ks],
                out=[torch.empty((B, N, C), dtype=self.dtype, device=dev) for _ in ks],
                cache_new=[torch.empty((B, N, C), dtype=self.dtype, device=dev) if keep else None for _ in ks],
                cache_prev=list(prev_cache))
            for j, k in enumerate(ks):
                need = max(need, self.nova.workspace_bytes(
                    BlockShape(self.code, B, N, C, self.heads, kv[j], self.cap, k, self.ffn_mult)))
                kv[j] += k
            if keep:
                prev_cache, prev_grid = plan.cache_new, g
            plans.append(plan)
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        return plans

    def enqueue(self, plan: ScalePlan) -> torch.Tensor:
        """Issues the launches of a planned scale on the current stream (no allocation, no host sync)."""
        n, g = self.nova, plan.grid
        N = g * g
        x = plan.x
        for j in range(self.L):
            k = plan.k[j]
            if plan.logits is not None:
                n.entropy(plan.logits[j], plan.entropy)
                n.select(plan.entropy, k, plan.idx[j], plan.mask[j])
            shape = BlockShape(self.code, self.B, N, self.C, self.heads, plan.kv_len[j], self.cap, k, self.ffn_mult)
            n.pruned_block_variant(shape, self.weights[j], self.variants[j], x, plan.idx[j], self.k_cache[j],
                                   self.v_cache[j], plan.y[j], self._workspace)
            n.merge_cache_interp(self.interp, g, g, plan.prev_grid, plan.prev_grid, k, x, plan.y[j], plan.idx[j],
                                 plan.mask[j], plan.cache_prev[j], plan.out[j], plan.cache_new[j])
            x = plan.out[j]
        return x

    def capture(self, plan: ScalePlan):
        """Records the scale's launches into a HIP graph (after one eager run that warms every code path)."""
        self.enqueue(plan)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.enqueue(plan)
        plan.graph = graph

    def launch(self, plan: ScalePlan) -> torch.Tensor:
        """Replays the scale's graph if it has one, otherwise issues its launches."""
        if plan.graph is not None:
            plan.graph.replay()
            return plan.out[-1]
        return self.enqueue(plan)

    # -- eager execution with per-call buffers ------------------------------------------------
    def run_scale(self, t: int, x: torch.Tensor, *, logits: Optional[List[torch.Tensor]] = None,
                  k_table: Optional[Sequence[int]] = None, ratio_t: Optional[torch.Tensor] = None,
                  keep_cache: bool = True, inspect: bool = False) -> ScaleResult:
        """Scale index t (0-based into ``grids``).  Dense when neither k_table nor ratio_t is given.

        logits    per block [B, N, V]; needed for a pruned scale, optional for a dense one (then
                  only the last block's are used, for the scale mean entropy)
        k_table   keep count of every block (host integers)
        ratio_t   [B] fp32 device tensor: the scale-linkage ratio of every image; the per-layer
                  counts then come from the layer-linkage controller
        """
        n, B, C = self.nova, self.B, self.C
        g = self.grids[t]
        N = g * g
        dense = k_table is None and ratio_t is None
        dev = self.device
        H = torch.empty((B, N), dtype=torch.float32, device=dev)
        mean = torch.empty(B, dtype=torch.float32, device=dev)
        mask = torch.empty((B, N), dtype=torch.uint8, device=dev)
        idx = torch.empty((B, N), dtype=torch.int32, device=dev)
        if dense:
            idx.copy_(torch.arange(N, dtype=torch.int32, device=dev).expand(B, N))
            mask.fill_(1)
        ks: List[int] = []
        outs: List[torch.Tensor] = []
        caches: List[torch.Tensor] = []
        ents: List[torch.Tensor] = []
        idxs: List[torch.Tensor] = []
        have_mean = False
        for j in range(self.L):
            k_rows = None                             # per-image counts of this block (device), controller mode only
            if dense:
                k = N
                if logits is not None and j == self.L - 1:
                    n.entropy(logits[j], H, mean)
                    have_mean = True
            else:
                n.entropy(logits[j], H, mean)
                have_mean = True
                if ratio_t is not None:
                    # per-image counts, on the device from here to the merge: row pitch N
                    n.layer_ratio(mean, self._state, ratio_t, j + 1, N, self._ratio_tj, self._k_row)
                    k, k_rows = N, self._k_row
                else:
                    k, k_rows = int(k_table[j]), None
                n.select(H, k, idx, mask, k_per_row=k_rows)
            shape = self._shape(N, j, k)
            self._ensure_workspace(shape)
            y = torch.empty((B, max(k, 1), C), dtype=self.dtype, device=dev)
            out = torch.empty((B, N, C), dtype=self.dtype, device=dev)
            cache_new = torch.empty((B, N, C), dtype=self.dtype, device=dev) if keep_cache else None
            # the block reads and advances the per-image cache lengths (equal to kv_len as long as every image
            # has kept the same number of tokens)
            n.pruned_block_rows(shape, self.weights[j], self.variants[j], k_rows, self.kv_rows[j], self.kv_rows[j], x,
                                idx, self.k_cache[j], self.v_cache[j], y, self._workspace)
            pg = self.cache_grid if self.cache[j] is not None else g
            if k_rows is None:
                n.merge_cache_interp(self.interp, g, g, pg, pg, k, x, y, idx, mask, self.cache[j], out, cache_new)
            else:
                n.merge_cache_rows(self.interp, g, g, pg, pg, k, k_rows, x, y, idx, mask, self.cache[j], out, cache_new)
            self.kv_len[j] += k
            if inspect:
                ents.append(H.clone())
                idxs.append(idx.flatten()[:B * k].view(B, k).clone())
            if keep_cache:
                self.cache[j] = cache_new
            ks.append(k if k_rows is None else k_rows.clone())
            outs.append(out)
            caches.append(cache_new)
            x = out
        if keep_cache:
            self.cache_grid = g
        return ScaleResult(out=x, k=ks, mean_entropy=mean if have_mean else None, block_out=outs, block_cache=caches,
                           block_entropy=ents, block_idx=idxs)
