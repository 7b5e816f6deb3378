"""One next-scale step through L entropy-pruned blocks: a sequence of C-ABI calls.

For every block j:  nova_entropy -> nova_select -> nova_pruned_block -> nova_merge_cache,
all enqueued on the current stream with no host synchronisation in between (the keep
count k_j is an input).  This module only owns device buffers and call order.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import torch

from .binding import NOVA_BF16, NOVA_F32, BlockShape, BlockVariant, Nova


@dataclass
class BlockState:
    """Device-resident inputs and outputs of one block at one step."""
    k: int
    logits: torch.Tensor                 # [B, N, V]
    weights: Dict[str, torch.Tensor]
    k_cache: torch.Tensor                # [B, heads, cap, dh]
    v_cache: torch.Tensor                # [B, heads, dh, cap]
    cache_prev: Optional[torch.Tensor]   # [B, hp*wp, C]
    entropy: torch.Tensor = None         # [B, N] f32
    kept_idx: torch.Tensor = None        # [B, k] i32
    keep_mask: torch.Tensor = None       # [B, N] u8
    y_kept: torch.Tensor = None          # [B, k, C]
    out: torch.Tensor = None             # [B, N, C]
    cache_new: torch.Tensor = None       # [B, N, C]
    variant: Optional[BlockVariant] = None   # block variations (nova_pruned_block_variant); None = the base block


class StepRunner:
    def __init__(self, nova: Nova, *, B: int, grid: int, prev_grid: int, C: int, heads: int, kv_len: int,
                 kv_capacity: int, dtype: torch.dtype, ffn_mult: int = 4):
        self.nova = nova
        self.B, self.grid, self.prev_grid, self.C, self.heads = B, grid, prev_grid, C, heads
        self.N = grid * grid
        self.kv_len, self.kv_capacity, self.ffn_mult = kv_len, kv_capacity, ffn_mult
        self.dtype = dtype
        self.code = NOVA_BF16 if dtype == torch.bfloat16 else NOVA_F32
        self.blocks: List[BlockState] = []
        self._workspace: Optional[torch.Tensor] = None

    def shape(self, k: int) -> BlockShape:
        return BlockShape(self.code, self.B, self.N, self.C, self.heads, self.kv_len, self.kv_capacity, k,
                          self.ffn_mult)

    def add_block(self, st: BlockState) -> BlockState:
        dev = st.logits.device
        B, N, C = self.B, self.N, self.C
        st.entropy = torch.empty((B, N), dtype=torch.float32, device=dev)
        st.kept_idx = torch.empty((B, max(st.k, 1)), dtype=torch.int32, device=dev)
        st.keep_mask = torch.empty((B, N), dtype=torch.uint8, device=dev)
        st.y_kept = torch.empty((B, max(st.k, 1), C), dtype=self.dtype, device=dev)
        st.out = torch.empty((B, N, C), dtype=self.dtype, device=dev)
        st.cache_new = torch.empty((B, N, C), dtype=self.dtype, device=dev)
        need = self.nova.workspace_bytes(self.shape(st.k))
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        self.blocks.append(st)
        return st

    def run_block(self, st: BlockState, x: torch.Tensor) -> torch.Tensor:
        n = self.nova
        n.entropy(st.logits, st.entropy)
        n.select(st.entropy, st.k, st.kept_idx, st.keep_mask)
        if st.variant is None:
            n.pruned_block(self.shape(st.k), st.weights, x, st.kept_idx, st.k_cache, st.v_cache, st.y_kept,
                           self._workspace)
        else:
            n.pruned_block_variant(self.shape(st.k), st.weights, st.variant, x, st.kept_idx, st.k_cache,
                                   st.v_cache, st.y_kept, self._workspace)
        n.merge_cache(self.grid, self.grid, self.prev_grid, self.prev_grid, st.k, x, st.y_kept, st.kept_idx,
                      st.keep_mask, st.cache_prev, st.out, st.cache_new)
        return st.out

    def run_step(self, x: torch.Tensor) -> torch.Tensor:
        for st in self.blocks:
            x = self.run_block(st, x)
        return x
