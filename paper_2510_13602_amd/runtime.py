"""Per-layer state of the decode path: caller-owned tensors and the order of the four calls.

Allocation and call sequencing only; all arithmetic happens inside libnosa.  One ``LayerCache``
owns the paged GPU pool, the residency maps, the pooled keys / importance and the per-step
outputs of one layer; the host pool (every block of the cache, pinned) is passed in.
"""
from __future__ import annotations

from typing import Optional

import torch

from .binding import Nosa


def pinned_like(t: torch.Tensor) -> torch.Tensor:
    """A page-locked host copy of ``t`` (hipHostMalloc through PyTorch's pinned allocator)."""
    out = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    out.copy_(t)
    return out


class LayerCache:
    def __init__(self, nosa: Nosa, host_k: torch.Tensor, host_v: torch.Tensor, host_bias: torch.Tensor,
                 n_tokens: torch.Tensor):
        p, dev = nosa.p, nosa.device
        self.nosa = nosa
        B, H, C, nb, d = p.batch, p.n_kv_heads, p.gpu_slots, p.block_size, p.head_dim
        self.host_k, self.host_v, self.host_bias = host_k, host_v, host_bias
        self.n_tokens = n_tokens.to(device=dev, dtype=torch.int32).contiguous()
        dt = nosa.tdtype
        self.pool_k = torch.zeros((B, H, C, nb, d), dtype=dt, device=dev)
        self.pool_v = torch.zeros((B, H, C, nb, d), dtype=dt, device=dev)
        self.pool_bias = torch.zeros((B, H, C, nb), dtype=torch.float32, device=dev)
        self.slot_of_block = torch.full((B, H, p.max_blocks), -1, dtype=torch.int32, device=dev)
        self.block_of_slot = torch.full((B, H, C), -1, dtype=torch.int32, device=dev)
        self.k_pooled = torch.zeros((B, H, p.n_sub_max, d), dtype=dt, device=dev)
        self.se_pooled = torch.zeros((B, H, p.n_sub_max), dtype=torch.float32, device=dev)
        self.sq_blk = torch.full((B, H, p.max_blocks), float("-inf"), dtype=torch.float32, device=dev)
        self.se_blk = torch.full((B, H, p.max_blocks), float("-inf"), dtype=torch.float32, device=dev)
        self.sel_idx = torch.empty((B, H, p.k_blocks), dtype=torch.int32, device=dev)
        self.n_sel = torch.empty((B, H), dtype=torch.int32, device=dev)
        self.load_list = torch.empty((B, H, p.k_blocks, 2), dtype=torch.int32, device=dev)
        self.n_load = torch.empty((B, H), dtype=torch.int32, device=dev)
        self.out = torch.empty((B, p.n_q_heads, d), dtype=dt, device=dev)
        self.lse = torch.empty((B, p.n_q_heads), dtype=torch.float32, device=dev)
        self._packed = None
        self._graph = None
        self.keep_scores = True      # False: the single-entry step does not write sq_blk / se_blk (fused Stage 1 only)

    def rebuild_pooled(self) -> None:
        """Pooled keys and pooled importance of the whole cache (reads the host pool from the GPU)."""
        self.nosa.nosa_pool_blocks(self.host_k, self.host_bias, self.n_tokens, self.k_pooled, self.se_pooled)

    def set_residency(self, slot_of_block: torch.Tensor, block_of_slot: torch.Tensor) -> None:
        """Installs a residency map and copies the named blocks from the host pool into their slots."""
        dev = self.nosa.device
        self.slot_of_block.copy_(slot_of_block.to(dev))
        self.block_of_slot.copy_(block_of_slot.to(dev))
        bos = block_of_slot.cpu()
        B, H, C = bos.shape
        for b in range(B):
            for h in range(H):
                s = torch.nonzero(bos[b, h] >= 0).flatten()
                blk = bos[b, h, s].long()
                self.pool_k[b, h, s.to(dev)] = self.host_k[b, h, blk].to(dev)
                self.pool_v[b, h, s.to(dev)] = self.host_v[b, h, blk].to(dev)
                self.pool_bias[b, h, s.to(dev)] = self.host_bias[b, h, blk].to(dev)

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, b_new: torch.Tensor) -> None:
        """Appends the current token of every unit (cache update that precedes Stage 1 in Alg. 1)."""
        self.nosa.nosa_append(k_new, v_new, b_new, self.pool_k, self.pool_v, self.pool_bias, self.host_k, self.host_v,
                              self.host_bias, self.k_pooled, self.se_pooled, self.se_blk, self.n_tokens,
                              self.slot_of_block, self.block_of_slot)

    # the four calls of one decode step, in the order of Alg. 1
    def score(self, q: torch.Tensor) -> None:
        self.nosa.nosa_block_score(q, self.k_pooled, self.se_pooled, self.n_tokens, self.sq_blk, self.se_blk)

    def select(self) -> None:
        self.nosa.nosa_select(self.sq_blk, self.se_blk, self.n_tokens, self.sel_idx, self.n_sel,
                              self.slot_of_block, self.block_of_slot, self.load_list, self.n_load)

    def fetch(self) -> None:
        self.nosa.nosa_fetch(self.host_k, self.host_v, self.host_bias, self.pool_k, self.pool_v, self.pool_bias,
                             self.load_list, self.n_load)

    def decode(self, q: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        out = self.out if out is None else out
        self.nosa.nosa_sparse_decode(q, self.pool_k, self.pool_v, self.pool_bias, self.sel_idx, self.n_sel,
                                     self.slot_of_block, self.n_tokens, out, self.lse)
        return out

    def step(self, q: torch.Tensor) -> torch.Tensor:
        self.score(q)
        self.select()
        self.fetch()
        return self.decode(q)

    def _args(self, q: torch.Tensor):
        sq, se = (self.sq_blk, self.se_blk) if self.keep_scores else (None, None)
        return self.nosa.step_args(q, self.k_pooled, self.se_pooled, self.n_tokens, sq, se, self.sel_idx,
                                   self.n_sel, self.slot_of_block, self.block_of_slot, self.load_list, self.n_load,
                                   self.host_k, self.host_v, self.host_bias, self.pool_k, self.pool_v, self.pool_bias,
                                   self.out, self.lse)

    def step_fused(self, q: torch.Tensor) -> torch.Tensor:
        """The same step through the single entry point (pointers are packed once per query buffer)."""
        key = q.data_ptr()
        if self._packed is None or self._packed[0] != key:
            self._packed = (key, self._args(q))
        self.nosa.nosa_decode_step(self._packed[1])
        return self.out

    def capture(self, q_static: torch.Tensor) -> None:
        """Records the step into a HIP graph that reads its query from ``q_static`` (refreshed in place)."""
        self.release_graph()
        self._graph = self.nosa.nosa_graph_create(self._args(q_static))

    def capture_generation(self, qkv_static: torch.Tensor, w1: torch.Tensor, w2: torch.Tensor, mode: int,
                           q_out: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, b_new: torch.Tensor) -> None:
        """Records the whole step of a growing context -- split of the fused QKV activation with the eviction
        head, append of the token, then score / select / fetch / attention -- into one HIP graph that reads the
        activation from ``qkv_static`` (refreshed in place before every replay)."""
        self.release_graph()
        args = self._args(q_out)
        self.nosa.nosa_graph_begin()
        try:
            self.nosa.nosa_split_qkv_evict(qkv_static, w1, w2, mode, q_out, k_new, v_new, b_new)
            self.append(k_new, v_new, b_new)
            self.nosa.nosa_decode_step(args)
        finally:
            self._graph = self.nosa.nosa_graph_end()
        self._keep = (args, qkv_static, w1, w2, q_out, k_new, v_new, b_new)

    def replay(self) -> torch.Tensor:
        self.nosa.nosa_graph_launch(self._graph)
        return self.out

    def release_graph(self) -> None:
        if self._graph is not None:
            self.nosa.nosa_graph_destroy(self._graph)
            self._graph = None
