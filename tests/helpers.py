"""Shared test plumbing: dtype conversions and parameter construction.  No method arithmetic."""
from __future__ import annotations

import math

import numpy as np
import torch

import oracle
from nosa_inputs import Workload


def to_np(t: torch.Tensor) -> np.ndarray:
    """torch -> numpy on the host; bf16 travels as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def widen(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns or fp32 -> float64 (exact)."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def oracle_params(w: Workload, **over) -> oracle.Params:
    kw = dict(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
              n_sub_max=w.n_sub_max, dtype=0 if w.dtype == "fp32" else 1,
              softmax_scale=1.0 / math.sqrt(w.head_dim), block_size=w.block_size,
              pool_kernel=w.pool_kernel, pool_stride=w.pool_stride)
    kw.update(over)
    return oracle.Params(**kw)


def small_workload(**kw) -> Workload:
    base = dict(name="small", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, context=64 * 12,
                k_blocks=6, kq_blocks=2, sink_blocks=1, window_blocks=1, gpu_slots=6, dtype="fp32",
                layers=1, steps=4, structure="key_offset")
    base.update(kw)
    return Workload(**base)
