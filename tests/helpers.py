"""Shared test plumbing: dtype conversions and parameter construction.  No method arithmetic."""
from __future__ import annotations

import math

import numpy as np
import torch

import oracle
from nosa_inputs import Workload


to_np = oracle.to_np


def widen(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns or fp32 -> float64 (exact)."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


oracle_params = oracle.params_from_workload


def small_workload(**kw) -> Workload:
    base = dict(name="small", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, context=64 * 12,
                k_blocks=6, kq_blocks=2, sink_blocks=1, window_blocks=1, gpu_slots=6, dtype="fp32",
                layers=1, steps=4, structure="key_offset")
    base.update(kw)
    return Workload(**base)


def gpu_params(w: Workload, **over):
    """nosa_params of a workload for the HIP library."""
    import paper_2510_13602_amd as nosa
    kw = dict(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
              n_sub_max=w.n_sub_max, dtype=w.dtype, softmax_scale=1.0 / math.sqrt(w.head_dim),
              block_size=w.block_size, pool_kernel=w.pool_kernel, pool_stride=w.pool_stride,
              victim_policy=w.victim_policy)
    kw.update(over)
    return nosa.make_params(**kw)


def from_np(a: np.ndarray, like_dtype: torch.dtype, device="cuda") -> torch.Tensor:
    """numpy (uint16 bit patterns for bf16) -> torch tensor on ``device``."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(a.copy()).to(device=device, dtype=like_dtype)


def out_tol(dtype: str) -> float:
    """Attention parity bar: max-abs error 1e-5 for fp32 (fp32 accumulation), 1e-2 for bf16."""
    return 1e-5 if dtype == "fp32" else 1e-2


def round_to_dtype(x64: np.ndarray, dtype: str) -> np.ndarray:
    """The oracle's fp64 output rounded to the output dtype, for the error measure only."""
    t = torch.from_numpy(x64)
    return t.to(torch.float32 if dtype == "fp32" else torch.bfloat16).double().numpy()
