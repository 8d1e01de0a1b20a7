"""Seeded synthetic inputs for the NOSA decode-step path.

This module only draws random tensors with the shapes and structure of the
five benchmark workloads.  It holds none of the method's arithmetic (no
pooling, scoring, selection or attention): the CPU oracle and the HIP path
both consume the bytes produced here, and neither is imported from here.

Every draw is keyed by a tuple (seed, tensor id, layer, step, retry) that is
mixed into a 63-bit seed for a fresh ``torch.Generator``, so any tensor can be
regenerated independently of the order in which others were drawn.  Bulk
tensors may be drawn directly on the GPU (``device="cuda"``); a CPU draw and a
GPU draw of the same key differ, which is fine: both sides of a parity test
always read the same bytes.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch

# tensor ids used in RNG keys
_T_K, _T_V, _T_BIAS, _T_DIR, _T_MU, _T_PLANT, _T_Q, _T_PERM, _T_BETA, _T_APPEND, _T_QM = range(11)

_MASK64 = (1 << 64) - 1


def _mix(*key: int) -> int:
    """splitmix64-style mixing of an integer key tuple into a 63-bit seed."""
    h = 0x9E3779B97F4A7C15
    for v in key:
        h = (h ^ (int(v) & _MASK64)) & _MASK64
        h = (h * 0xBF58476D1CE4E5B9) & _MASK64
        h ^= h >> 31
        h = (h * 0x94D049BB133111EB) & _MASK64
        h ^= h >> 29
    return h & ((1 << 63) - 1)


def _gen(device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_mix(*key))
    return g


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and structure of one benchmark configuration.

    Block counts follow the paper's default split of the budget
    (App. B.2, "Hyperparameters of each method"): K = Ns + Nw + Kq + Ke.
    """
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int                 # tokens in the cache at step 0
    k_blocks: int                # K
    kq_blocks: int               # Kq  (= fetch budget per step)
    sink_blocks: int             # Ns
    window_blocks: int           # Nw
    gpu_slots: int               # C
    dtype: str                   # "fp32" | "bf16"
    layers: int
    steps: int
    structure: str               # planted | key_offset | ar1 | heavy | drift
    block_size: int = 64
    pool_kernel: int = 64
    pool_stride: int = 64
    generated: int = 0           # tokens appended during the run (growing context)
    victim_policy: int = 0       # residency policy passed through to both sides (no arithmetic here)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_tokens(self) -> int:
        return self.context + self.generated

    @property
    def max_blocks(self) -> int:
        return (self.max_tokens + self.block_size - 1) // self.block_size

    @property
    def n_sub_max(self) -> int:
        if self.max_tokens < self.pool_kernel:
            return 0
        return (self.max_tokens - self.pool_kernel) // self.pool_stride + 1

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Workload] = {
    # batch 1, GQA group 4, d64, 2048 tokens, fp32, <=2 newly fetched blocks per step
    "tiny": Workload("tiny", 1, 4, 1, 64, 2048, 8, 2, 1, 1, 8, "fp32", 1, 16, "planted"),
    # 50 % of the 128 blocks resident on the GPU (C = 64)
    "1b": Workload("1b", 16, 16, 2, 64, 8192, 32, 8, 1, 8, 64, "bf16", 1, 64, "key_offset"),
    "3b": Workload("3b", 32, 24, 4, 128, 16384, 64, 8, 1, 16, 64, "bf16", 28, 128, "ar1"),
    "8b": Workload("8b", 64, 32, 8, 128, 32768, 64, 8, 1, 16, 64, "bf16", 32, 256, "heavy"),
    "longgen": Workload("longgen", 32, 32, 8, 128, 4096, 64, 8, 1, 16, 64, "bf16", 1, 16384,
                        "drift", generated=16384),
}


def _randn(shape, device, dtype, *key) -> torch.Tensor:
    return torch.randn(shape, generator=_gen(device, *key), device=device, dtype=torch.float32).to(dtype)


def unit_directions(w: Workload, seed: int, layer: int, device="cpu") -> torch.Tensor:
    """One unit-norm direction per (batch, KV head): [B, Hkv, d] fp32."""
    u = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=_gen(device, seed, _T_DIR, layer),
                    device=device, dtype=torch.float32)
    return u / u.norm(dim=-1, keepdim=True)


def planted_blocks(w: Workload, seed: int, layer: int, n_blocks: Optional[int] = None) -> torch.Tensor:
    """Indices of the planted (high-similarity / heavy-hitter) blocks per unit: [B, Hkv, P] int64.

    Planted blocks are drawn from the blocks that are neither sink nor window
    blocks at the initial context, so that they are ordinary candidates.
    """
    n = w.context // w.block_size if n_blocks is None else n_blocks
    lo, hi = w.sink_blocks, max(w.sink_blocks, n - w.window_blocks)
    if w.structure == "planted":
        p = 3
    elif w.structure == "heavy":
        p = max(1, round(0.05 * n))
    else:
        p = 0
    p = min(p, hi - lo)
    g = _gen("cpu", seed, _T_PLANT, layer)
    out = torch.empty((w.batch, w.n_kv_heads, p), dtype=torch.int64)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            out[b, h] = torch.randperm(hi - lo, generator=g)[:p] + lo
    return out


def make_layer(w: Workload, seed: int, layer: int, device="cpu", n_blocks: Optional[int] = None) -> dict:
    """Draw the whole (host-side) KV cache of one layer.

    Returns ``host_k``/``host_v`` [B, Hkv, Nmax, nb, d] in the workload dtype and
    ``host_bias`` [B, Hkv, Nmax, nb] fp32.  Blocks beyond the initial context are
    zero (they are filled by appends in the growing-context workload).
    The per-token bias is ``beta_J + 0.1 * eps`` with block levels ``beta_J`` a
    random permutation of ``linspace(-2, 2, N)``: every block has a distinct
    level, so block-level importance scores are well separated.
    """
    nb, d = w.block_size, w.head_dim
    n_init = w.context // nb if n_blocks is None else n_blocks
    tail = w.context - n_init * nb if n_blocks is None else 0
    n_fill = n_init + (1 if tail else 0)
    nmax = max(w.max_blocks, n_fill)
    B, H = w.batch, w.n_kv_heads
    dt = w.torch_dtype

    k = torch.zeros((B, H, nmax, nb, d), device=device, dtype=dt)
    v = torch.zeros((B, H, nmax, nb, d), device=device, dtype=dt)
    bias = torch.zeros((B, H, nmax, nb), device=device, dtype=torch.float32)

    # draw per batch element to bound the fp32 temporaries
    u = unit_directions(w, seed, layer, device)
    plant = planted_blocks(w, seed, layer, n_init).to(device)
    mu = None
    if w.structure == "key_offset":
        mu = 0.5 * torch.randn((H, d), generator=_gen(device, seed, _T_MU, layer), device=device,
                               dtype=torch.float32)
    plant_gain = {"planted": 3.0, "heavy": 2.0}.get(w.structure, 0.0)
    for b in range(B):
        kb = torch.randn((H, n_fill, nb, d), generator=_gen(device, seed, _T_K, layer, b), device=device,
                         dtype=torch.float32)
        if mu is not None:
            kb += mu[:, None, None, :]
        if plant.shape[-1]:
            for h in range(H):
                kb[h, plant[b, h]] += plant_gain * u[b, h]
        k[b, :, :n_fill] = kb.to(dt)
        del kb
        v[b, :, :n_fill] = torch.randn((H, n_fill, nb, d), generator=_gen(device, seed, _T_V, layer, b),
                                       device=device, dtype=torch.float32).to(dt)
        gb = _gen("cpu", seed, _T_BETA, layer, b)
        levels = torch.linspace(-2.0, 2.0, n_fill)
        beta = torch.stack([levels[torch.randperm(n_fill, generator=gb)] for _ in range(H)]).to(device)
        eps = torch.randn((H, n_fill, nb), generator=_gen(device, seed, _T_BIAS, layer, b), device=device,
                          dtype=torch.float32)
        bias[b, :, :n_fill] = beta[:, :, None] + 0.1 * eps
    if tail:
        k[:, :, n_init, tail:] = 0
        v[:, :, n_init, tail:] = 0
        bias[:, :, n_init, tail:] = 0
    return {"host_k": k, "host_v": v, "host_bias": bias, "directions": u, "planted": plant}


class QueryStream:
    """Per-step decode queries [B, Hq, d] in the workload dtype.

    ``planted`` / ``heavy``: q = a * u_unit + noise, redrawn i.i.d. every step
    (a = 3), so the query-aware picks concentrate on the planted blocks.
    ``key_offset``: i.i.d. N(0, 1).
    ``ar1``:   q_t = 0.9 q_{t-1} + sqrt(1 - 0.81) eps_t  (slowly moving picks).
    ``drift``: q_t = m_t + x_t, x_t AR(1) rho = 0.9, m_t AR(1) rho = 0.999.

    ``draw(step, retry)`` proposes the queries of ``step`` from the committed
    state of step - 1; ``commit(q32)`` fixes them.  A harness that needs a
    selection margin may redraw single units with ``retry + 1`` before
    committing; the stream itself never looks at scores.
    """

    def __init__(self, w: Workload, seed: int, layer: int, device="cpu"):
        self.w, self.seed, self.layer, self.device = w, seed, layer, device
        self.u = unit_directions(w, seed, layer, device)           # [B,Hkv,d]
        self.x = None        # AR(1) fast state, fp32 [B,Hq,d]
        self.m = None        # AR(1) slow state (drift only)

    def _noise(self, tid, step, retry):
        w = self.w
        return torch.randn((w.batch, w.n_q_heads, w.head_dim),
                           generator=_gen(self.device, self.seed, tid, self.layer, step, retry),
                           device=self.device, dtype=torch.float32)

    def draw(self, step: int, retry: int = 0) -> dict:
        w = self.w
        eps = self._noise(_T_Q, step, retry)
        if w.structure in ("planted", "heavy"):
            u = self.u.repeat_interleave(w.group, dim=1)           # [B,Hq,d]
            return {"q32": 3.0 * u + eps, "x": None, "m": None}
        if w.structure == "key_offset":
            return {"q32": eps, "x": None, "m": None}
        if w.structure == "ar1":
            x = eps if self.x is None else 0.9 * self.x + math.sqrt(1 - 0.81) * eps
            return {"q32": x, "x": x, "m": None}
        if w.structure == "drift":
            em = self._noise(_T_QM, step, retry)
            x = eps if self.x is None else 0.9 * self.x + math.sqrt(1 - 0.81) * eps
            m = em if self.m is None else 0.999 * self.m + math.sqrt(1 - 0.999 ** 2) * em
            return {"q32": m + x, "x": x, "m": m}
        raise ValueError(w.structure)

    def commit(self, drawn: dict) -> torch.Tensor:
        self.x, self.m = drawn["x"], drawn["m"]
        return drawn["q32"].to(self.w.torch_dtype)

    def next(self, step: int) -> torch.Tensor:
        return self.commit(self.draw(step))


def chunk_queries(w: Workload, seed: int, layer: int, lq: int, retry: int = 0, device="cpu") -> torch.Tensor:
    """Queries of a prefill chunk, fp32 [B, lq, Hq, d]: q_t = 3 u + x_t with x_t AR(1) along the positions
    (rho = 0.9), u the unit direction of the KV head -- neighbouring positions look for similar blocks, as
    neighbouring tokens of a text do.  ``retry`` gives an independent draw of the same law.
    """
    u = unit_directions(w, seed, layer, device).repeat_interleave(w.group, dim=1)      # [B,Hq,d]
    eps = torch.randn((lq, w.batch, w.n_q_heads, w.head_dim), generator=_gen(device, seed, _T_Q, layer, 1 << 20, retry),
                      device=device, dtype=torch.float32)
    x = torch.empty_like(eps)
    x[0] = eps[0]
    c = math.sqrt(1 - 0.81)
    for t in range(1, lq):
        x[t] = 0.9 * x[t - 1] + c * eps[t]
    return (3.0 * u.unsqueeze(0) + x).permute(1, 0, 2, 3).contiguous()


def append_token(w: Workload, seed: int, layer: int, step: int, device="cpu") -> dict:
    """Key, value and bias of the token appended at ``step`` (growing-context workload).

    k_new, v_new: [B, Hkv, d] workload dtype; b_new: [B, Hkv] fp32.  Same law as the
    prompt (N(0,1) keys/values); the bias level of the block a token falls in is
    drawn per block so that a finished block again has its own level.
    """
    B, H, d = w.batch, w.n_kv_heads, w.head_dim
    g = _gen(device, seed, _T_APPEND, layer, step)
    k = torch.randn((B, H, d), generator=g, device=device, dtype=torch.float32).to(w.torch_dtype)
    v = torch.randn((B, H, d), generator=g, device=device, dtype=torch.float32).to(w.torch_dtype)
    blk = (w.context + step) // w.block_size
    level = 4.0 * torch.rand((B, H), generator=_gen(device, seed, _T_BETA, layer, 1 << 20, blk), device=device) - 2.0
    b = level + 0.1 * torch.randn((B, H), generator=g, device=device, dtype=torch.float32)
    return {"k_new": k, "v_new": v, "b_new": b}


def random_residency(w: Workload, seed: int, layer: int, n_blocks: int, fill: Optional[int] = None):
    """A seeded initial residency: ``fill`` (default C) distinct blocks placed in slots 0..fill-1.

    Returns (slot_of_block [B,Hkv,Nmax] int32, block_of_slot [B,Hkv,C] int32), -1 = none.
    Pure bookkeeping; the caller copies the block bytes into the pool slots.
    """
    B, H, C = w.batch, w.n_kv_heads, w.gpu_slots
    nmax = max(w.max_blocks, n_blocks)
    fill = min(C if fill is None else fill, n_blocks)
    sob = torch.full((B, H, nmax), -1, dtype=torch.int32)
    bos = torch.full((B, H, C), -1, dtype=torch.int32)
    g = _gen("cpu", seed, _T_PERM, layer)
    for b in range(B):
        for h in range(H):
            blocks = torch.randperm(n_blocks, generator=g)[:fill].to(torch.int32)
            bos[b, h, :fill] = blocks
            sob[b, h, blocks.long()] = torch.arange(fill, dtype=torch.int32)
    return sob, bos
