"""ctypes binding of the fp64 CPU oracle (oracle/nosa_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module, and
this module never imports the product package.

All arrays are numpy, C-contiguous, host memory.  bf16 tensors travel as ``uint16``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nosa_oracle.c")
_LIB = os.path.join(_HERE, "libnosa_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over units) into oracle/libnosa_oracle.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "block_size", "pool_kernel", "pool_stride",
        "k_blocks", "kq_blocks", "sink_blocks", "window_blocks", "gpu_slots", "max_blocks",
        "n_sub_max", "dtype", "victim_policy")] + [("softmax_scale", ctypes.c_double)]


@dataclass
class Params:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    k_blocks: int
    kq_blocks: int
    sink_blocks: int
    window_blocks: int
    gpu_slots: int
    max_blocks: int
    n_sub_max: int
    dtype: int                      # 0 fp32, 1 bf16
    softmax_scale: float
    block_size: int = 64
    pool_kernel: int = 64
    pool_stride: int = 64
    victim_policy: int = 0

    def c(self) -> _Params:
        return _Params(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.block_size,
                       self.pool_kernel, self.pool_stride, self.k_blocks, self.kq_blocks,
                       self.sink_blocks, self.window_blocks, self.gpu_slots, self.max_blocks,
                       self.n_sub_max, self.dtype, self.victim_policy, float(self.softmax_scale))

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == 0 else np.uint16


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_attention.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(ctypes.c_int(n))


def _ptr(a: Optional[np.ndarray], dtype=None):
    if a is None:
        return ctypes.c_void_p(0)
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"], "oracle needs C-contiguous numpy arrays"
    if dtype is not None:
        assert a.dtype == dtype, (a.dtype, dtype)
    return ctypes.c_void_p(a.ctypes.data)


def _check(a: np.ndarray, shape, dtype, name: str):
    assert a.shape == tuple(shape), f"{name}: shape {a.shape} != {tuple(shape)}"
    assert a.dtype == dtype, f"{name}: dtype {a.dtype} != {dtype}"


def pool(p: Params, keys: np.ndarray, bias: np.ndarray, n_tokens: np.ndarray):
    """Mean pooling of keys and of the importance score over sub-blocks (Sec. 3.1, mean-pooling Eq.)."""
    B, H, d, nb = p.batch, p.n_kv_heads, p.head_dim, p.block_size
    _check(keys, (B, H, p.max_blocks, nb, d), p.np_dtype, "keys")
    _check(bias, (B, H, p.max_blocks, nb), np.float32, "bias")
    _check(n_tokens, (B,), np.int32, "n_tokens")
    k_pooled = np.zeros((B, H, p.n_sub_max, d), dtype=p.np_dtype)
    se_pooled = np.zeros((B, H, p.n_sub_max), dtype=np.float32)
    pc = p.c()
    lib().oracle_pool(ctypes.byref(pc), _ptr(keys), _ptr(bias), _ptr(n_tokens), _ptr(k_pooled), _ptr(se_pooled))
    return k_pooled, se_pooled


def block_score(p: Params, q: np.ndarray, k_pooled: np.ndarray, se_pooled: np.ndarray, n_tokens: np.ndarray,
                per_head: bool = False):
    """Block-level query-aware and query-agnostic scores (Alg. 1, Stage 1 up to fused pooling)."""
    B, H = p.batch, p.n_kv_heads
    _check(q, (B, p.n_q_heads, p.head_dim), p.np_dtype, "q")
    _check(k_pooled, (B, H, p.n_sub_max, p.head_dim), p.np_dtype, "k_pooled")
    _check(se_pooled, (B, H, p.n_sub_max), np.float32, "se_pooled")
    _check(n_tokens, (B,), np.int32, "n_tokens")
    sq = np.empty((B, H, p.max_blocks), dtype=np.float64)
    se = np.empty((B, H, p.max_blocks), dtype=np.float64)
    head = np.zeros((B, p.n_q_heads, p.n_sub_max), dtype=np.float64) if per_head else None
    pc = p.c()
    lib().oracle_block_score(ctypes.byref(pc), _ptr(q), _ptr(k_pooled), _ptr(se_pooled), _ptr(n_tokens),
                             _ptr(sq), _ptr(se), _ptr(head))
    return (sq, se, head) if per_head else (sq, se)


def select(p: Params, sq_blk: np.ndarray, se_blk: np.ndarray, n_tokens: np.ndarray, with_kind: bool = False):
    """Constrained top-k block selection (selection Eq., Sec. 3.1)."""
    B, H = p.batch, p.n_kv_heads
    sq_blk = np.ascontiguousarray(sq_blk, dtype=np.float64)
    se_blk = np.ascontiguousarray(se_blk, dtype=np.float64)
    _check(sq_blk, (B, H, p.max_blocks), np.float64, "sq_blk")
    _check(se_blk, (B, H, p.max_blocks), np.float64, "se_blk")
    _check(n_tokens, (B,), np.int32, "n_tokens")
    if p.sink_blocks + p.window_blocks + p.kq_blocks > p.k_blocks or p.window_blocks < 1:
        raise ValueError("budget must satisfy Ns + Nw + Kq <= K and Nw >= 1")
    sel = np.empty((B, H, p.k_blocks), dtype=np.int32)
    n_sel = np.empty((B, H), dtype=np.int32)
    kind = np.empty((B, H, p.k_blocks), dtype=np.int32) if with_kind else None
    pc = p.c()
    lib().oracle_select(ctypes.byref(pc), _ptr(sq_blk), _ptr(se_blk), _ptr(n_tokens), _ptr(sel), _ptr(n_sel),
                        _ptr(kind))
    return (sel, n_sel, kind) if with_kind else (sel, n_sel)


def load(p: Params, sel_idx: np.ndarray, n_sel: np.ndarray, slot_of_block: np.ndarray, block_of_slot: np.ndarray,
         se_blk: Optional[np.ndarray] = None, n_tokens: Optional[np.ndarray] = None):
    """Set difference of the selection against the resident map; updates both maps in place.
    With ``p.victim_policy == 1`` the block-level importance ``se_blk`` ranks the victims."""
    if p.victim_policy == 1:
        B, H = p.batch, p.n_kv_heads
        se_blk = np.ascontiguousarray(se_blk, dtype=np.float64)
        _check(se_blk, (B, H, p.max_blocks), np.float64, "se_blk")
        _check(n_tokens, (B,), np.int32, "n_tokens")
        load_list = np.empty((B, H, p.k_blocks, 2), dtype=np.int32)
        n_load = np.empty((B, H), dtype=np.int32)
        pc = p.c()
        lib().oracle_load_policy(ctypes.byref(pc), _ptr(sel_idx), _ptr(n_sel), _ptr(se_blk), _ptr(n_tokens),
                                 _ptr(slot_of_block), _ptr(block_of_slot), _ptr(load_list), _ptr(n_load))
        return load_list, n_load
    B, H = p.batch, p.n_kv_heads
    _check(sel_idx, (B, H, p.k_blocks), np.int32, "sel_idx")
    _check(n_sel, (B, H), np.int32, "n_sel")
    _check(slot_of_block, (B, H, p.max_blocks), np.int32, "slot_of_block")
    _check(block_of_slot, (B, H, p.gpu_slots), np.int32, "block_of_slot")
    load_list = np.empty((B, H, p.k_blocks, 2), dtype=np.int32)
    n_load = np.empty((B, H), dtype=np.int32)
    pc = p.c()
    lib().oracle_load(ctypes.byref(pc), _ptr(sel_idx), _ptr(n_sel), _ptr(slot_of_block), _ptr(block_of_slot),
                      _ptr(load_list), _ptr(n_load))
    return load_list, n_load


def fetch(p: Params, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, load_list, n_load) -> None:
    """Copy the missed blocks from the host pool into their slots (in place on the pool arrays)."""
    B, H, d, nb = p.batch, p.n_kv_heads, p.head_dim, p.block_size
    _check(host_k, (B, H, p.max_blocks, nb, d), p.np_dtype, "host_k")
    _check(host_v, (B, H, p.max_blocks, nb, d), p.np_dtype, "host_v")
    _check(pool_k, (B, H, p.gpu_slots, nb, d), p.np_dtype, "pool_k")
    _check(pool_v, (B, H, p.gpu_slots, nb, d), p.np_dtype, "pool_v")
    if host_bias is not None:
        _check(host_bias, (B, H, p.max_blocks, nb), np.float32, "host_bias")
        _check(pool_bias, (B, H, p.gpu_slots, nb), np.float32, "pool_bias")
    _check(load_list, (B, H, p.k_blocks, 2), np.int32, "load_list")
    _check(n_load, (B, H), np.int32, "n_load")
    pc = p.c()
    lib().oracle_fetch(ctypes.byref(pc), _ptr(host_k), _ptr(host_v), _ptr(host_bias), _ptr(pool_k), _ptr(pool_v),
                       _ptr(pool_bias), _ptr(load_list), _ptr(n_load))


def attention(p: Params, q, pool_k, pool_v, pool_bias, sel_idx, n_sel, slot_of_block, n_tokens,
              with_probs: bool = False):
    """Biased softmax attention over the tokens of the selected blocks (Sec. 3.1, output Eq.)."""
    B, H, d, nb = p.batch, p.n_kv_heads, p.head_dim, p.block_size
    _check(q, (B, p.n_q_heads, d), p.np_dtype, "q")
    _check(pool_k, (B, H, p.gpu_slots, nb, d), p.np_dtype, "pool_k")
    _check(pool_v, (B, H, p.gpu_slots, nb, d), p.np_dtype, "pool_v")
    if pool_bias is not None:
        _check(pool_bias, (B, H, p.gpu_slots, nb), np.float32, "pool_bias")
    _check(sel_idx, (B, H, p.k_blocks), np.int32, "sel_idx")
    _check(n_sel, (B, H), np.int32, "n_sel")
    _check(slot_of_block, (B, H, p.max_blocks), np.int32, "slot_of_block")
    _check(n_tokens, (B,), np.int32, "n_tokens")
    out = np.zeros((B, p.n_q_heads, d), dtype=np.float64)
    lse = np.zeros((B, p.n_q_heads), dtype=np.float64)
    probs = np.zeros((B, p.n_q_heads, p.k_blocks * nb), dtype=np.float64) if with_probs else None
    pc = p.c()
    bad = lib().oracle_attention(ctypes.byref(pc), _ptr(q), _ptr(pool_k), _ptr(pool_v), _ptr(pool_bias),
                                 _ptr(sel_idx), _ptr(n_sel), _ptr(slot_of_block), _ptr(n_tokens), _ptr(out),
                                 _ptr(lse), _ptr(probs))
    if bad:
        raise RuntimeError(f"oracle_attention: {bad} selected blocks have no slot")
    return (out, lse, probs) if with_probs else (out, lse)


# ---- conveniences for callers that hold torch tensors / workload descriptions -------------------

def to_np(t) -> np.ndarray:
    """torch tensor -> numpy on the host; bf16 travels as uint16 bit patterns."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def params_from_workload(w, **over) -> Params:
    """Oracle parameters of a workload description (any object with the shape attributes)."""
    kw = dict(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
              n_sub_max=w.n_sub_max, dtype=0 if w.dtype == "fp32" else 1,
              softmax_scale=1.0 / float(w.head_dim) ** 0.5, block_size=w.block_size,
              pool_kernel=w.pool_kernel, pool_stride=w.pool_stride, victim_policy=getattr(w, "victim_policy", 0))
    kw.update(over)
    return Params(**kw)


def append(p: Params, k_new, v_new, b_new, pool_k, pool_v, pool_bias, host_k, host_v, host_bias, se_blk,
           n_tokens, slot_of_block, block_of_slot) -> None:
    """Append one token per unit to the cache (host pool, and the GPU slot of its block); in place."""
    B, H, d, nb = p.batch, p.n_kv_heads, p.head_dim, p.block_size
    _check(k_new, (B, H, d), p.np_dtype, "k_new")
    _check(v_new, (B, H, d), p.np_dtype, "v_new")
    _check(b_new, (B, H), np.float32, "b_new")
    _check(pool_k, (B, H, p.gpu_slots, nb, d), p.np_dtype, "pool_k")
    _check(pool_v, (B, H, p.gpu_slots, nb, d), p.np_dtype, "pool_v")
    _check(pool_bias, (B, H, p.gpu_slots, nb), np.float32, "pool_bias")
    _check(host_k, (B, H, p.max_blocks, nb, d), p.np_dtype, "host_k")
    _check(host_v, (B, H, p.max_blocks, nb, d), p.np_dtype, "host_v")
    _check(host_bias, (B, H, p.max_blocks, nb), np.float32, "host_bias")
    se_blk = np.ascontiguousarray(se_blk, dtype=np.float64)
    _check(se_blk, (B, H, p.max_blocks), np.float64, "se_blk")
    _check(n_tokens, (B,), np.int32, "n_tokens")
    _check(slot_of_block, (B, H, p.max_blocks), np.int32, "slot_of_block")
    _check(block_of_slot, (B, H, p.gpu_slots), np.int32, "block_of_slot")
    pc = p.c()
    lib().oracle_append(ctypes.byref(pc), _ptr(k_new), _ptr(v_new), _ptr(b_new), _ptr(pool_k), _ptr(pool_v),
                        _ptr(pool_bias), _ptr(host_k), _ptr(host_v), _ptr(host_bias), _ptr(se_blk), _ptr(n_tokens),
                        _ptr(slot_of_block), _ptr(block_of_slot))


def split_qkv_evict(p: Params, qkv: np.ndarray, w1: np.ndarray, w2: np.ndarray, mode: int = 0):
    """Split of the fused QKV activation and the eviction head b = softplus(v W1) (.) W2 (Sec. 3.1)."""
    B, Hq, H, d = p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim
    _check(qkv, (B, (Hq + 2 * H) * d), p.np_dtype, "qkv")
    _check(w1, (d, H), np.float32, "w1")
    _check(w2, (H,), np.float32, "w2")
    q = np.empty((B, Hq, d), p.np_dtype)
    k = np.empty((B, H, d), p.np_dtype)
    v = np.empty((B, H, d), p.np_dtype)
    b = np.empty((B, H), np.float64)
    pc = p.c()
    lib().oracle_split_qkv_evict(ctypes.byref(pc), _ptr(qkv), _ptr(w1), _ptr(w2), ctypes.c_int(mode), _ptr(q), _ptr(k),
                                 _ptr(v), _ptr(b))
    return q, k, v, b


def fetch_tokens(p: Params, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, token_list, n_list) -> None:
    """Element-wise (token-granular) host-to-pool copies; in place on the pool arrays."""
    B, H = p.batch, p.n_kv_heads
    M = token_list.shape[2]
    _check(token_list, (B, H, M, 2), np.int32, "token_list")
    _check(n_list, (B, H), np.int32, "n_list")
    pc = p.c()
    lib().oracle_fetch_tokens(ctypes.byref(pc), _ptr(host_k), _ptr(host_v), _ptr(host_bias), _ptr(pool_k), _ptr(pool_v),
                              _ptr(pool_bias), _ptr(token_list), _ptr(n_list), ctypes.c_int(M))


def prefill(p: Params, q_chunk: np.ndarray, cache_k, cache_v, cache_bias, k_pooled, se_pooled, p0: int,
            positions=None):
    """Sparse prefill of a chunk of query tokens (NOSA with sparse prefill: the mask Eq. of Sec. 2.1 with the
    selection Eq. of Sec. 3.1 evaluated at every query position).

    q_chunk [B, Lq, Hq, d] holds the queries of positions p0 .. p0+Lq-1; the cache tensors (contiguous
    block layout [B,Hkv,Nmax,nb,d], bias [B,Hkv,Nmax,nb]) already hold the keys / values / biases of all
    positions < p0 + Lq.  Position p0 + t sees T = p0 + t + 1 tokens: its output is, by definition, the
    decode step's output on a cache of those T tokens -- so this function is a plain loop over positions
    calling block_score, select and attention, with every block resident (slot = block index).
    Returns sel [B,Hkv,Lq,K], n_sel [B,Hkv,Lq], out [B,Lq,Hq,d] fp64, lse [B,Lq,Hq].  ``positions`` (chunk
    offsets t) limits the loop to a sample; the rows of the other positions are left at -1 / NaN.
    """
    B, H, d = p.batch, p.n_kv_heads, p.head_dim
    Lq = q_chunk.shape[1]
    _check(q_chunk, (B, Lq, p.n_q_heads, d), p.np_dtype, "q_chunk")
    assert p.gpu_slots == p.max_blocks, "prefill runs on a fully resident cache: gpu_slots must equal max_blocks"
    ident = np.tile(np.arange(p.max_blocks, dtype=np.int32), (B, H, 1))
    sel_all = np.full((B, H, Lq, p.k_blocks), -1, np.int32)
    nsel_all = np.full((B, H, Lq), -1, np.int32)
    out_all = np.full((B, Lq, p.n_q_heads, d), np.nan, np.float64)
    lse_all = np.full((B, Lq, p.n_q_heads), np.nan, np.float64)
    for t in (range(Lq) if positions is None else positions):
        n_tok = np.full((B,), p0 + t + 1, np.int32)
        q = np.ascontiguousarray(q_chunk[:, t])
        sq, se = block_score(p, q, k_pooled, se_pooled, n_tok)
        sel, n_sel = select(p, sq, se, n_tok)
        out, lse = attention(p, q, cache_k, cache_v, cache_bias, sel, n_sel, ident, n_tok)
        sel_all[:, :, t], nsel_all[:, :, t], out_all[:, t], lse_all[:, t] = sel, n_sel, out, lse
    return sel_all, nsel_all, out_all, lse_all
