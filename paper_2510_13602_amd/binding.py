"""Thin ctypes binding of libnosa.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/nosa.h;
PyTorch tensors are used here for device / pinned memory and for the stream handle, nothing else.
There is no CPU fallback: if the library is missing or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnosa.so")

NOSA_OK, NOSA_EINVAL, NOSA_ESHAPE, NOSA_EHIP = 0, -1, -2, -3
DTYPE_F32, DTYPE_BF16 = 0, 1
(KERNEL_SCORE, KERNEL_SELECT, KERNEL_FETCH, KERNEL_DECODE, KERNEL_COMBINE, KERNEL_EVICT, KERNEL_APPEND,
 KERNEL_PREFILL) = range(8)
KERNEL_NAMES = ["block_score", "select", "fetch", "sparse_decode", "combine", "split_qkv_evict", "append", "prefill_attend"]
MAX_SPLITS = 16
STATIC_SCRATCH_BYTES = 8 << 20

EXPORTS = [
    "nosa_validate_params", "nosa_create", "nosa_destroy", "nosa_workspace_bytes", "nosa_set_workspace",
    "nosa_set_splits", "nosa_get_splits", "nosa_set_merge_in_kernel", "nosa_set_attention_kernel", "nosa_set_overlap", "nosa_set_fetch_workgroups", "nosa_last_error", "nosa_block_score",
    "nosa_select", "nosa_fetch", "nosa_sparse_decode", "nosa_sparse_decode_static", "nosa_pool_blocks", "nosa_append", "nosa_split_qkv_evict", "nosa_fetch_tokens", "nosa_decode_step", "nosa_set_fused_select", "nosa_graph_create", "nosa_graph_begin", "nosa_graph_end", "nosa_graph_launch",
    "nosa_graph_destroy", "nosa_prefill_select", "nosa_prefill_attend", "nosa_timing_enable",
    "nosa_timing_read", "nosa_set_trace",
]


class NosaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libnosa error {code}: {msg}")
        self.code = code


class Params(ctypes.Structure):
    """Mirror of ``nosa_params`` (include/nosa.h)."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "block_size", "pool_kernel", "pool_stride",
        "k_blocks", "kq_blocks", "sink_blocks", "window_blocks", "gpu_slots", "max_blocks", "n_sub_max",
        "dtype", "victim_policy")] + [("softmax_scale", ctypes.c_float)]


class StepArgs(ctypes.Structure):
    """Mirror of ``nosa_step_args`` (include/nosa.h): the tensors of one whole decode step."""
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "q", "k_pooled", "se_pooled", "n_tokens", "sq_blk", "se_blk", "sel_idx", "n_sel", "slot_of_block",
        "block_of_slot", "load_list", "n_load", "host_k", "host_v", "host_bias", "pool_k", "pool_v", "pool_bias",
        "out", "lse")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree libnosa.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback for the NOSA hot path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    lib.nosa_validate_params.argtypes = [ctypes.POINTER(Params), ctypes.c_char_p, ctypes.c_size_t]
    lib.nosa_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(Params), vp]
    lib.nosa_destroy.argtypes = [vp]
    lib.nosa_workspace_bytes.argtypes = [ctypes.POINTER(Params)]
    lib.nosa_workspace_bytes.restype = ctypes.c_size_t
    lib.nosa_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.nosa_set_splits.argtypes = [vp, ctypes.c_int]
    lib.nosa_get_splits.argtypes = [vp]
    lib.nosa_set_merge_in_kernel.argtypes = [vp, ctypes.c_int]
    lib.nosa_set_attention_kernel.argtypes = [vp, ctypes.c_int]
    lib.nosa_set_overlap.argtypes = [vp, ctypes.c_int]
    lib.nosa_set_fetch_workgroups.argtypes = [vp, ctypes.c_int]
    lib.nosa_set_fused_select.argtypes = [vp, ctypes.c_int]
    lib.nosa_last_error.argtypes = [vp]
    lib.nosa_last_error.restype = ctypes.c_char_p
    lib.nosa_block_score.argtypes = [vp, vp, vp, fp, i32p, fp, fp]
    lib.nosa_select.argtypes = [vp, fp, fp, i32p, i32p, i32p, i32p, i32p, i32p, i32p]
    lib.nosa_fetch.argtypes = [vp, vp, vp, fp, vp, vp, fp, i32p, i32p]
    lib.nosa_sparse_decode.argtypes = [vp, vp, vp, vp, fp, i32p, i32p, i32p, i32p, vp, fp]
    lib.nosa_sparse_decode_static.argtypes = lib.nosa_sparse_decode.argtypes
    lib.nosa_pool_blocks.argtypes = [vp, vp, fp, i32p, vp, fp]
    lib.nosa_append.argtypes = [vp] + [vp] * 15
    lib.nosa_split_qkv_evict.argtypes = [vp, vp, fp, fp, ctypes.c_int, vp, vp, vp, fp]
    lib.nosa_fetch_tokens.argtypes = [vp, vp, vp, fp, vp, vp, fp, i32p, i32p, ctypes.c_int32]
    lib.nosa_decode_step.argtypes = [vp, ctypes.POINTER(StepArgs)]
    lib.nosa_graph_create.argtypes = [vp, ctypes.POINTER(StepArgs), ctypes.POINTER(vp)]
    lib.nosa_graph_begin.argtypes = [vp]
    lib.nosa_graph_end.argtypes = [vp, ctypes.POINTER(vp)]
    lib.nosa_graph_launch.argtypes = [vp, vp]
    lib.nosa_graph_destroy.argtypes = [vp]
    lib.nosa_timing_enable.argtypes = [vp, ctypes.c_int]
    lib.nosa_set_trace.argtypes = [vp, vp, ctypes.c_int32]
    lib.nosa_timing_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    for name in EXPORTS:
        if name not in ("nosa_workspace_bytes", "nosa_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def make_params(*, batch, n_q_heads, n_kv_heads, head_dim, k_blocks, kq_blocks, sink_blocks, window_blocks,
                gpu_slots, max_blocks, n_sub_max, dtype, softmax_scale=0.0, block_size=64, pool_kernel=64,
                pool_stride=64, victim_policy=0) -> Params:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: DTYPE_F32, torch.bfloat16: DTYPE_BF16}[dtype]
    elif isinstance(dtype, str):
        dtype = {"fp32": DTYPE_F32, "bf16": DTYPE_BF16}[dtype]
    return Params(batch, n_q_heads, n_kv_heads, head_dim, block_size, pool_kernel, pool_stride, k_blocks,
                  kq_blocks, sink_blocks, window_blocks, gpu_slots, max_blocks, n_sub_max, dtype, victim_policy,
                  float(softmax_scale))


def validate_params(p: Params) -> None:
    buf = ctypes.create_string_buffer(256)
    rc = load_library().nosa_validate_params(ctypes.byref(p), buf, 256)
    if rc != NOSA_OK:
        raise NosaError(rc, buf.value.decode())


def _dev(t: Optional[torch.Tensor], dtype, shape, name: str):
    """Device tensor -> raw pointer, after checking dtype / shape / contiguity."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    return _raw(t, dtype, shape, name)


def _raw(t: torch.Tensor, dtype, shape, name: str):
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


class Nosa:
    """One context = one layer shape (see ``nosa_create``).  Methods mirror the C entry points."""

    def __init__(self, params: Params, stream: Optional[torch.cuda.Stream] = None, device="cuda:0", workspace: bool = True):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise NosaError(NOSA_EHIP, "no GPU: the NOSA hot path has no CPU fallback")
        self.p = params
        self.device = torch.device(device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._ctx = ctypes.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.lib.nosa_create(ctypes.byref(self._ctx), ctypes.byref(params), ctypes.c_void_p(self.stream.cuda_stream))
        if rc != NOSA_OK:
            raise NosaError(rc, self.lib.nosa_last_error(None).decode())
        self.workspace = None
        if workspace:
            nbytes = self.lib.nosa_workspace_bytes(ctypes.byref(params))
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._check(self.lib.nosa_set_workspace(self._ctx, ctypes.c_void_p(self.workspace.data_ptr()), nbytes))
        self.tdtype = torch.float32 if params.dtype == DTYPE_F32 else torch.bfloat16

    # -- plumbing ------------------------------------------------------------------------------
    def _check(self, rc: int) -> None:
        if rc != NOSA_OK:
            raise NosaError(rc, self.lib.nosa_last_error(self._ctx).decode())

    def close(self) -> None:
        if self._ctx:
            self.lib.nosa_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def splits(self) -> int:
        return self.lib.nosa_get_splits(self._ctx)

    def set_splits(self, s: int) -> None:
        self._check(self.lib.nosa_set_splits(self._ctx, s))

    def set_attention_kernel(self, which: int) -> None:
        """0 chosen from the shape, 1 vector-ALU kernel, 2 matrix-core kernel."""
        self._check(self.lib.nosa_set_attention_kernel(self._ctx, int(which)))

    def set_merge_in_kernel(self, on: bool) -> None:
        self._check(self.lib.nosa_set_merge_in_kernel(self._ctx, 1 if on else 0))

    def set_overlap(self, on: bool) -> None:
        self._check(self.lib.nosa_set_overlap(self._ctx, 1 if on else 0))

    def set_fused_select(self, on: bool) -> None:
        self._check(self.lib.nosa_set_fused_select(self._ctx, 1 if on else 0))

    def set_fetch_workgroups(self, n: int) -> None:
        self._check(self.lib.nosa_set_fetch_workgroups(self._ctx, n))

    def set_trace(self, buf: Optional[torch.Tensor]) -> None:
        """``buf``: int64 device tensor [workgroups, 4] (or None to switch the trace off)."""
        if buf is None:
            self._check(self.lib.nosa_set_trace(self._ctx, None, 0))
        else:
            if not (buf.is_cuda and buf.dtype == torch.int64 and buf.is_contiguous() and buf.dim() == 2 and buf.shape[1] == 4):
                raise ValueError("trace buffer must be a contiguous int64 device tensor [workgroups, 4]")
            self._check(self.lib.nosa_set_trace(self._ctx, ctypes.c_void_p(buf.data_ptr()), buf.shape[0]))

    def timing_enable(self, on: bool) -> None:
        self._check(self.lib.nosa_timing_enable(self._ctx, 1 if on else 0))

    def timing_read(self, kernel: int):
        ms, n = ctypes.c_double(), ctypes.c_int32()
        self._check(self.lib.nosa_timing_read(self._ctx, kernel, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    # -- shapes --------------------------------------------------------------------------------
    @property
    def _B(self): return self.p.batch
    @property
    def _H(self): return self.p.n_kv_heads

    # -- the calls -----------------------------------------------------------------------------
    def nosa_block_score(self, q, k_pooled, se_pooled, n_tokens, sq_blk, se_blk) -> None:
        p, B, H = self.p, self._B, self._H
        self._check(self.lib.nosa_block_score(
            self._ctx, _dev(q, self.tdtype, (B, p.n_q_heads, p.head_dim), "q"),
            _dev(k_pooled, self.tdtype, (B, H, p.n_sub_max, p.head_dim), "k_pooled"),
            _dev(se_pooled, torch.float32, (B, H, p.n_sub_max), "se_pooled"),
            _dev(n_tokens, torch.int32, (B,), "n_tokens"),
            _dev(sq_blk, torch.float32, (B, H, p.max_blocks), "sq_blk"),
            _dev(se_blk, torch.float32, (B, H, p.max_blocks), "se_blk")))

    def nosa_select(self, sq_blk, se_blk, n_tokens, sel_idx, n_sel, slot_of_block, block_of_slot, load_list, n_load) -> None:
        p, B, H = self.p, self._B, self._H
        self._check(self.lib.nosa_select(
            self._ctx, _dev(sq_blk, torch.float32, (B, H, p.max_blocks), "sq_blk"),
            _dev(se_blk, torch.float32, (B, H, p.max_blocks), "se_blk"),
            _dev(n_tokens, torch.int32, (B,), "n_tokens"),
            _dev(sel_idx, torch.int32, (B, H, p.k_blocks), "sel_idx"),
            _dev(n_sel, torch.int32, (B, H), "n_sel"),
            _dev(slot_of_block, torch.int32, (B, H, p.max_blocks), "slot_of_block"),
            _dev(block_of_slot, torch.int32, (B, H, p.gpu_slots), "block_of_slot"),
            _dev(load_list, torch.int32, (B, H, p.k_blocks, 2), "load_list"),
            _dev(n_load, torch.int32, (B, H), "n_load")))

    def nosa_fetch(self, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, load_list, n_load) -> None:
        p, B, H = self.p, self._B, self._H
        kv_host = (B, H, p.max_blocks, p.block_size, p.head_dim)
        kv_pool = (B, H, p.gpu_slots, p.block_size, p.head_dim)
        for t, name in ((host_k, "host_k"), (host_v, "host_v"), (host_bias, "host_bias")):
            if t is not None and not (t.is_cuda or t.is_pinned()):
                raise ValueError(f"{name} must be pinned host memory (or device memory)")
        self._check(self.lib.nosa_fetch(
            self._ctx, _raw(host_k, self.tdtype, kv_host, "host_k"), _raw(host_v, self.tdtype, kv_host, "host_v"),
            None if host_bias is None else _raw(host_bias, torch.float32, kv_host[:4], "host_bias"),
            _dev(pool_k, self.tdtype, kv_pool, "pool_k"), _dev(pool_v, self.tdtype, kv_pool, "pool_v"),
            _dev(pool_bias, torch.float32, kv_pool[:4], "pool_bias"),
            _dev(load_list, torch.int32, (B, H, p.k_blocks, 2), "load_list"),
            _dev(n_load, torch.int32, (B, H), "n_load")))

    def nosa_sparse_decode(self, q, pool_k, pool_v, pool_bias, sel_idx, n_sel, slot_of_block, n_tokens, out, lse=None,
                           static_scratch: bool = False) -> None:
        """``static_scratch=True`` calls nosa_sparse_decode_static (split results in the library's own array)."""
        p, B, H = self.p, self._B, self._H
        kv_pool = (B, H, p.gpu_slots, p.block_size, p.head_dim)
        fn = self.lib.nosa_sparse_decode_static if static_scratch else self.lib.nosa_sparse_decode
        self._check(fn(
            self._ctx, _dev(q, self.tdtype, (B, p.n_q_heads, p.head_dim), "q"),
            _dev(pool_k, self.tdtype, kv_pool, "pool_k"), _dev(pool_v, self.tdtype, kv_pool, "pool_v"),
            _dev(pool_bias, torch.float32, kv_pool[:4], "pool_bias"),
            _dev(sel_idx, torch.int32, (B, H, p.k_blocks), "sel_idx"),
            _dev(n_sel, torch.int32, (B, H), "n_sel"),
            _dev(slot_of_block, torch.int32, (B, H, p.max_blocks), "slot_of_block"),
            _dev(n_tokens, torch.int32, (B,), "n_tokens"),
            _dev(out, self.tdtype, (B, p.n_q_heads, p.head_dim), "out"),
            _dev(lse, torch.float32, (B, p.n_q_heads), "lse")))

    def nosa_pool_blocks(self, keys, bias, n_tokens, k_pooled, se_pooled) -> None:
        p, B, H = self.p, self._B, self._H
        kv = (B, H, p.max_blocks, p.block_size, p.head_dim)
        for t, name in ((keys, "keys"), (bias, "bias")):
            if not (t.is_cuda or t.is_pinned()):
                raise ValueError(f"{name} must be device or pinned host memory")
        self._check(self.lib.nosa_pool_blocks(
            self._ctx, _raw(keys, self.tdtype, kv, "keys"), _raw(bias, torch.float32, kv[:4], "bias"),
            _dev(n_tokens, torch.int32, (B,), "n_tokens"),
            _dev(k_pooled, self.tdtype, (B, H, p.n_sub_max, p.head_dim), "k_pooled"),
            _dev(se_pooled, torch.float32, (B, H, p.n_sub_max), "se_pooled")))

    def nosa_append(self, k_new, v_new, b_new, pool_k, pool_v, pool_bias, host_k, host_v, host_bias, k_pooled,
                    se_pooled, se_blk, n_tokens, slot_of_block, block_of_slot) -> None:
        p, B, H = self.p, self._B, self._H
        kv_host = (B, H, p.max_blocks, p.block_size, p.head_dim)
        kv_pool = (B, H, p.gpu_slots, p.block_size, p.head_dim)
        for t, name in ((host_k, "host_k"), (host_v, "host_v"), (host_bias, "host_bias")):
            if not (t.is_cuda or t.is_pinned()):
                raise ValueError(f"{name} must be pinned host memory (or device memory)")
        self._check(self.lib.nosa_append(
            self._ctx, _dev(k_new, self.tdtype, (B, H, p.head_dim), "k_new"), _dev(v_new, self.tdtype, (B, H, p.head_dim), "v_new"),
            _dev(b_new, torch.float32, (B, H), "b_new"),
            _dev(pool_k, self.tdtype, kv_pool, "pool_k"), _dev(pool_v, self.tdtype, kv_pool, "pool_v"),
            _dev(pool_bias, torch.float32, kv_pool[:4], "pool_bias"),
            _raw(host_k, self.tdtype, kv_host, "host_k"), _raw(host_v, self.tdtype, kv_host, "host_v"),
            _raw(host_bias, torch.float32, kv_host[:4], "host_bias"),
            _dev(k_pooled, self.tdtype, (B, H, p.n_sub_max, p.head_dim), "k_pooled"),
            _dev(se_pooled, torch.float32, (B, H, p.n_sub_max), "se_pooled"),
            _dev(se_blk, torch.float32, (B, H, p.max_blocks), "se_blk"),
            _dev(n_tokens, torch.int32, (B,), "n_tokens"),
            _dev(slot_of_block, torch.int32, (B, H, p.max_blocks), "slot_of_block"),
            _dev(block_of_slot, torch.int32, (B, H, p.gpu_slots), "block_of_slot")))

    def nosa_split_qkv_evict(self, qkv, w1, w2, mode, q_out, k_new, v_new, b_new) -> None:
        p, B, H = self.p, self._B, self._H
        d = p.head_dim
        self._check(self.lib.nosa_split_qkv_evict(
            self._ctx, _dev(qkv, self.tdtype, (B, (p.n_q_heads + 2 * H) * d), "qkv"),
            _dev(w1, torch.float32, (d, H), "w1"), _dev(w2, torch.float32, (H,), "w2"), int(mode),
            _dev(q_out, self.tdtype, (B, p.n_q_heads, d), "q_out"), _dev(k_new, self.tdtype, (B, H, d), "k_new"),
            _dev(v_new, self.tdtype, (B, H, d), "v_new"), _dev(b_new, torch.float32, (B, H), "b_new")))

    def nosa_prefill_select(self, q_chunk, k_pooled, se_pooled, p0, lq, n_tok_scratch, sq_scratch, se_scratch, sel_idx,
                            n_sel) -> None:
        p, B, H = self.p, self._B, self._H
        self._check(self.lib.nosa_prefill_select(
            self._ctx, _dev(q_chunk, self.tdtype, (B, lq, p.n_q_heads, p.head_dim), "q_chunk"),
            _dev(k_pooled, self.tdtype, (B, H, p.n_sub_max, p.head_dim), "k_pooled"),
            _dev(se_pooled, torch.float32, (B, H, p.n_sub_max), "se_pooled"), int(p0), int(lq),
            _dev(n_tok_scratch, torch.int32, (B * lq,), "n_tok_scratch"),
            _dev(sq_scratch, torch.float32, (B, lq, H, p.max_blocks), "sq_scratch"),
            _dev(se_scratch, torch.float32, (B, lq, H, p.max_blocks), "se_scratch"),
            _dev(sel_idx, torch.int32, (B, lq, H, p.k_blocks), "sel_idx"),
            _dev(n_sel, torch.int32, (B, lq, H), "n_sel")))

    def nosa_prefill_attend(self, q_chunk, cache_k, cache_v, cache_bias, sel_idx, n_sel, p0, lq, out, lse) -> None:
        p, B, H = self.p, self._B, self._H
        kv = (B, H, p.max_blocks, p.block_size, p.head_dim)
        self._check(self.lib.nosa_prefill_attend(
            self._ctx, _dev(q_chunk, self.tdtype, (B, lq, p.n_q_heads, p.head_dim), "q_chunk"),
            _dev(cache_k, self.tdtype, kv, "cache_k"), _dev(cache_v, self.tdtype, kv, "cache_v"),
            _dev(cache_bias, torch.float32, kv[:4], "cache_bias"),
            _dev(sel_idx, torch.int32, (B, lq, H, p.k_blocks), "sel_idx"),
            _dev(n_sel, torch.int32, (B, lq, H), "n_sel"), int(p0), int(lq),
            _dev(out, self.tdtype, (B, lq, p.n_q_heads, p.head_dim), "out"),
            _dev(lse, torch.float32, (B, lq, p.n_q_heads), "lse")))

    def step_args(self, q, k_pooled, se_pooled, n_tokens, sq_blk, se_blk, sel_idx, n_sel, slot_of_block, block_of_slot,
                  load_list, n_load, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, out, lse=None) -> StepArgs:
        """Checks every tensor once and packs the pointers of one whole step."""
        p, B, H = self.p, self._B, self._H
        d, nb = p.head_dim, p.block_size
        kv_host, kv_pool = (B, H, p.max_blocks, nb, d), (B, H, p.gpu_slots, nb, d)
        for t, name in ((host_k, "host_k"), (host_v, "host_v"), (host_bias, "host_bias")):
            if t is not None and not (t.is_cuda or t.is_pinned()):
                raise ValueError(f"{name} must be pinned host memory (or device memory)")
        v = lambda x: None if x is None else x.value
        return StepArgs(
            v(_dev(q, self.tdtype, (B, p.n_q_heads, d), "q")), v(_dev(k_pooled, self.tdtype, (B, H, p.n_sub_max, d), "k_pooled")),
            v(_dev(se_pooled, torch.float32, (B, H, p.n_sub_max), "se_pooled")), v(_dev(n_tokens, torch.int32, (B,), "n_tokens")),
            v(_dev(sq_blk, torch.float32, (B, H, p.max_blocks), "sq_blk")), v(_dev(se_blk, torch.float32, (B, H, p.max_blocks), "se_blk")),   # optional
            v(_dev(sel_idx, torch.int32, (B, H, p.k_blocks), "sel_idx")), v(_dev(n_sel, torch.int32, (B, H), "n_sel")),
            v(_dev(slot_of_block, torch.int32, (B, H, p.max_blocks), "slot_of_block")),
            v(_dev(block_of_slot, torch.int32, (B, H, p.gpu_slots), "block_of_slot")),
            v(_dev(load_list, torch.int32, (B, H, p.k_blocks, 2), "load_list")), v(_dev(n_load, torch.int32, (B, H), "n_load")),
            v(_raw(host_k, self.tdtype, kv_host, "host_k")), v(_raw(host_v, self.tdtype, kv_host, "host_v")),
            None if host_bias is None else v(_raw(host_bias, torch.float32, kv_host[:4], "host_bias")),
            v(_dev(pool_k, self.tdtype, kv_pool, "pool_k")), v(_dev(pool_v, self.tdtype, kv_pool, "pool_v")),
            v(_dev(pool_bias, torch.float32, kv_pool[:4], "pool_bias")),
            v(_dev(out, self.tdtype, (B, p.n_q_heads, d), "out")), v(_dev(lse, torch.float32, (B, p.n_q_heads), "lse")))

    def nosa_decode_step(self, args: StepArgs) -> None:
        self._check(self.lib.nosa_decode_step(self._ctx, ctypes.byref(args)))

    def nosa_graph_create(self, args: StepArgs) -> ctypes.c_void_p:
        g = ctypes.c_void_p()
        self._check(self.lib.nosa_graph_create(self._ctx, ctypes.byref(args), ctypes.byref(g)))
        return g

    def nosa_graph_begin(self) -> None:
        self._check(self.lib.nosa_graph_begin(self._ctx))

    def nosa_graph_end(self) -> ctypes.c_void_p:
        g = ctypes.c_void_p()
        self._check(self.lib.nosa_graph_end(self._ctx, ctypes.byref(g)))
        return g

    def nosa_graph_launch(self, graph: ctypes.c_void_p) -> None:
        self._check(self.lib.nosa_graph_launch(self._ctx, graph))

    def nosa_graph_destroy(self, graph: ctypes.c_void_p) -> None:
        self.lib.nosa_graph_destroy(graph)

    def nosa_fetch_tokens(self, host_k, host_v, host_bias, pool_k, pool_v, pool_bias, token_list, n_list) -> None:
        p, B, H = self.p, self._B, self._H
        kv_host = (B, H, p.max_blocks, p.block_size, p.head_dim)
        kv_pool = (B, H, p.gpu_slots, p.block_size, p.head_dim)
        M = token_list.shape[2]
        for t, name in ((host_k, "host_k"), (host_v, "host_v"), (host_bias, "host_bias")):
            if t is not None and not (t.is_cuda or t.is_pinned()):
                raise ValueError(f"{name} must be pinned host memory (or device memory)")
        self._check(self.lib.nosa_fetch_tokens(
            self._ctx, _raw(host_k, self.tdtype, kv_host, "host_k"), _raw(host_v, self.tdtype, kv_host, "host_v"),
            None if host_bias is None else _raw(host_bias, torch.float32, kv_host[:4], "host_bias"),
            _dev(pool_k, self.tdtype, kv_pool, "pool_k"), _dev(pool_v, self.tdtype, kv_pool, "pool_v"),
            _dev(pool_bias, torch.float32, kv_pool[:4], "pool_bias"),
            _dev(token_list, torch.int32, (B, H, M, 2), "token_list"), _dev(n_list, torch.int32, (B, H), "n_list"), M))
