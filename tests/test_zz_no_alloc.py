"""nosa_sparse_decode_static -- the attention entry point that allocates nothing and keeps its split
partial results in the library's static device array -- against nosa_sparse_decode with a caller
workspace: same kernels, so the outputs must agree bit for bit, and both must meet the oracle's bar.
Two calls in a row share the array; the second is smaller (fewer units, fewer tokens, fewer splits),
so stale partial results of the first sit right behind the ones it writes.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from helpers import gpu_params, oracle_params, out_tol, to_np
from nosa_inputs import CONFIGS, QueryStream, make_layer

pytestmark = pytest.mark.gpu


def _twin_run(w, seed, steps, overlap, splits=None):
    """Twin layer states: A runs whole steps through nosa_sparse_decode (workspace), B through
    nosa_sparse_decode_static (a context that was never given a workspace).  Returns the worst error
    of B against the oracle's attention on B's own state."""
    import paper_2510_13602_amd as nosa
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    dev = "cuda:0"
    layer = make_layer(w, seed, 0)
    hk, hv, hb = pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"])
    n_tok = torch.full((w.batch,), w.context, dtype=torch.int32)
    ctx_a = nosa.Nosa(gpu_params(w))
    ctx_b = nosa.Nosa(gpu_params(w), workspace=False)
    assert ctx_b.workspace is None
    for c in (ctx_a, ctx_b):
        c.set_overlap(overlap)
        if splits:
            c.set_splits(splits)
    assert ctx_b.splits > 1, "the case must use the scratch: more than one split"
    a, b = LayerCache(ctx_a, hk, hv, hb, n_tok), LayerCache(ctx_b, hk, hv, hb, n_tok)
    a.rebuild_pooled()
    b.rebuild_pooled()
    po = oracle_params(w)
    n_np = n_tok.numpy()
    qs = QueryStream(w, seed, 0)
    worst = 0.0
    for t in range(steps):
        q = qs.next(t).to(dev)
        oa = a.step(q)
        b.score(q)
        b.select()
        b.fetch()
        ctx_b.nosa_sparse_decode(q, b.pool_k, b.pool_v, b.pool_bias, b.sel_idx, b.n_sel, b.slot_of_block, b.n_tokens,
                                 b.out, b.lse, static_scratch=True)
        torch.cuda.synchronize()
        assert (a.sel_idx == b.sel_idx).all() and (a.slot_of_block == b.slot_of_block).all()
        assert to_np(oa).tobytes() == to_np(b.out).tobytes(), f"step {t}: static-scratch output differs from the workspace one"
        assert to_np(a.lse).tobytes() == to_np(b.lse).tobytes()
        ref, ref_lse = oracle.attention(po, to_np(q), to_np(b.pool_k), to_np(b.pool_v), to_np(b.pool_bias),
                                        b.sel_idx.cpu().numpy(), b.n_sel.cpu().numpy(), b.slot_of_block.cpu().numpy(), n_np)
        got = b.out.double().cpu().numpy()
        assert np.isfinite(got).all()
        worst = max(worst, float(np.abs(got - ref).max()))
        assert worst <= out_tol(w.dtype), f"step {t}: max abs err {worst}"
        assert np.abs(b.lse.double().cpu().numpy() - ref_lse).max() <= 1e-3
    ctx_a.close()
    ctx_b.close()
    return worst


@pytest.mark.parametrize("overlap", [False, True])
def test_static_scratch_decode_two_calls_second_smaller(overlap):
    big = CONFIGS["1b"].replace(batch=4)                                      # 8 units x 8 splits, G = 8, d = 64
    small = CONFIGS["1b"].replace(batch=1, context=64 * 40 + 17)              # 2 units, ragged tail, 5 splits
    e1 = _twin_run(big, seed=21, steps=3, overlap=overlap)
    e2 = _twin_run(small, seed=22, steps=3, overlap=overlap, splits=5)
    # a third call with many more units than either: its arrival counters lie where a layout that packed the
    # partial results right behind each context's own counters would have left the earlier calls' floats
    wide = CONFIGS["1b"].replace(batch=80)                                    # 160 units x 4 splits
    e3 = _twin_run(wide, seed=24, steps=2, overlap=overlap)
    print(f"static scratch (overlap={overlap}): worst err big {e1:.2e}, small {e2:.2e}, wide {e3:.2e}", flush=True)


def test_static_scratch_fp32_group4():
    w = CONFIGS["tiny"].replace(batch=3, n_q_heads=8, n_kv_heads=2)
    e = _twin_run(w, seed=23, steps=2, overlap=False, splits=4)
    print(f"static scratch fp32: worst err {e:.2e}", flush=True)


def test_static_scratch_rejects_sizes_beyond_the_array():
    """8B shape at 16 splits needs 512 x 16 x 4 x 130 x 4 B = 17 MB of partial results: more than the array."""
    import paper_2510_13602_amd as nosa
    w = CONFIGS["8b"]
    ctx = nosa.Nosa(gpu_params(w), workspace=False)
    ctx.set_splits(16)
    dummy = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    ptr = ctypes.c_void_p(dummy.data_ptr())
    rc = ctx.lib.nosa_sparse_decode_static(ctx._ctx, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr)   # rejected before any launch
    assert rc == nosa.binding.NOSA_ESHAPE
    msg = ctx.lib.nosa_last_error(ctx._ctx).decode()
    assert "static" in msg and str(nosa.STATIC_SCRATCH_BYTES) in msg
    big = nosa.Nosa(gpu_params(w.replace(batch=4096)), workspace=False)      # 32768 units: more than the counter region holds
    big.set_splits(1)
    assert big.lib.nosa_sparse_decode_static(big._ctx, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == nosa.binding.NOSA_ESHAPE
    assert "arrival counters" in big.lib.nosa_last_error(big._ctx).decode()
    big.close()
    ctx.set_splits(1)                                                         # 1 MB: fits
    assert 65536 + 512 * 4 * 130 * 4 <= nosa.STATIC_SCRATCH_BYTES
    # the workspace entry point, on the other hand, refuses to split without a workspace
    ctx.set_splits(2)
    rc = ctx.lib.nosa_sparse_decode(ctx._ctx, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr)
    assert rc == nosa.binding.NOSA_EINVAL
    ctx.close()
