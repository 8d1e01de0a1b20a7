"""GPU parity of the sparse prefill path (nosa_prefill_select + nosa_prefill_attend) against
oracle.prefill: the selection of every query position bit-exact, attention outputs within the
bf16 bar (max abs 1e-2), log-sum-exp within 1e-2.

Shapes cover both head dims, groups of 2 / 4 / 6 / 8 / 16 query heads per KV head (fewer, exactly and
more than the four waves of a workgroup), chunks that start at position 0 (positions with fewer
blocks than the budget), chunks deep in a context, one and several 64-position workgroups, and the
8B-shaped case at full size on sampled positions.
"""
import numpy as np
import pytest
import torch

from helpers import gpu_params, small_workload
from nosa_inputs import CONFIGS
from pipeline import run_prefill_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw,p0,lq", [
    ("d64_g2_deep", dict(n_q_heads=4, n_kv_heads=2, head_dim=64, k_blocks=6, kq_blocks=2, window_blocks=2), 64 * 11, 64 * 3),
    ("d128_g4_from_zero", dict(n_q_heads=8, n_kv_heads=2, head_dim=128, k_blocks=8, kq_blocks=2, window_blocks=2), 0, 64 * 12),
    ("d128_g6", dict(n_q_heads=12, n_kv_heads=2, head_dim=128, k_blocks=8, kq_blocks=3, window_blocks=1), 64 * 5, 64 * 4),
    ("d64_g8", dict(n_q_heads=16, n_kv_heads=2, head_dim=64, k_blocks=10, kq_blocks=2, window_blocks=3), 64 * 20, 64 * 4),
    ("d128_g4_one_wg", dict(batch=1, n_q_heads=4, n_kv_heads=1, head_dim=128, k_blocks=5, kq_blocks=1, window_blocks=1), 64 * 9, 64),
    ("overlapping_pool_windows", dict(n_q_heads=8, n_kv_heads=2, head_dim=128, k_blocks=8, kq_blocks=2, window_blocks=2,
                                      pool_kernel=32, pool_stride=16), 64 * 6, 64 * 4),
    ("d128_g16", dict(n_q_heads=16, n_kv_heads=1, head_dim=128, k_blocks=7, kq_blocks=2, window_blocks=2), 64 * 7, 64 * 2),
    ("d128_g7", dict(n_q_heads=14, n_kv_heads=2, head_dim=128, k_blocks=8, kq_blocks=2, window_blocks=2), 64 * 6, 64 * 3),
    ("budget_covers_all", dict(n_q_heads=8, n_kv_heads=2, head_dim=128, k_blocks=10, kq_blocks=4, window_blocks=2), 0, 64 * 8),
])
def test_prefill_parity(name, kw, p0, lq):
    n_blocks = (p0 + lq) // 64 + 2          # two blocks of slack behind the chunk
    base = dict(batch=2, context=p0 + lq, gpu_slots=n_blocks, dtype="bf16", structure="planted", generated=128)
    base.update(kw)
    w = small_workload(**base)
    assert w.max_blocks == n_blocks
    r = run_prefill_parity(w, seed=31, p0=p0, lq=lq)
    print(name, r)


def test_prefill_rejects_what_it_does_not_support():
    import paper_2510_13602_amd as nosa
    w = small_workload(batch=1, context=64 * 8, gpu_slots=8, dtype="bf16", k_blocks=6)
    ctx = nosa.Nosa(gpu_params(w))
    B, H, d, K, lq = w.batch, w.n_kv_heads, w.head_dim, w.k_blocks, 64
    dev = "cuda:0"
    q = torch.zeros((B, lq, w.n_q_heads, d), dtype=torch.bfloat16, device=dev)
    kv = torch.zeros((B, H, w.max_blocks, 64, d), dtype=torch.bfloat16, device=dev)
    bias = torch.zeros((B, H, w.max_blocks, 64), dtype=torch.float32, device=dev)
    sel = torch.zeros((B, lq, H, K), dtype=torch.int32, device=dev)
    n_sel = torch.zeros((B, lq, H), dtype=torch.int32, device=dev)
    out = torch.zeros_like(q)
    lse = torch.zeros((B, lq, w.n_q_heads), dtype=torch.float32, device=dev)
    with pytest.raises(nosa.NosaError, match="multiples of the block size"):
        ctx.nosa_prefill_attend(q, kv, kv, bias, sel, n_sel, 32, lq, out, lse)
    with pytest.raises(nosa.NosaError, match="exceeds the cache"):
        ctx.nosa_prefill_attend(q, kv, kv, bias, sel, n_sel, 64 * 8, lq, out, lse)
    ctx.close()
    w2 = small_workload(batch=1, context=64 * 8, gpu_slots=6, dtype="bf16", k_blocks=6)
    ctx = nosa.Nosa(gpu_params(w2))
    kv2 = torch.zeros((B, H, w2.max_blocks, 64, d), dtype=torch.bfloat16, device=dev)
    bias2 = torch.zeros((B, H, w2.max_blocks, 64), dtype=torch.float32, device=dev)
    with pytest.raises(nosa.NosaError, match="gpu_slots"):
        ctx.nosa_prefill_attend(q, kv2, kv2, bias2, sel, n_sel, 0, lq, out, lse)
    ctx.close()
    # fewer pooled keys than blocks in the prefix: the selection would read past the pooled arrays
    ctx = nosa.Nosa(gpu_params(w, n_sub_max=4))
    with pytest.raises(nosa.NosaError, match="pooled keys do not cover"):
        ctx.nosa_prefill_attend(q, kv, kv, bias, sel, n_sel, 64 * 5, lq, out, lse)
    ctx.close()
    w3 = small_workload(batch=1, context=64 * 8, gpu_slots=8, dtype="fp32", k_blocks=6)
    ctx = nosa.Nosa(gpu_params(w3))
    with pytest.raises(nosa.NosaError, match="bf16 only"):
        ctx.nosa_prefill_attend(q.float(), kv.float(), kv.float(), bias, sel, n_sel, 0, lq, out.float(), lse)
    ctx.close()


def test_prefill_8b_shape_full_size_sampled():
    """The configuration bench.py's prefill study times (8B shape, chunk of 2048 positions at the end of a
    32768-token context), batch 2; the oracle computes a sample of positions one by one."""
    lq = 2048
    w = CONFIGS["8b"].replace(batch=2)
    w = w.replace(gpu_slots=w.max_blocks)
    p0 = w.context - lq
    rng = np.random.default_rng(5)
    positions = sorted(set([0, 1, 63, 64, 65, 1023, 1024, lq - 65, lq - 64, lq - 1] + rng.integers(0, lq, 22).tolist()))
    r = run_prefill_parity(w, seed=11, p0=p0, lq=lq, positions=positions)
    print("8b sampled", r)
