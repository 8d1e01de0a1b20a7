"""Pins for the oracle's eviction head (importance-score Eq. of Sec. 3.1; ED-DMA row of the table in
App. D) and QKV split.

 - against torch: softplus(v @ W1) in fp64 through torch.nn.functional.softplus, both readings
   (one gate per KV head; the shared two-layer form of the Eq. as printed);
 - closed forms: softplus(0) = ln 2; softplus(x) - softplus(-x) = x; large |x| limits; w2 = 0 -> b = 0;
   the bias is linear in w2;
 - the split is a bit copy of the three segments of the fused activation, in q | k | v order;
 - mode 1 with Hkv = 1 equals mode 0.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from helpers import oracle_params, small_workload, to_np, widen


def _case(dtype, B=3, Hq=8, Hkv=2, d=64, seed=0):
    w = small_workload(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, dtype=dtype)
    g = torch.Generator().manual_seed(seed)
    qkv = torch.randn((B, (Hq + 2 * Hkv) * d), generator=g).to(w.torch_dtype)
    w1 = (torch.randn((d, Hkv), generator=g) / math.sqrt(d)).float()
    w2 = torch.randn((Hkv,), generator=g).float()
    return w, qkv, w1, w2


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("mode", [0, 1])
def test_eviction_head_against_torch_softplus(dtype, mode):
    w, qkv, w1, w2 = _case(dtype)
    p = oracle_params(w)
    q, k, v, b = oracle.split_qkv_evict(p, to_np(qkv), w1.numpy(), w2.numpy(), mode)
    B, Hq, H, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    seg = qkv.view(B, Hq + 2 * H, d)
    assert to_np(seg[:, :Hq].contiguous()).tobytes() == q.tobytes()
    assert to_np(seg[:, Hq:Hq + H].contiguous()).tobytes() == k.tobytes()
    assert to_np(seg[:, Hq + H:].contiguous()).tobytes() == v.tobytes()
    v64 = seg[:, Hq + H:].double()                                        # [B,H,d]
    hidden = torch.nn.functional.softplus(v64 @ w1.double())              # [B,H,Hkv]
    if mode == 0:
        ref = torch.diagonal(hidden, dim1=1, dim2=2) * w2.double()
    else:
        ref = hidden @ w2.double()
    np.testing.assert_allclose(b, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_softplus_closed_forms_through_the_head():
    # one head, d = 64, v = x * e_0 and w1 = e_0  ->  v . w1 = x exactly
    w = small_workload(batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, dtype="fp32")
    p = oracle_params(w)
    w1 = np.zeros((64, 1), np.float32); w1[0, 0] = 1.0
    w2 = np.array([1.0], np.float32)

    def head(x, w2v=w2):
        qkv = np.zeros((1, 3 * 64), np.float32)
        qkv[0, 2 * 64] = x
        return oracle.split_qkv_evict(p, qkv, w1, w2v, 0)[3][0, 0]

    assert abs(head(0.0) - math.log(2.0)) < 1e-15
    for x in (0.5, 3.0, 17.0):
        assert abs(head(x) - head(-x) - x) < 1e-12                       # softplus(x) - softplus(-x) = x
    assert abs(head(50.0) - 50.0) < 1e-12 and 0 < head(-50.0) < 1e-20       # limits, no overflow
    assert head(800.0) == 800.0
    assert head(1.25, np.array([0.0], np.float32)) == 0.0
    assert abs(head(1.25, np.array([-2.0], np.float32)) + 2 * head(1.25)) < 1e-15   # linear in w2


def test_shared_form_reduces_to_per_head_form_for_one_kv_head():
    w, qkv, w1, w2 = _case("bf16", Hq=4, Hkv=1, d=128, seed=3)
    p = oracle_params(w)
    b0 = oracle.split_qkv_evict(p, to_np(qkv), w1.numpy(), w2.numpy(), 0)[3]
    b1 = oracle.split_qkv_evict(p, to_np(qkv), w1.numpy(), w2.numpy(), 1)[3]
    assert (b0 == b1).all()
