"""Pins for the oracle's sparse prefill (a loop of decode steps over query positions).

 - with a budget that covers every block (K >= N) and b = 0 the result is plain causal attention:
   compared with torch's SDPA (is_causal) in fp64;
 - brute force from the mask Eq. of Sec. 2.1: for every query position, a 0 / -inf token mask built from
   causal AND (selected block), with the exp(b) exp(q k + m) form of the output Eq.;
 - the selection at position p0 + t only ever names blocks <= floor((p0 + t) / nb), contains the sink and
   the window blocks, and the block holding the query itself.
"""
import numpy as np
import torch

import oracle
from helpers import oracle_params, small_workload, to_np, widen
from nosa_inputs import make_layer


def _chunk_queries(w, Lq, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn((w.batch, Lq, w.n_q_heads, w.head_dim), generator=g).to(w.torch_dtype)


def test_full_budget_is_causal_dense_attention():
    n_blocks, Lq, p0 = 6, 128, 64 * 4
    w = small_workload(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, context=64 * n_blocks, k_blocks=n_blocks,
                       kq_blocks=1, gpu_slots=n_blocks, dtype="fp32")
    p = oracle_params(w)
    layer = make_layer(w, 3, 0)
    q = _chunk_queries(w, Lq, 1)
    hk, hv = to_np(layer["host_k"]), to_np(layer["host_v"])
    zero_b = np.zeros((w.batch, w.n_kv_heads, n_blocks, 64), np.float32)
    kc, sec = oracle.pool(p, hk, zero_b, np.full((w.batch,), 64 * n_blocks, np.int32))
    _, n_sel, out, _ = oracle.prefill(p, to_np(q), hk, hv, zero_b, kc, sec, p0)
    G = w.group
    T = p0 + Lq
    K = layer["host_k"].double().reshape(w.batch, w.n_kv_heads, -1, 64)[:, :, :T].repeat_interleave(G, 1)
    V = layer["host_v"].double().reshape(w.batch, w.n_kv_heads, -1, 64)[:, :, :T].repeat_interleave(G, 1)
    Q = q.double().permute(0, 2, 1, 3)                                  # [B,Hq,Lq,d]
    mask = torch.ones(Lq, T, dtype=torch.bool).tril(diagonal=p0)        # query t sees keys <= p0 + t
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask, scale=p.softmax_scale)
    np.testing.assert_allclose(out, ref.permute(0, 2, 1, 3).numpy(), rtol=0, atol=1e-12)


def test_prefill_equals_bruteforce_masked_attention_per_position():
    n_blocks, Lq, p0 = 14, 64 * 3, 64 * 11
    w = small_workload(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, context=64 * n_blocks, k_blocks=6,
                       kq_blocks=2, sink_blocks=1, window_blocks=2, gpu_slots=n_blocks, dtype="bf16")
    p = oracle_params(w)
    layer = make_layer(w, 5, 0)
    q = _chunk_queries(w, Lq, 2)
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    kc, sec = oracle.pool(p, hk, hb, np.full((w.batch,), 64 * n_blocks, np.int32))
    sel, n_sel, out, lse = oracle.prefill(p, to_np(q), hk, hv, hb, kc, sec, p0)
    K64, V64 = widen(hk).reshape(w.batch, w.n_kv_heads, -1, 64), widen(hv).reshape(w.batch, w.n_kv_heads, -1, 64)
    B64 = hb.astype(np.float64).reshape(w.batch, w.n_kv_heads, -1)
    Q64 = widen(to_np(q))
    for t in range(0, Lq, 7):
        pos = p0 + t
        N = pos // 64 + 1
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                g = sel[b, h, t, :n_sel[b, h, t]]
                assert n_sel[b, h, t] == min(6, N) and g.max() == pos // 64 and g[0] == 0      # own block, sink
                assert set(range(N - 2, N)) <= set(g.tolist())                                # window
                for gq in range(w.group):
                    hq = h * w.group + gq
                    m = np.full(K64.shape[2], -np.inf)
                    for J in g:
                        m[J * 64:(J + 1) * 64] = 0
                    m[pos + 1:] = -np.inf                                                      # causal
                    z = p.softmax_scale * (K64[b, h] @ Q64[b, t, hq]) + m
                    wgt = np.exp(B64[b, h]) * np.exp(z - z.max())
                    ref = (wgt[:, None] * V64[b, h]).sum(0) / wgt.sum()
                    np.testing.assert_allclose(out[b, t, hq], ref, rtol=0, atol=1e-12)
