"""Pins for the oracle's attention step against things other than itself.

 (i)   everything selected and b = 0  ==  textbook softmax(scale * Q K^T) V  (attention Eq. of
       Sec. 2.1 with M = 0), evaluated by torch's SDPA in fp64;
 (ii)  brute-force dense attention over ALL tokens of the host cache with the 0 / -inf token
       mask of Sec. 3.1 "Attention Calculation" and the exp(b) * exp(q k + m) product form;
 (iii) the softmax weights sum to one;
 (iv)  splitting Gamma into chunks and merging with log-sum-exp equals the one-shot result
       (this also pins the lse output);
 (v)   shift invariance of the bias (b + c leaves the output unchanged, lse moves by c).
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import oracle_params, small_workload, to_np, widen
from nosa_inputs import QueryStream, make_layer


def _all_resident(w, layer):
    """Pool = first C blocks of the host cache, identity slot map."""
    C = w.gpu_slots
    pk = layer["host_k"][:, :, :C].contiguous()
    pv = layer["host_v"][:, :, :C].contiguous()
    pb = layer["host_bias"][:, :, :C].contiguous()
    sob = np.full((w.batch, w.n_kv_heads, w.max_blocks), -1, np.int32)
    sob[:, :, :C] = np.arange(C, dtype=np.int32)
    return to_np(pk), to_np(pv), to_np(pb), sob


def _scattered(w, layer, sel, seed=0):
    """Pool whose slots hold the selected blocks in a shuffled order (tests the indirection)."""
    rng = np.random.default_rng(seed)
    B, H, C, nb, d = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    pk = np.zeros((B, H, C, nb, d), hk.dtype)
    pv = np.zeros((B, H, C, nb, d), hv.dtype)
    pb = np.zeros((B, H, C, nb), np.float32)
    sob = np.full((B, H, w.max_blocks), -1, np.int32)
    for b in range(B):
        for h in range(H):
            slots = rng.permutation(C)
            for i, J in enumerate(sel[b, h]):
                if J < 0:
                    continue
                s = slots[i]
                pk[b, h, s], pv[b, h, s], pb[b, h, s] = hk[b, h, J], hv[b, h, J], hb[b, h, J]
                sob[b, h, J] = s
    return pk, pv, pb, sob


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_select_all_no_bias_is_textbook_attention(dtype):
    n = 5
    w = small_workload(context=64 * n, k_blocks=n, gpu_slots=n, kq_blocks=1, dtype=dtype, n_q_heads=6,
                       n_kv_heads=2, head_dim=64)
    p = oracle_params(w)
    layer = make_layer(w, seed=3, layer=0)
    q = QueryStream(w, 3, 0).next(0)
    pk, pv, _, sob = _all_resident(w, layer)
    sel = np.tile(np.arange(n, dtype=np.int32), (w.batch, w.n_kv_heads, 1))
    n_sel = np.full((w.batch, w.n_kv_heads), n, np.int32)
    n_tok = np.full((w.batch,), w.context, np.int32)
    out, lse = oracle.attention(p, to_np(q), pk, pv, None, sel, n_sel, sob, n_tok)

    G = w.group
    q64 = q.double()[:, :, None, :]                                        # [B,Hq,1,d]
    k64 = layer["host_k"].double().reshape(w.batch, w.n_kv_heads, -1, w.head_dim).repeat_interleave(G, 1)
    v64 = layer["host_v"].double().reshape(w.batch, w.n_kv_heads, -1, w.head_dim).repeat_interleave(G, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(q64, k64, v64, scale=p.softmax_scale)[:, :, 0]
    np.testing.assert_allclose(out, ref.numpy(), rtol=0, atol=1e-12)
    ref_lse = torch.logsumexp(p.softmax_scale * (q64 @ k64.transpose(-1, -2))[:, :, 0], dim=-1)
    np.testing.assert_allclose(lse, ref_lse.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype,tail", [("fp32", 0), ("bf16", 0), ("bf16", 17), ("fp32", 63)])
def test_brute_force_masked_dense_attention(dtype, tail):
    """Eq. for o_t with m_j in {0, -inf} over every token of the cache, product form."""
    n_full = 11
    T = 64 * n_full + tail
    w = small_workload(context=T, k_blocks=6, gpu_slots=6, dtype=dtype)
    p = oracle_params(w)
    layer = make_layer(w, seed=5, layer=0)
    q = QueryStream(w, 5, 0).next(0)
    N = w.max_blocks
    rng = np.random.default_rng(7)
    sel = np.full((w.batch, w.n_kv_heads, w.k_blocks), -1, np.int32)
    n_sel = np.zeros((w.batch, w.n_kv_heads), np.int32)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            m = w.k_blocks - (b + h) % 2          # also exercise n_sel < K
            others = rng.choice(N - 1, size=m - 1, replace=False)
            blocks = np.sort(np.concatenate([others, [N - 1]]))   # tail block always attended
            sel[b, h, :m] = blocks
            n_sel[b, h] = m
    pk, pv, pb, sob = _scattered(w, layer, sel)
    n_tok = np.full((w.batch,), T, np.int32)
    out, lse, probs = oracle.attention(p, to_np(q), pk, pv, pb, sel, n_sel, sob, n_tok, with_probs=True)

    K = widen(to_np(layer["host_k"])).reshape(w.batch, w.n_kv_heads, -1, w.head_dim)
    V = widen(to_np(layer["host_v"])).reshape(w.batch, w.n_kv_heads, -1, w.head_dim)
    Bi = to_np(layer["host_bias"]).astype(np.float64).reshape(w.batch, w.n_kv_heads, -1)
    Q = widen(to_np(q))
    for b in range(w.batch):
        for hq in range(w.n_q_heads):
            h = hq // w.group
            mask = np.full(N * 64, -np.inf)
            for J in sel[b, h, :n_sel[b, h]]:
                mask[J * 64:(J + 1) * 64] = 0.0
            mask[T:] = -np.inf                                      # causal: tokens that exist
            logits = p.softmax_scale * (K[b, h] @ Q[b, hq]) + mask
            c = logits.max()
            wgt = np.exp(Bi[b, h]) * np.exp(logits - c)             # exp(b_j) * exp(q k_j + m_j)
            ref = (wgt[:, None] * V[b, h]).sum(0) / wgt.sum()
            np.testing.assert_allclose(out[b, hq], ref, rtol=0, atol=1e-12)
            np.testing.assert_allclose(lse[b, hq], c + np.log(wgt.sum()), rtol=0, atol=1e-12)
    np.testing.assert_allclose(probs.sum(-1), 1.0, rtol=0, atol=1e-13)
    assert (probs >= 0).all()


def test_chunked_lse_merge_equals_one_shot():
    w = small_workload(context=64 * 12, k_blocks=8, gpu_slots=8, dtype="bf16")
    p = oracle_params(w)
    layer = make_layer(w, seed=9, layer=0)
    q = to_np(QueryStream(w, 9, 0).next(0))
    sel = np.tile(np.array([0, 2, 3, 5, 7, 8, 10, 11], np.int32), (w.batch, w.n_kv_heads, 1))
    n_sel = np.full((w.batch, w.n_kv_heads), 8, np.int32)
    pk, pv, pb, sob = _scattered(w, layer, sel, seed=1)
    n_tok = np.full((w.batch,), w.context, np.int32)
    out, lse = oracle.attention(p, q, pk, pv, pb, sel, n_sel, sob, n_tok)

    parts = []
    for lo, hi in [(0, 3), (3, 4), (4, 8)]:
        s = np.full_like(sel, -1)
        s[:, :, :hi - lo] = sel[:, :, lo:hi]
        parts.append(oracle.attention(p, q, pk, pv, pb, s, np.full_like(n_sel, hi - lo), sob, n_tok))
    m = np.max([l for _, l in parts], axis=0)
    wsum = sum(np.exp(l - m) for _, l in parts)
    merged = sum(np.exp(l - m)[..., None] * o for o, l in parts) / wsum[..., None]
    np.testing.assert_allclose(merged, out, rtol=0, atol=1e-13)
    np.testing.assert_allclose(m + np.log(wsum), lse, rtol=0, atol=1e-13)


def test_bias_shift_invariance_and_effect():
    w = small_workload(context=64 * 6, k_blocks=6, gpu_slots=6, dtype="fp32")
    p = oracle_params(w)
    layer = make_layer(w, seed=11, layer=0)
    q = to_np(QueryStream(w, 11, 0).next(0))
    pk, pv, pb, sob = _all_resident(w, layer)
    sel = np.tile(np.arange(6, dtype=np.int32), (w.batch, w.n_kv_heads, 1))
    n_sel = np.full((w.batch, w.n_kv_heads), 6, np.int32)
    n_tok = np.full((w.batch,), w.context, np.int32)
    o0, l0 = oracle.attention(p, q, pk, pv, pb, sel, n_sel, sob, n_tok)
    o1, l1 = oracle.attention(p, q, pk, pv, (pb + np.float32(1.5)), sel, n_sel, sob, n_tok)
    np.testing.assert_allclose(o1, o0, rtol=0, atol=1e-6)      # fp32 bias + 1.5 rounds
    np.testing.assert_allclose(l1 - l0, 1.5, rtol=0, atol=1e-6)
    o2, _ = oracle.attention(p, q, pk, pv, None, sel, n_sel, sob, n_tok)
    assert np.abs(o2 - o0).max() > 1e-3                         # the bias is not ignored
    # a bias of -inf-like magnitude on all but one token returns that token's value row
    pb2 = np.full_like(pb, -1e4)
    pb2[:, :, 2, 5] = 0.0
    o3, _ = oracle.attention(p, q, pk, pv, pb2, sel, n_sel, sob, n_tok)
    v = widen(pv)[:, :, 2, 5]                                   # [B,Hkv,d]
    np.testing.assert_allclose(o3, np.repeat(v, w.group, axis=1), rtol=0, atol=1e-12)


def test_missing_slot_is_an_error():
    w = small_workload(context=64 * 6, k_blocks=6, gpu_slots=6)
    p = oracle_params(w)
    layer = make_layer(w, seed=1, layer=0)
    q = to_np(QueryStream(w, 1, 0).next(0))
    pk, pv, pb, sob = _all_resident(w, layer)
    sob[0, 0, 3] = -1
    sel = np.tile(np.arange(6, dtype=np.int32), (w.batch, w.n_kv_heads, 1))
    n_sel = np.full((w.batch, w.n_kv_heads), 6, np.int32)
    with pytest.raises(RuntimeError):
        oracle.attention(p, q, pk, pv, pb, sel, n_sel, sob, np.full((w.batch,), w.context, np.int32))
