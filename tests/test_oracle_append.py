"""Pins for the oracle's growing-context step (cache update before Stage 1, Alg. 1).

 - after every append the token sits at (block t // nb, row t % nb) of the host cache and the token
   count has advanced;
 - attention computed through the GPU-pool model (slots, maps, appended rows) equals brute-force
   masked attention over the host cache restricted to Gamma: a token written to the wrong slot or
   row, or a stale row that leaks in, breaks this;
 - the fetch bound of Theorem 1 (n_load <= Kq after the first step, C = K) holds across block
   boundaries with the stated slot rule;
 - incremental facts: a new block gets a slot at its first token without a fetch, and is never
   listed as a miss afterwards;
 - the fetch bound over many budgets, the tight ones included (Kq = 0: nothing may ever be fetched
   after the first step; Nw = 1: the block that leaves the window at a boundary must be allowed
   to give up its slot; Ke = 0: it is the only block that can).
"""
import numpy as np
import pytest

import oracle
from helpers import oracle_params, small_workload, to_np, widen
from nosa_inputs import CONFIGS, QueryStream, append_token, make_layer


def test_append_places_tokens_and_keeps_attention_and_fetch_bound():
    w = CONFIGS["tiny"].replace(context=64 * 14 + 61, generated=140, batch=2, n_q_heads=4, n_kv_heads=2)
    p = oracle_params(w)
    seed = 4
    layer = make_layer(w, seed, 0)
    hk, hv, hb = to_np(layer["host_k"]).copy(), to_np(layer["host_v"]).copy(), to_np(layer["host_bias"]).copy()
    n_tok = np.full((w.batch,), w.context, np.int32)
    B, H, C, nb, d = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim
    pk, pv = np.full((B, H, C, nb, d), np.nan, np.float32), np.full((B, H, C, nb, d), np.nan, np.float32)
    pb = np.full((B, H, C, nb), np.nan, np.float32)
    sob, bos = np.full((B, H, w.max_blocks), -1, np.int32), np.full((B, H, C), -1, np.int32)
    qs = QueryStream(w, seed, 0)
    prev_se = np.full((B, H, w.max_blocks), -np.inf)
    for t in range(140):
        if t > 0:
            tok = append_token(w, seed, 0, t)
            T0 = int(n_tok[0])
            J, row = T0 // nb, T0 % nb
            had_slot = sob[:, :, J].copy()
            bos_before = bos.copy()
            oracle.append(p, to_np(tok["k_new"]), to_np(tok["v_new"]), to_np(tok["b_new"]), pk, pv, pb, hk, hv, hb,
                          prev_se, n_tok, sob, bos)
            assert (n_tok == T0 + 1).all()
            assert (hk[:, :, J, row] == to_np(tok["k_new"])).all() and (hv[:, :, J, row] == to_np(tok["v_new"])).all()
            assert (hb[:, :, J, row] == to_np(tok["b_new"])).all()
            if row == 0:
                assert (had_slot < 0).all() and (sob[:, :, J] >= 0).all()      # new block: slot without a fetch
                for b in range(B):
                    for h in range(H):
                        s_new = sob[b, h, J]
                        empty = np.nonzero(bos_before[b, h] < 0)[0]
                        if len(empty):
                            assert s_new == empty[0]                             # lowest empty slot first
                        else:                                                    # else the least important candidate
                            protect = w.window_blocks       # J-Nw+1 .. J-1 stay in the window
                            cand = [s for s in range(C) if w.sink_blocks <= bos_before[b, h, s] <= J - protect]
                            want = min(cand, key=lambda s: (prev_se[b, h, bos_before[b, h, s]], s))
                            assert s_new == want
                            assert sob[b, h, bos_before[b, h, want]] == -1       # the evicted block lost its slot
        kc, sec = oracle.pool(p, hk, hb, n_tok)
        q = to_np(qs.next(t))
        sq, se = oracle.block_score(p, q, kc, sec, n_tok)
        prev_se = se
        sel, n_sel = oracle.select(p, sq, se, n_tok)
        ll, n_load = oracle.load(p, sel, n_sel, sob, bos)
        if t > 0:
            assert n_load.max() <= w.kq_blocks, (t, n_load.max())
            assert not (ll[..., 0] == (int(n_tok[0]) - 1) // nb).any()         # the tail block is never a miss
        oracle.fetch(p, hk, hv, hb, pk, pv, pb, ll, n_load)
        out, _ = oracle.attention(p, q, pk, pv, pb, sel, n_sel, sob, n_tok)
        T = int(n_tok[0])
        K64, V64 = widen(hk).reshape(B, H, -1, d), widen(hv).reshape(B, H, -1, d)
        B64 = hb.astype(np.float64).reshape(B, H, -1)
        for b in range(B):
            for hq in range(w.n_q_heads):
                h = hq // w.group
                mask = np.full(K64.shape[2], -np.inf)
                for J in sel[b, h, :n_sel[b, h]]:
                    mask[J * nb:(J + 1) * nb] = 0
                mask[T:] = -np.inf
                z = p.softmax_scale * (K64[b, h] @ widen(q)[b, hq]) + B64[b, h] + mask
                pr = np.exp(z - z.max())
                pr /= pr.sum()
                np.testing.assert_allclose(out[b, hq], pr @ V64[b, h], rtol=0, atol=1e-12)


@pytest.mark.parametrize("ns,nw,kq,ke", [(1, 1, 0, 1), (2, 1, 0, 0), (1, 1, 0, 2), (1, 2, 0, 1), (1, 3, 0, 2), (1, 1, 1, 1),
                                         (2, 2, 1, 0), (1, 1, 2, 3), (1, 3, 2, 0)])
def test_fetch_bound_holds_across_block_boundaries_for_tight_budgets(ns, nw, kq, ke):
    K = ns + nw + kq + ke
    for seed in (3, 17):
        rng = np.random.default_rng(seed * 100 + K)
        T = 64 * int(rng.integers(K, 2 * K + 3)) + int(rng.integers(0, 64))
        steps = 150
        w = small_workload(batch=1, n_q_heads=2, n_kv_heads=1, head_dim=64, context=T, k_blocks=K, kq_blocks=kq,
                           sink_blocks=ns, window_blocks=nw, gpu_slots=K, dtype="fp32", generated=steps + 1,
                           structure="key_offset" if seed == 3 else "drift")
        p = oracle_params(w)
        layer = make_layer(w, seed, 0)
        hk, hv, hb = to_np(layer["host_k"]).copy(), to_np(layer["host_v"]).copy(), to_np(layer["host_bias"]).copy()
        pk = np.zeros((1, 1, K, 64, 64), np.float32)
        pv, pb = np.zeros_like(pk), np.zeros((1, 1, K, 64), np.float32)
        sob, bos = np.full((1, 1, w.max_blocks), -1, np.int32), np.full((1, 1, K), -1, np.int32)
        n_tok = np.full((1,), T, np.int32)
        qs = QueryStream(w, seed, 0)
        prev_se = np.full((1, 1, w.max_blocks), -np.inf)
        for t in range(steps):
            if t > 0:
                tok = append_token(w, seed, 0, t)
                oracle.append(p, to_np(tok["k_new"]), to_np(tok["v_new"]), to_np(tok["b_new"]), pk, pv, pb, hk, hv, hb,
                              prev_se, n_tok, sob, bos)
            kc, sec = oracle.pool(p, hk, hb, n_tok)
            sq, se = oracle.block_score(p, to_np(qs.next(t)), kc, sec, n_tok)
            prev_se = se
            sel, n_sel = oracle.select(p, sq, se, n_tok)
            ll, n_load = oracle.load(p, sel, n_sel, sob, bos)
            oracle.fetch(p, hk, hv, hb, pk, pv, pb, ll, n_load)
            if t > 0:
                assert n_load.max() <= kq, f"seed {seed}, step {t}, T = {int(n_tok[0])}: {int(n_load.max())} blocks fetched, budget {kq}"
