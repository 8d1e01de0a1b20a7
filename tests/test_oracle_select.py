"""Pins for the oracle's constrained selection (selection Eq., Sec. 3.1) and block scores.

 (i)   exhaustive subset search on tiny inputs: the query-aware picks are the size-Kq subset of
       the candidates with the largest total s^q, the query-agnostic picks the size-Ke subset of
       the remaining candidates with the largest total s^e;
 (ii)  the single-pass form of the selection Eq.: set the query-aware picks (and the forced
       blocks) to +inf, otherwise use s^e, then take one ArgTop_K;
 (iii) Kq = 0 -> selection independent of the query (Sec. 2.1 "query-agnostic ... fixed
       eviction pattern"); Ke = 0 -> plain query-aware top-k (InfLLMv2 mask Eq.);
 (iv)  counts: |Gamma| = min(K, N), forced blocks inside, ascending, unique;
 (v)   the Ke best-by-s^e candidates are always selected (proof of Theorem 1, App. E);
 (vi)  the paper's worked budget: tests/golden/budget_example.txt.
 Scores: pooled-key scoring equals pooling of per-token scores (linearity); the block max of
 the max-pooling Eq. against a brute-force enumeration of sub-blocks for several (lk, ls).
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from helpers import oracle_params, small_workload, to_np, widen
from nosa_inputs import QueryStream, make_layer

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _geometry(T, nb, Ns, Nw):
    N, Nc = -(-T // nb), T // nb
    forced = sorted(set(range(min(Ns, N))) | set(range(max(0, N - Nw), N)))
    cand = [J for J in range(Nc) if J not in forced]
    return N, Nc, forced, cand


def _rand_scores(rng, B, H, nmax, distinct=True):
    if distinct:
        sq = np.stack([rng.permutation(nmax) for _ in range(B * H)]).reshape(B, H, nmax).astype(np.float64)
        se = np.stack([rng.permutation(nmax) for _ in range(B * H)]).reshape(B, H, nmax).astype(np.float64)
        return sq + 0.25, -se * 0.5
    return (rng.integers(0, 3, (B, H, nmax)).astype(np.float64),
            rng.integers(0, 3, (B, H, nmax)).astype(np.float64))


@pytest.mark.parametrize("T,K,Kq,Ns,Nw", [
    (64 * 12, 6, 2, 1, 1), (64 * 12, 7, 3, 1, 2), (64 * 11 + 5, 6, 2, 1, 1), (64 * 10 + 63, 8, 2, 2, 2),
    (64 * 9, 5, 0, 1, 1), (64 * 9, 5, 3, 1, 1), (64 * 8, 8, 2, 1, 1), (64 * 3, 6, 2, 1, 1), (64 * 12, 4, 2, 0, 1),
    (30, 4, 1, 1, 1), (64 * 12, 8, 2, 1, 4),
])
def test_exhaustive_subset_search(T, K, Kq, Ns, Nw):
    rng = np.random.default_rng(T * 131 + K * 17 + Kq)
    w = small_workload(batch=3, n_q_heads=2, n_kv_heads=2, context=T, k_blocks=K, kq_blocks=Kq,
                       sink_blocks=Ns, window_blocks=Nw, gpu_slots=max(K, 1))
    p = oracle_params(w)
    sq, se = _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks)
    n_tok = np.full((w.batch,), T, np.int32)
    sel, n_sel, kind = oracle.select(p, sq, se, n_tok, with_kind=True)
    N, Nc, forced, cand = _geometry(T, 64, Ns, Nw)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            kq = min(Kq, len(cand))
            best_q = max(itertools.combinations(cand, kq), key=lambda S: sum(sq[b, h, J] for J in S))
            rest = [J for J in cand if J not in best_q]
            ke = min(max(K - len(forced) - Kq, 0), len(rest))
            best_e = max(itertools.combinations(rest, ke), key=lambda S: sum(se[b, h, J] for J in S))
            want = sorted(set(forced) | set(best_q) | set(best_e))
            got = sel[b, h, :n_sel[b, h]].tolist()
            assert got == want, (b, h, got, want)
            assert (sel[b, h, n_sel[b, h]:] == -1).all()
            assert n_sel[b, h] == min(K, N)
            kd = dict(zip(got, kind[b, h, :n_sel[b, h]].tolist()))
            assert all(kd[J] == 0 for J in forced)
            assert all(kd[J] == 1 for J in best_q)
            assert all(kd[J] == 2 for J in best_e)


@pytest.mark.parametrize("distinct", [True, False])
def test_single_pass_infinity_form(distinct):
    """One ArgTop_K over s = +inf on forced/query-aware blocks, s^e elsewhere (ties -> lower index)."""
    rng = np.random.default_rng(21)
    T, K, Kq, Ns, Nw = 64 * 40 + 9, 16, 4, 1, 4
    w = small_workload(batch=4, context=T, k_blocks=K, kq_blocks=Kq, sink_blocks=Ns, window_blocks=Nw, gpu_slots=K)
    p = oracle_params(w)
    sq, se = _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks, distinct)
    sel, n_sel = oracle.select(p, sq, se, np.full((w.batch,), T, np.int32))
    N, Nc, forced, cand = _geometry(T, 64, Ns, Nw)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            order_q = sorted(cand, key=lambda J: (-sq[b, h, J], J))[:Kq]
            s = np.full(N, -np.inf)
            s[cand] = se[b, h, cand]
            s[order_q] = np.inf
            s[forced] = np.inf
            top = sorted(range(N), key=lambda J: (-s[J], J))[:K]
            assert sorted(top) == sel[b, h, :n_sel[b, h]].tolist()


def test_kq_zero_is_query_agnostic_and_ke_zero_is_plain_topk():
    rng = np.random.default_rng(5)
    T, Ns, Nw = 64 * 30, 1, 3
    w = small_workload(batch=2, context=T, k_blocks=10, kq_blocks=0, sink_blocks=Ns, window_blocks=Nw, gpu_slots=10)
    p = oracle_params(w)
    _, se = _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks)
    n_tok = np.full((w.batch,), T, np.int32)
    sels = [oracle.select(p, _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks)[0], se, n_tok)[0] for _ in range(4)]
    for s in sels[1:]:
        assert (s == sels[0]).all()                 # Kq = 0: the same set whatever the query scores
    # Ke = 0: K = |F| + Kq -> forced + plain top-Kq by the query-aware score
    w2 = w.replace(k_blocks=4 + 6, kq_blocks=6)
    p2 = oracle_params(w2)
    sq, se2 = _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks)
    sel, n_sel = oracle.select(p2, sq, se2, n_tok)
    N, Nc, forced, cand = _geometry(T, 64, Ns, Nw)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            top = sorted(cand, key=lambda J: -sq[b, h, J])[:6]
            assert sel[b, h].tolist() == sorted(set(forced) | set(top))
            # and it does not depend on s^e at all
    sel3, _ = oracle.select(p2, sq, -se2, n_tok)
    assert (sel3 == sel).all()


def test_invariants_and_best_agnostic_always_selected():
    rng = np.random.default_rng(8)
    Ns, Nw, K, Kq = 1, 16, 64, 8
    for T in [64 * 512, 64 * 100 + 1, 64 * 64, 64 * 70 + 63, 64 * 20]:
        w = small_workload(batch=2, context=T, k_blocks=K, kq_blocks=Kq, sink_blocks=Ns, window_blocks=Nw, gpu_slots=K)
        p = oracle_params(w)
        sq, se = _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks)
        sel, n_sel = oracle.select(p, sq, se, np.full((w.batch,), T, np.int32))
        N, Nc, forced, cand = _geometry(T, 64, Ns, Nw)
        Ke = K - len(forced) - Kq
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                g = sel[b, h, :n_sel[b, h]]
                assert n_sel[b, h] == min(K, N)
                assert (np.diff(g) > 0).all() and g.min() >= 0 and g.max() < N
                assert set(forced) <= set(g.tolist())
                best_e = sorted(cand, key=lambda J: -se[b, h, J])[:max(Ke, 0)]
                assert set(best_e) <= set(g.tolist())       # b_1..b_ke of the proof of Theorem 1
                top_q = sorted(cand, key=lambda J: -sq[b, h, J])[:Kq]
                assert set(top_q) <= set(g.tolist())        # "query-aware selection is prioritised"


def test_per_batch_token_counts():
    rng = np.random.default_rng(3)
    w = small_workload(batch=3, context=64 * 20, k_blocks=6, kq_blocks=2, gpu_slots=6)
    p = oracle_params(w)
    sq, se = _rand_scores(rng, w.batch, w.n_kv_heads, w.max_blocks)
    n_tok = np.array([64 * 20, 64 * 7 + 3, 100], np.int32)
    sel, n_sel = oracle.select(p, sq, se, n_tok)
    for b in range(3):
        p1 = oracle_params(w.replace(batch=1))
        s1, n1 = oracle.select(p1, sq[b:b + 1], se[b:b + 1], n_tok[b:b + 1])
        assert (s1[0] == sel[b]).all() and (n1[0] == n_sel[b]).all()
        N = -(-int(n_tok[b]) // 64)
        assert sel[b].max() == N - 1                         # the tail block is attended (window)


def test_golden_budget_example():
    """App. B.2: k = 4096, nb = 64 -> 1 sink + 16 window + 16 query-aware + 31 query-agnostic blocks;
    48 of 64 blocks are query-agnostic -> locality >= 75 %."""
    vals = {}
    with open(os.path.join(GOLDEN, "budget_example.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    K = int(vals["k_tokens"] // vals["block_size"])
    Kq = int(vals["kq_tokens"] // vals["block_size"])
    Ns, Nw = int(vals["sink_blocks"]), int(vals["window_blocks"])
    assert K == 64 and Kq == int(vals["query_aware_blocks"])
    assert K - Ns - Nw == int(vals["dynamic_blocks"])
    assert K - Ns - Nw - Kq == int(vals["query_agnostic_dynamic_blocks"])
    assert K - Kq == int(vals["query_agnostic_blocks_total"])
    assert (K - Kq) / K == vals["locality_lower_bound"]
    # and the oracle, run with these budgets, marks exactly that many of each kind
    w = small_workload(batch=1, n_q_heads=1, n_kv_heads=1, context=16384, k_blocks=K, kq_blocks=Kq,
                       sink_blocks=Ns, window_blocks=Nw, gpu_slots=K)
    rng = np.random.default_rng(0)
    sq, se = _rand_scores(rng, 1, 1, w.max_blocks)
    _, n_sel, kind = oracle.select(oracle_params(w), sq, se, np.array([16384], np.int32), with_kind=True)
    assert n_sel[0, 0] == 64
    assert [(kind == c).sum() for c in (0, 1, 2)] == [Ns + Nw, Kq, int(vals["query_agnostic_dynamic_blocks"])]


# ----------------------------------------------------------------------------------- scores

@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_pooled_key_score_equals_pooled_token_scores(dtype):
    """mean_t(q . k_t) == q . mean_t(k_t): Alg. 1 scores pooled keys, the pooling Eq. pools scores."""
    w = small_workload(batch=2, n_q_heads=6, n_kv_heads=2, context=64 * 9 + 20, dtype=dtype)
    layer = make_layer(w, 2, 0)
    q = to_np(QueryStream(w, 2, 0).next(0))
    n_tok = np.full((w.batch,), w.context, np.int32)
    p = oracle_params(w)
    kc, sec = oracle.pool(p, to_np(layer["host_k"]), to_np(layer["host_bias"]), n_tok)
    sq, se, head = oracle.block_score(p, q, kc, sec, n_tok, per_head=True)
    K = widen(to_np(layer["host_k"])).reshape(w.batch, w.n_kv_heads, -1, w.head_dim)
    Bi = to_np(layer["host_bias"]).astype(np.float64).reshape(w.batch, w.n_kv_heads, -1)
    Q = widen(q)
    Nc = w.context // 64
    tol = 1e-5 if dtype == "fp32" else 0.05          # K_c is stored rounded to the cache dtype
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            tok = np.stack([K[b, h] @ Q[b, h * w.group + g] for g in range(w.group)])    # [G, T]
            for J in range(Nc):
                per_head = tok[:, J * 64:(J + 1) * 64].mean(1)
                np.testing.assert_allclose(head[b, h * w.group:(h + 1) * w.group, J], per_head, atol=tol, rtol=0)
                np.testing.assert_allclose(sq[b, h, J], per_head.sum(), atol=tol * w.group, rtol=0)
                np.testing.assert_allclose(se[b, h, J], Bi[b, h, J * 64:(J + 1) * 64].mean(), atol=1e-6, rtol=0)
            assert np.isneginf(sq[b, h, Nc:]).all() and np.isneginf(se[b, h, Nc:]).all()


@pytest.mark.parametrize("lk,ls", [(64, 64), (16, 32), (32, 16), (32, 32), (16, 16), (64, 16)])
def test_two_stage_pooling_geometry(lk, ls):
    """Sub-block j covers tokens [j*ls, j*ls+lk); it counts for block J only if wholly inside it."""
    T = 64 * 7 + 40
    w = small_workload(batch=1, n_q_heads=2, n_kv_heads=1, context=T, pool_kernel=lk, pool_stride=ls, dtype="fp32")
    layer = make_layer(w, 4, 0)
    q = to_np(QueryStream(w, 4, 0).next(0))
    n_tok = np.array([T], np.int32)
    p = oracle_params(w)
    assert p.n_sub_max == (T - lk) // ls + 1
    kc, sec = oracle.pool(p, to_np(layer["host_k"]), to_np(layer["host_bias"]), n_tok)
    sq, se = oracle.block_score(p, q, kc, sec, n_tok)
    K = to_np(layer["host_k"]).astype(np.float64).reshape(-1, w.head_dim)
    Bi = to_np(layer["host_bias"]).astype(np.float64).reshape(-1)
    Q = q.astype(np.float64)[0]
    tok = (K @ Q.T).sum(1)                              # group-summed token scores [T']
    for J in range(w.max_blocks):
        subs = [(j * ls, j * ls + lk) for j in range(10 ** 4)
                if j * ls >= J * 64 and j * ls + lk <= (J + 1) * 64 and j * ls + lk <= T]
        if not subs:
            assert np.isneginf(sq[0, 0, J]) and np.isneginf(se[0, 0, J])
            continue
        np.testing.assert_allclose(sq[0, 0, J], max(tok[a:b].mean() for a, b in subs), atol=1e-4, rtol=0)
        np.testing.assert_allclose(se[0, 0, J], max(Bi[a:b].mean() for a, b in subs), atol=1e-6, rtol=0)


def test_pool_rounds_to_nearest_even_bf16():
    """K_c in bf16 is the correctly rounded mean (checked against torch's fp64 -> bf16 conversion)."""
    import torch
    w = small_workload(batch=1, n_q_heads=1, n_kv_heads=1, context=64 * 4, dtype="bf16")
    layer = make_layer(w, 6, 0)
    p = oracle_params(w)
    kc, _ = oracle.pool(p, to_np(layer["host_k"]), to_np(layer["host_bias"]), np.array([w.context], np.int32))
    ref = layer["host_k"].double().mean(dim=3).to(torch.bfloat16)       # [1,1,4,d]
    assert (kc == to_np(ref)).all()
