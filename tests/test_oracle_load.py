"""Pins for the oracle's residency / fetch model (Sec. 4 "Memory Layout and Block Selection").

 - Theorem 1 (Sec. 3.1, proof in App. E): with the GPU holding exactly the previous selection
   (C = K), every step after the first loads at most Kq blocks, i.e. locality >= (K - Kq) / K;
   the paper's instance is 48 / 64 = 75 %.
 - after a step every selected block has a slot, no slot is booked twice, the two maps are
   inverse to each other, and each selected slot holds the host copy of its block byte for byte;
 - the load list is exactly the set difference Gamma(t) \\ resident(t-1), computed here with
   Python sets;
 - whole-step check: scores -> selection -> load -> fetch -> attention through the pool equals
   brute-force attention over the host cache restricted to Gamma.
"""
import numpy as np
import pytest

import oracle
from helpers import oracle_params, small_workload, to_np, widen
from nosa_inputs import CONFIGS, QueryStream, make_layer, random_residency


def _check_maps(p, sob, bos, sel, n_sel):
    for b in range(p.batch):
        for h in range(p.n_kv_heads):
            used = bos[b, h][bos[b, h] >= 0]
            assert len(set(used.tolist())) == len(used)                    # no block in two slots
            for s, J in enumerate(bos[b, h]):
                if J >= 0:
                    assert sob[b, h, J] == s
            for J in np.nonzero(sob[b, h] >= 0)[0]:
                assert bos[b, h, sob[b, h, J]] == J
            for J in sel[b, h, :n_sel[b, h]]:
                assert sob[b, h, J] >= 0                                   # every selected block resident


@pytest.mark.parametrize("K,Kq,Ns,Nw,C,N", [(64, 16, 1, 16, 64, 256), (64, 8, 1, 16, 64, 512), (8, 2, 1, 1, 8, 32),
                                            (32, 8, 1, 8, 64, 128), (16, 0, 1, 3, 16, 40)])
def test_theorem1_locality_bound_over_steps(K, Kq, Ns, Nw, C, N):
    rng = np.random.default_rng(K * 1000 + Kq)
    T = 64 * N
    w = small_workload(batch=2, context=T, k_blocks=K, kq_blocks=Kq, sink_blocks=Ns, window_blocks=Nw, gpu_slots=C)
    p = oracle_params(w)
    n_tok = np.full((w.batch,), T, np.int32)
    se = rng.standard_normal((w.batch, w.n_kv_heads, N))
    sob = np.full((w.batch, w.n_kv_heads, N), -1, np.int32)
    bos = np.full((w.batch, w.n_kv_heads, C), -1, np.int32)
    prev = None
    for t in range(12):
        sq = rng.standard_normal((w.batch, w.n_kv_heads, N)) * 3          # adversarial: fresh query every step
        sel, n_sel = oracle.select(p, sq, se, n_tok)
        resident_before = [[set(np.nonzero(sob[b, h] >= 0)[0].tolist()) for h in range(w.n_kv_heads)]
                           for b in range(w.batch)]
        ll, n_load = oracle.load(p, sel, n_sel, sob, bos)
        _check_maps(p, sob, bos, sel, n_sel)
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                gamma = set(sel[b, h, :n_sel[b, h]].tolist())
                miss = sorted(gamma - resident_before[b][h])
                assert ll[b, h, :n_load[b, h], 0].tolist() == miss         # the set difference, ascending
                assert (ll[b, h, n_load[b, h]:] == -1).all()
                slots = ll[b, h, :n_load[b, h], 1]
                assert len(set(slots.tolist())) == len(slots)
                if t == 0:
                    assert n_load[b, h] == K                               # cold start
                elif C == K:
                    assert n_load[b, h] <= Kq                              # Theorem 1
                    g_prev = set(prev[b, h].tolist())
                    assert len(gamma & g_prev) / len(gamma) >= (K - Kq) / K
        prev = sel.copy()
    if (K, Kq) == (64, 16):
        assert (K - Kq) / K == 0.75                                        # the paper's 48/64 instance


def test_full_step_through_pool_equals_bruteforce_on_host_cache():
    w = CONFIGS["tiny"].replace(context=64 * 24 + 30, steps=5)
    p = oracle_params(w)
    seed = 13
    layer = make_layer(w, seed, 0)
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    n_tok = np.full((w.batch,), w.context, np.int32)
    kc, sec = oracle.pool(p, hk, hb, n_tok)
    B, H, C, nb, d = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim
    pk = np.full((B, H, C, nb, d), np.nan, hk.dtype)
    pv = np.full((B, H, C, nb, d), np.nan, hv.dtype)
    pb = np.full((B, H, C, nb), np.nan, np.float32)
    sob = np.full((B, H, w.max_blocks), -1, np.int32)
    bos = np.full((B, H, C), -1, np.int32)
    qs = QueryStream(w, seed, 0)
    Kd, Vd = widen(hk).reshape(B, H, -1, d), widen(hv).reshape(B, H, -1, d)
    Bd = hb.astype(np.float64).reshape(B, H, -1)
    for t in range(w.steps):
        q = to_np(qs.next(t))
        sq, se = oracle.block_score(p, q, kc, sec, n_tok)
        sel, n_sel = oracle.select(p, sq, se, n_tok)
        ll, n_load = oracle.load(p, sel, n_sel, sob, bos)
        if t > 0:
            assert (n_load <= w.kq_blocks).all()
        oracle.fetch(p, hk, hv, hb, pk, pv, pb, ll, n_load)
        for b in range(B):
            for h in range(H):
                for J in sel[b, h, :n_sel[b, h]]:
                    s = sob[b, h, J]
                    assert pk[b, h, s].tobytes() == hk[b, h, J].tobytes()
                    assert pv[b, h, s].tobytes() == hv[b, h, J].tobytes()
                    assert pb[b, h, s].tobytes() == hb[b, h, J].tobytes()
        out, _ = oracle.attention(p, q, pk, pv, pb, sel, n_sel, sob, n_tok)
        Q = widen(q)
        for b in range(B):
            for hq in range(w.n_q_heads):
                h = hq // w.group
                mask = np.full(Kd.shape[2], -np.inf)
                for J in sel[b, h, :n_sel[b, h]]:
                    mask[J * nb:(J + 1) * nb] = 0
                mask[w.context:] = -np.inf
                z = p.softmax_scale * (Kd[b, h] @ Q[b, hq]) + Bd[b, h] + mask
                pr = np.exp(z - z.max())
                pr /= pr.sum()
                np.testing.assert_allclose(out[b, hq], pr @ Vd[b, h], rtol=0, atol=1e-12)


def test_planted_blocks_are_picked_query_aware_on_tiny():
    """The tiny workload plants 3 high-similarity blocks; with Kq = 2 the query-aware picks are
    two of them at every step (clear margin), and the fetch budget of 2 blocks per step holds."""
    w = CONFIGS["tiny"]
    p = oracle_params(w)
    layer = make_layer(w, 0, 0)
    hk, hb = to_np(layer["host_k"]), to_np(layer["host_bias"])
    n_tok = np.full((w.batch,), w.context, np.int32)
    kc, sec = oracle.pool(p, hk, hb, n_tok)
    planted = set(layer["planted"][0, 0].tolist())
    qs = QueryStream(w, 0, 0)
    sob, bos = random_residency(w, 0, 0, w.max_blocks)
    sob, bos = sob.numpy(), bos.numpy()
    for t in range(w.steps):
        q = to_np(qs.next(t))
        sq, se = oracle.block_score(p, q, kc, sec, n_tok)
        sel, n_sel, kind = oracle.select(p, sq, se, n_tok, with_kind=True)
        picks = set(sel[0, 0][kind[0, 0] == 1].tolist())
        assert len(picks) == 2 and picks <= planted
        order = np.sort(sq[0, 0, 1:31])[::-1]
        assert order[1] - order[3] > 1.0                      # planted vs the rest: wide margin
        _, n_load = oracle.load(p, sel, n_sel, sob, bos)
        if t > 0:
            assert n_load[0, 0] <= 2


def test_importance_ranked_victims_against_brute_force():
    """victim_policy 1 (C > K): the slots overwritten are the empty ones first, then the free slots whose
    block has the smallest block-level importance; the misses themselves are the same set difference."""
    rng = np.random.default_rng(77)
    K, Kq, Ns, Nw, C, N = 16, 4, 1, 3, 40, 90
    T = 64 * N
    w = small_workload(batch=3, context=T, k_blocks=K, kq_blocks=Kq, sink_blocks=Ns, window_blocks=Nw, gpu_slots=C,
                       victim_policy=1)
    p = oracle_params(w)
    n_tok = np.full((w.batch,), T, np.int32)
    se = rng.standard_normal((w.batch, w.n_kv_heads, N))
    sob = np.full((w.batch, w.n_kv_heads, N), -1, np.int32)
    bos = np.full((w.batch, w.n_kv_heads, C), -1, np.int32)
    for t in range(10):
        sq = rng.standard_normal((w.batch, w.n_kv_heads, N)) * 3
        sel, n_sel = oracle.select(p, sq, se, n_tok)
        before_sob, before_bos = sob.copy(), bos.copy()
        ll, n_load = oracle.load(p, sel, n_sel, sob, bos, se, n_tok)
        _check_maps(p, sob, bos, sel, n_sel)
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                gamma = set(sel[b, h, :n_sel[b, h]].tolist())
                resident = set(np.nonzero(before_sob[b, h] >= 0)[0].tolist())
                miss = sorted(gamma - resident)
                assert ll[b, h, :n_load[b, h], 0].tolist() == miss
                free = [s for s in range(C) if before_bos[b, h, s] < 0 or before_bos[b, h, s] not in gamma]
                rank = sorted(free, key=lambda s: (0, 0.0, s) if before_bos[b, h, s] < 0
                              else (1, se[b, h, before_bos[b, h, s]], s))
                want = sorted(rank[:len(miss)])
                assert ll[b, h, :n_load[b, h], 1].tolist() == want


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_token_fetch_is_a_row_gather(dtype):
    """Element-wise transfer (Sec. 3.2 "Comparison with DMA"): copying listed token rows is, by definition, a
    gather/scatter of rows, which numpy's fancy indexing states in one line per tensor.  Lists of every length
    from empty to the whole pool, distinct destinations; rows not listed must keep their old bytes; entries
    beyond n_list must be ignored."""
    rng = np.random.default_rng(5 if dtype == "bf16" else 6)
    w = small_workload(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, context=64 * 9, k_blocks=4, kq_blocks=1,
                       gpu_slots=5, dtype=dtype)
    p = oracle_params(w)
    layer = make_layer(w, 31, 0)
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    B, H, C, nb, d, N = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim, w.max_blocks
    M = C * nb
    lengths = np.array([[0, M], [1, 77]], np.int32)                 # empty, full, one row, ragged
    tl = np.full((B, H, M, 2), -1, np.int32)
    for b in range(B):
        for h in range(H):
            n = lengths[b, h]
            tl[b, h, :n, 0] = rng.choice(N * nb, n, replace=False)
            tl[b, h, :n, 1] = rng.choice(C * nb, n, replace=False)
            tl[b, h, n:, 0] = rng.integers(0, N * nb, M - n)         # junk beyond the list length
            tl[b, h, n:, 1] = rng.integers(0, C * nb, M - n)
    old_k = rng.integers(0, 2 ** 16, (B, H, C, nb, d)).astype(hk.dtype) if hk.dtype == np.uint16 \
        else rng.standard_normal((B, H, C, nb, d)).astype(np.float32)
    old_v = old_k[..., ::-1].copy()
    old_b = rng.standard_normal((B, H, C, nb)).astype(np.float32)
    pk, pv, pb = old_k.copy(), old_v.copy(), old_b.copy()
    oracle.fetch_tokens(p, hk, hv, hb, pk, pv, pb, tl, lengths)
    for b in range(B):
        for h in range(H):
            n = lengths[b, h]
            src, dst = tl[b, h, :n, 0], tl[b, h, :n, 1]
            want_k, want_v, want_b = old_k[b, h].reshape(M, d).copy(), old_v[b, h].reshape(M, d).copy(), old_b[b, h].reshape(M).copy()
            want_k[dst] = hk[b, h].reshape(N * nb, d)[src]
            want_v[dst] = hv[b, h].reshape(N * nb, d)[src]
            want_b[dst] = hb[b, h].reshape(N * nb)[src]
            assert pk[b, h].reshape(M, d).tobytes() == want_k.tobytes()
            assert pv[b, h].reshape(M, d).tobytes() == want_v.tobytes()
            assert pb[b, h].reshape(M).tobytes() == want_b.tobytes()
    # bias pointers may be absent: keys and values still move, the bias pool is left alone
    pk2, pv2 = old_k.copy(), old_v.copy()
    oracle.fetch_tokens(p, hk, hv, None, pk2, pv2, None, tl, lengths)
    assert pk2.tobytes() == pk.tobytes() and pv2.tobytes() == pv.tobytes()


def test_token_fetch_of_whole_blocks_equals_block_fetch():
    """A block-wise load list expanded into its 64 token rows must give the same pool as the block-wise fetch."""
    rng = np.random.default_rng(9)
    w = small_workload(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, context=64 * 12, k_blocks=6, kq_blocks=2,
                       gpu_slots=6, dtype="bf16")
    p = oracle_params(w)
    layer = make_layer(w, 32, 0)
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    B, H, C, nb, d, K = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim, w.k_blocks
    ll = np.full((B, H, K, 2), -1, np.int32)
    n_load = rng.integers(0, K + 1, (B, H)).astype(np.int32)
    tl = np.full((B, H, K * nb, 2), -1, np.int32)
    for b in range(B):
        for h in range(H):
            n = n_load[b, h]
            ll[b, h, :n, 0] = np.sort(rng.choice(w.max_blocks, n, replace=False))
            ll[b, h, :n, 1] = rng.choice(C, n, replace=False)
            for i in range(n):
                tl[b, h, i * nb:(i + 1) * nb, 0] = ll[b, h, i, 0] * nb + np.arange(nb)
                tl[b, h, i * nb:(i + 1) * nb, 1] = ll[b, h, i, 1] * nb + np.arange(nb)
    pools = []
    for mode in ("block", "token"):
        pk, pv = np.zeros((B, H, C, nb, d), hk.dtype), np.zeros((B, H, C, nb, d), hv.dtype)
        pb = np.zeros((B, H, C, nb), np.float32)
        if mode == "block":
            oracle.fetch(p, hk, hv, hb, pk, pv, pb, ll, n_load)
        else:
            oracle.fetch_tokens(p, hk, hv, hb, pk, pv, pb, tl, (n_load * nb).astype(np.int32))
        pools.append((pk, pv, pb))
    for x, y in zip(*pools):
        assert x.tobytes() == y.tobytes()
