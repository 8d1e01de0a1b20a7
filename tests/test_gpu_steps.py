"""Whole decode steps (score -> select -> fetch -> attention) through the C ABI against the
oracle, over several steps with the residency state carried along (needs an MI355X).

Covers the Tiny and the 1B-shaped configuration in full, reduced-batch versions of the 3B- and
8B-shaped ones, the serial (no side stream) order, and poisoned victim slots.
"""
import numpy as np
import pytest
import torch

from nosa_inputs import CONFIGS, random_residency
from pipeline import run_parity

pytestmark = pytest.mark.gpu


def test_tiny_all_steps():
    w = CONFIGS["tiny"]
    rec = run_parity(w, seed=0, steps=w.steps)
    assert rec[0]["n_load_max"] == w.k_blocks                       # cold start fills the pool
    assert max(r["n_load_max"] for r in rec[1:]) <= 2                # <= 2 newly fetched blocks per step
    print("tiny: max err", max(r["err"] for r in rec), "retries", sum(r["retries"] for r in rec), flush=True)


def test_tiny_ragged_context_serial_order():
    w = CONFIGS["tiny"].replace(context=2048 - 37)
    run_parity(w, seed=1, steps=6, overlap=False)


@pytest.mark.parametrize("d,hq,hkv", [(128, 28, 4), (64, 10, 2), (128, 15, 1)])
def test_steps_with_group_sizes_of_seven_five_fifteen(d, hq, hkv):
    """bf16 groups that are no power of two or multiple of three (28 query heads over 4 KV heads is a common layout):
    whole steps with the side-stream fetch, growing context included."""
    from helpers import small_workload
    from pipeline import run_growing
    w = small_workload(batch=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, context=64 * 40 + 11, k_blocks=12, kq_blocks=3,
                       window_blocks=2, gpu_slots=14, dtype="bf16", structure="planted", generated=70)
    run_parity(w, seed=hq, steps=5, overlap=True)
    run_growing(w, hq + 1, 66)


def test_1b_shaped_half_resident():
    """batch 16, 16 q heads / 2 KV heads, d64, 8192 tokens, C = 64 of 128 blocks resident at start."""
    w = CONFIGS["1b"]
    res = random_residency(w, seed=0, layer=0, n_blocks=w.context // w.block_size)
    rec = run_parity(w, seed=0, steps=w.steps, residency=res)
    assert len(rec) == 64
    print("1b: n_load mean per step", [round(r["n_load_mean"], 2) for r in rec], flush=True)


def test_1b_shaped_half_resident_one_stream_single_entry():
    """The same workload in the order bench.py times: everything on one stream."""
    w = CONFIGS["1b"]
    res = random_residency(w, seed=1, layer=0, n_blocks=w.context // w.block_size)
    run_parity(w, seed=1, steps=16, residency=res, overlap=False)


def test_1b_overlap_and_serial_orders_agree():
    """Fetch on the side stream with two-phase attention (resident blocks first, fetched blocks after the
    gather) against everything in call order on one stream: identical selections and miss counts; outputs
    equal up to the summation order of the merge and the rounding of the softmax weights."""
    w = CONFIGS["1b"].replace(batch=4)
    outs = []
    for overlap in (True, False):
        import paper_2510_13602_amd as nosa
        from helpers import gpu_params, to_np
        from nosa_inputs import QueryStream, make_layer
        from paper_2510_13602_amd.runtime import LayerCache, pinned_like
        layer = make_layer(w, 5, 0)
        ctx = nosa.Nosa(gpu_params(w))
        ctx.set_overlap(overlap)
        gl = LayerCache(ctx, pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"]),
                        torch.full((w.batch,), w.context, dtype=torch.int32))
        gl.rebuild_pooled()
        gl.pool_k.fill_(float("nan")); gl.pool_v.fill_(float("nan")); gl.pool_bias.fill_(float("nan"))
        qs = QueryStream(w, 5, 0)
        res = []
        for t in range(8):
            o = gl.step(qs.next(t).to("cuda:0"))
            res.append((to_np(o).copy(), gl.sel_idx.cpu().numpy().copy(), gl.n_load.cpu().numpy().copy()))
        torch.cuda.synchronize()
        outs.append(res)
        ctx.close()
    from helpers import widen
    for (o1, s1, n1), (o2, s2, n2) in zip(*outs):
        assert (s1 == s2).all() and (n1 == n2).all()
        a, b = widen(o1), widen(o2)
        assert np.isfinite(a).all() and np.isfinite(b).all()
        # the matrix-core kernel rounds the softmax weights to bf16 relative to the running maximum of the moment,
        # which differs between the two orders: a few 1e-3 on outputs of size O(1), far inside the oracle's bar
        assert (np.abs(a - b) <= 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + 4e-3).all()


def test_3b_shaped_reduced_batch():
    """24 q heads / 4 KV heads (group 6), d128, 16384 tokens, K = 64, AR(1) queries; batch cut to 2."""
    w = CONFIGS["3b"].replace(batch=2)
    rec = run_parity(w, seed=0, steps=6)
    print("3b: n_load mean per step", [round(r["n_load_mean"], 2) for r in rec], flush=True)


def test_8b_shaped_reduced_batch():
    """32 q heads / 8 KV heads (group 4), d128, 32768 tokens, K = 64, heavy hitters; batch cut to 1."""
    w = CONFIGS["8b"].replace(batch=1)
    rec = run_parity(w, seed=0, steps=5)
    print("8b: n_load mean per step", [round(r["n_load_mean"], 2) for r in rec], flush=True)


def test_long_generation_growing_context():
    """Long-generation 8B-shaped: prompt 4096 (N = 64 = K, the first step is dense), then tokens are
    appended one per step; 200 steps cross three block boundaries.  Batch cut to 2 for the oracle."""
    from pipeline import run_growing
    w = CONFIGS["longgen"].replace(batch=2, generated=200)
    r = run_growing(w, seed=0, steps=200)
    print("longgen: worst err", r["worst"], "n_load max at block boundaries", r["boundary_loads"], flush=True)
    assert len(r["boundary_loads"]) == 4 and max(r["boundary_loads"][1:]) <= w.kq_blocks   # step 0 (cold) + 3 boundaries


def test_long_generation_full_length():
    """The whole long-generation run: prompt 4096, then all 16384 generated tokens (N grows from 64 to 320
    blocks over 256 block boundaries), batch cut to 4 (32 units).  Token counts, Gamma, miss counts, load lists and
    both maps are compared with the oracle at every one of the 16385 steps and n_load <= Kq is asserted
    throughout; pooled arrays and attention outputs at steps 0-8, around each of the first 8 block
    boundaries, at 64 seeded random steps and at the last 16; host pool, GPU pool and pooled arrays at the end."""
    from pipeline import run_growing
    w = CONFIGS["longgen"].replace(batch=4)
    steps = w.generated + 1
    att = set(range(9)) | set(range(steps - 16, steps))
    for k in range(1, 9):                                    # token that opens block 64 + k - 1 is step 64 k
        att |= {64 * k - 1, 64 * k, 64 * k + 1}
    att |= set(np.random.default_rng(2024).integers(9, steps - 16, 64).tolist())
    r = run_growing(w, seed=0, steps=steps, attention_steps=att, progress=1024)
    print("longgen full: worst err", r["worst"], "attention checks", r["checked"], "boundaries", len(r["boundary_loads"]),
          "max n_load at a boundary", max(r["boundary_loads"][1:]), flush=True)
    assert len(r["boundary_loads"]) == 257 and max(r["boundary_loads"][1:]) <= w.kq_blocks
    assert r["checked"] == len(att)


def test_growing_context_small_ragged_fp32():
    """fp32, d64, group 4, K = 8, starting mid-block, two-stage pooling with several sub-blocks per block."""
    from pipeline import run_growing
    w = CONFIGS["tiny"].replace(context=64 * 20 + 50, generated=150, pool_kernel=32, pool_stride=16, batch=2)
    run_growing(w, seed=3, steps=150)


def _two_layers(w, seed, stream=None):
    import paper_2510_13602_amd as nosa
    from helpers import gpu_params
    from nosa_inputs import make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    layer = make_layer(w, seed, 0)
    ctx = nosa.Nosa(gpu_params(w), stream=stream)
    ctx.set_overlap(True)      # the two-launch order with the side-stream gather, whatever the shape's default
    hk, hv, hb = pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"])
    n_tok = torch.full((w.batch,), w.context, dtype=torch.int32)
    a, b = LayerCache(ctx, hk, hv, hb, n_tok), LayerCache(ctx, hk, hv, hb, n_tok)
    a.rebuild_pooled()
    b.rebuild_pooled()
    return ctx, a, b


def test_single_entry_step_equals_four_calls():
    from helpers import to_np
    from nosa_inputs import QueryStream
    w = CONFIGS["1b"].replace(batch=4)
    ctx, a, b = _two_layers(w, 7)
    qs = QueryStream(w, 7, 0)
    for t in range(6):
        q = qs.next(t).to("cuda:0")
        oa = a.step(q)
        ob = b.step_fused(q)
        torch.cuda.synchronize()
        assert to_np(oa).tobytes() == to_np(ob).tobytes()
        assert (a.sel_idx == b.sel_idx).all() and (a.n_load == b.n_load).all() and (a.slot_of_block == b.slot_of_block).all()
    ctx.close()


@pytest.mark.parametrize("name,over", [
    ("1b", dict(batch=3)),                                                        # d64, group 8, C = 64 > K = 32
    ("1b", dict(batch=2, victim_policy=1, gpu_slots=80)),                         # ranked victims, C = 80 of 128 blocks
    ("tiny", dict(batch=2, n_q_heads=8, n_kv_heads=2)),                           # fp32
    ("3b", dict(batch=1, context=64 * 1000 + 11, gpu_slots=70)),                  # 1001 blocks: 16 keys per lane, ragged tail
    ("8b", dict(batch=1, context=64 * 300)),
])
def test_fused_stage1_equals_score_then_select(name, over):
    """nosa_decode_step with scores + selection + load positions in ONE kernel against the separate
    nosa_block_score and nosa_select kernels, on twin state over several steps: scores (when asked for),
    Gamma, load lists, maps and outputs bit for bit; and with sq_blk / se_blk = NULL the rest is unchanged."""
    from helpers import to_np
    from nosa_inputs import QueryStream
    w = CONFIGS[name].replace(**over)
    ctx, a, b = _two_layers(w, 13)
    import paper_2510_13602_amd as nosa
    from paper_2510_13602_amd.runtime import LayerCache
    c = LayerCache(ctx, a.host_k, a.host_v, a.host_bias, a.n_tokens.cpu())
    c.rebuild_pooled()
    c.keep_scores = False
    c.sq_blk.fill_(7.0)
    qs = QueryStream(w, 13, 0)
    for t in range(5):
        q = qs.next(t).to("cuda:0")
        ctx.set_fused_select(False)
        oa = a.step_fused(q).clone()                 # separate kernels behind the single entry
        ctx.set_fused_select(True)
        ob = b.step_fused(q).clone()                 # one kernel, scores written out as well
        oc = c.step_fused(q).clone()                 # one kernel, scores stay on chip
        torch.cuda.synchronize()
        for x in (b, c):
            assert (a.sel_idx == x.sel_idx).all() and (a.n_sel == x.n_sel).all(), f"step {t}: selections differ"
            assert (a.n_load == x.n_load).all() and (a.load_list == x.load_list).all()
            assert (a.slot_of_block == x.slot_of_block).all() and (a.block_of_slot == x.block_of_slot).all()
        assert to_np(a.sq_blk).tobytes() == to_np(b.sq_blk).tobytes() and to_np(a.se_blk).tobytes() == to_np(b.se_blk).tobytes()
        assert (c.sq_blk == 7.0).all()                                   # untouched
        assert to_np(oa).tobytes() == to_np(ob).tobytes() == to_np(oc).tobytes()
    ctx.close()


def test_fused_stage1_degenerate_token_counts():
    """Empty caches, a single token, exactly one block, the table's capacity -- per batch element -- through
    the fused kernel against the separate kernels."""
    import paper_2510_13602_amd as nosa
    from helpers import gpu_params
    from nosa_inputs import QueryStream, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    tokens = [0, 1, 64, 65, 700, 768]
    w = CONFIGS["tiny"].replace(batch=len(tokens), n_q_heads=8, n_kv_heads=2, context=768, k_blocks=6, kq_blocks=2,
                                sink_blocks=1, window_blocks=1, gpu_slots=7, dtype="bf16", head_dim=128)
    layer = make_layer(w, 12, 0)
    ctx = nosa.Nosa(gpu_params(w))
    ctx.set_overlap(True)
    hk, hv, hb = pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"])
    n_tok = torch.tensor(tokens, dtype=torch.int32)
    a, b = LayerCache(ctx, hk, hv, hb, n_tok), LayerCache(ctx, hk, hv, hb, n_tok)
    a.rebuild_pooled(); b.rebuild_pooled()
    qs = QueryStream(w, 12, 0)
    for t in range(3):
        q = qs.next(t).to("cuda:0")
        ctx.set_fused_select(False)
        oa = a.step_fused(q).clone()
        ctx.set_fused_select(True)
        ob = b.step_fused(q).clone()
        torch.cuda.synchronize()
        assert (a.sel_idx == b.sel_idx).all() and (a.n_sel == b.n_sel).all() and (a.load_list == b.load_list).all()
        assert (a.sq_blk == b.sq_blk).all() and (a.se_blk == b.se_blk).all()
        assert (oa == ob).all()
    ctx.close()


def test_graph_replays_match_eager_steps():
    """The step recorded into a HIP graph, replayed 8 times with the program's own eager work and
    synchronisations between the replays; every replay must equal the eager step on twin state."""
    from helpers import to_np
    from nosa_inputs import QueryStream
    w = CONFIGS["1b"].replace(batch=4)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ctx, a, b = _two_layers(w, 9, stream=s)
        qs = QueryStream(w, 9, 0)
        q_static = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=w.torch_dtype, device="cuda:0")
        s.synchronize()
        b.capture(q_static)
        s.synchronize()
        # the capture itself launches nothing: state is still the initial one
        assert (b.slot_of_block == -1).all()
        scratch = torch.randn(1 << 20, device="cuda:0")
        for t in range(8):
            q = qs.next(t).to("cuda:0")
            q_static.copy_(q)
            oa = a.step(q)
            ob = b.replay()
            s.synchronize()
            assert (a.sel_idx == b.sel_idx).all(), f"replay {t}: selections differ"
            assert (a.n_load == b.n_load).all() and (a.load_list == b.load_list).all()
            assert (a.slot_of_block == b.slot_of_block).all() and (a.block_of_slot == b.block_of_slot).all()
            assert to_np(oa).tobytes() == to_np(ob).tobytes(), f"replay {t}: outputs differ"
            assert to_np(a.pool_k).tobytes() == to_np(b.pool_k).tobytes()
            scratch = (scratch * 1.0001 + 1.0).sort().values          # unrelated eager work between replays
            float(scratch.sum().item())
        b.release_graph()
        ctx.close()


def test_graph_of_a_generation_step_replays_like_eager():
    """The whole step of a growing context (QKV split + eviction head, append, score / select / fetch /
    attention) recorded into one HIP graph and replayed 140 times -- two block boundaries, eager work and
    synchronisations between the replays -- against the same calls made eagerly on twin state: token
    counts, selections, load lists, maps, appended keys / values / biases, pooled arrays and outputs bit
    for bit at every step, host pools at the end."""
    import paper_2510_13602_amd as nosa
    from helpers import gpu_params, to_np
    from nosa_inputs import QueryStream, append_token, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    w = CONFIGS["longgen"].replace(batch=2, generated=150)
    dev = "cuda:0"
    B, Hq, H, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        layer = make_layer(w, 31, 0)
        ctx = nosa.Nosa(gpu_params(w), stream=s)
        ctx.set_overlap(True)
        n_tok = torch.full((B,), w.context, dtype=torch.int32)
        twins = []
        for _ in range(2):                        # each twin appends into its own host pool
            lc = LayerCache(ctx, pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"]), n_tok)
            lc.rebuild_pooled()
            twins.append(lc)
        a, b = twins
        g = torch.Generator().manual_seed(5)
        w1 = (torch.randn((d, H), generator=g) / d ** 0.5).to(dev)
        w2 = torch.randn((H,), generator=g).to(dev)
        td = w.torch_dtype
        bufs = [dict(q=torch.empty((B, Hq, d), dtype=td, device=dev), k=torch.empty((B, H, d), dtype=td, device=dev),
                     v=torch.empty((B, H, d), dtype=td, device=dev), b=torch.empty((B, H), dtype=torch.float32, device=dev))
                for _ in range(2)]
        qkv_static = torch.zeros((B, (Hq + 2 * H) * d), dtype=td, device=dev)
        qs = QueryStream(w, 31, 0)
        q0 = qs.next(0).to(dev)
        a.step_fused(q0)                         # step 0: the prompt's last token is already in the cache
        b.step_fused(q0)
        s.synchronize()
        b.capture_generation(qkv_static, w1, w2, 0, bufs[1]["q"], bufs[1]["k"], bufs[1]["v"], bufs[1]["b"])
        s.synchronize()
        assert (a.n_tokens == b.n_tokens).all()           # recording launched nothing
        scratch = torch.randn(1 << 18, device=dev)
        for t in range(1, 141):
            tok = append_token(w, 31, 0, t)
            qkv = torch.cat([qs.next(t).reshape(B, Hq * d), tok["k_new"].reshape(B, H * d), tok["v_new"].reshape(B, H * d)], dim=1).to(dev)
            ctx.nosa_split_qkv_evict(qkv, w1, w2, 0, bufs[0]["q"], bufs[0]["k"], bufs[0]["v"], bufs[0]["b"])
            a.append(bufs[0]["k"], bufs[0]["v"], bufs[0]["b"])
            oa = a.step_fused(bufs[0]["q"])
            qkv_static.copy_(qkv)
            ob = b.replay()
            s.synchronize()
            assert (a.n_tokens == b.n_tokens).all() and int(a.n_tokens[0]) == w.context + t, f"step {t}: token counts"
            for key in ("q", "k", "v", "b"):
                assert to_np(bufs[0][key]).tobytes() == to_np(bufs[1][key]).tobytes(), f"step {t}: {key} differs"
            assert (a.sel_idx == b.sel_idx).all(), f"replay {t}: selections differ"
            assert (a.n_load == b.n_load).all() and (a.load_list == b.load_list).all()
            assert (a.slot_of_block == b.slot_of_block).all() and (a.block_of_slot == b.block_of_slot).all()
            assert to_np(oa).tobytes() == to_np(ob).tobytes(), f"replay {t}: outputs differ"
            if (w.context + t) % 64 in (0, 1, 63):
                assert to_np(a.k_pooled).tobytes() == to_np(b.k_pooled).tobytes()
                assert to_np(a.se_pooled).tobytes() == to_np(b.se_pooled).tobytes()
                assert to_np(a.pool_k).tobytes() == to_np(b.pool_k).tobytes()
            scratch = (scratch * 1.0001 + 1.0).sort().values          # unrelated eager work between replays
            float(scratch.sum().item())
        assert to_np(a.host_k).tobytes() == to_np(b.host_k).tobytes() and to_np(a.host_v).tobytes() == to_np(b.host_v).tobytes()
        assert to_np(a.host_bias).tobytes() == to_np(b.host_bias).tobytes()
        assert int(a.n_tokens[0]) == w.context + 140
        b.release_graph()
        ctx.close()


def test_1b_shaped_importance_ranked_victims():
    """C = 64 slots for K = 32 selected blocks: with victim_policy 1 a miss overwrites the least important
    non-selected block instead of the first free slot.  Parity with the oracle at every step, and fewer
    misses than the slot-order policy on the same inputs."""
    w0 = CONFIGS["1b"].replace(batch=4)
    w1 = w0.replace(victim_policy=1)
    res = random_residency(w0, seed=0, layer=0, n_blocks=w0.context // w0.block_size)
    r0 = run_parity(w0, seed=2, steps=16, residency=res)
    r1 = run_parity(w1, seed=2, steps=16, residency=res)
    m0 = sum(r["n_load_mean"] for r in r0[4:]) / len(r0[4:])
    m1 = sum(r["n_load_mean"] for r in r1[4:]) / len(r1[4:])
    print(f"1b, C=64: mean misses per unit and step, slot order {m0:.2f}, importance ranked {m1:.2f}", flush=True)
    assert m1 < m0


@pytest.mark.parametrize("K,Kq,Ns,Nw,tokens", [(6, 2, 1, 1, [0, 1, 64, 65, 700, 768]), (1, 0, 0, 1, [1, 63, 64, 130, 500, 768]),
                                               (4, 1, 0, 2, [0, 0, 2, 128, 129, 767])])
def test_degenerate_token_counts_per_batch_element(K, Kq, Ns, Nw, tokens):
    """Empty caches, a single token, exactly one block, one token into the next block, and the
    table's capacity, all in one batch; K = 1 keeps only the tail block.  Whole step against the oracle."""
    import oracle
    import paper_2510_13602_amd as nosa
    from helpers import gpu_params, oracle_params, out_tol, to_np
    from nosa_inputs import QueryStream, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    w = CONFIGS["tiny"].replace(batch=len(tokens), n_q_heads=8, n_kv_heads=2, context=768, k_blocks=K, kq_blocks=Kq,
                                sink_blocks=Ns, window_blocks=Nw, gpu_slots=K + 1, dtype="bf16", head_dim=128)
    layer = make_layer(w, 11, 0)
    n_tok = np.array(tokens, np.int32)
    po = oracle_params(w)
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    kc, sec = oracle.pool(po, hk, hb, n_tok)
    B, H, C, nb, d = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim
    pk, pv = np.zeros((B, H, C, nb, d), hk.dtype), np.zeros((B, H, C, nb, d), hv.dtype)
    pb = np.zeros((B, H, C, nb), np.float32)
    sob, bos = np.full((B, H, w.max_blocks), -1, np.int32), np.full((B, H, C), -1, np.int32)
    ctx = nosa.Nosa(gpu_params(w))
    ctx.set_overlap(True)
    gl = LayerCache(ctx, pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"]),
                    torch.from_numpy(n_tok))
    gl.rebuild_pooled()
    torch.cuda.synchronize()
    assert to_np(gl.k_pooled).tobytes() == kc.tobytes()
    gl.pool_k.fill_(float("nan")); gl.pool_v.fill_(float("nan")); gl.pool_bias.fill_(float("nan"))
    qs = QueryStream(w, 11, 0)
    for t in range(4):
        q = qs.next(t)
        sq, se = oracle.block_score(po, to_np(q), kc, sec, n_tok)
        sel, n_sel = oracle.select(po, sq, se, n_tok)
        ll, n_load = oracle.load(po, sel, n_sel, sob, bos)
        oracle.fetch(po, hk, hv, hb, pk, pv, pb, ll, n_load)
        ref, ref_lse = oracle.attention(po, to_np(q), pk, pv, pb, sel, n_sel, sob, n_tok)
        out = gl.step(q.to("cuda:0"))
        torch.cuda.synchronize()
        assert (gl.sel_idx.cpu().numpy() == sel).all() and (gl.n_sel.cpu().numpy() == n_sel).all()
        assert (gl.n_load.cpu().numpy() == n_load).all() and (gl.load_list.cpu().numpy() == ll).all()
        got = out.double().cpu().numpy()
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= out_tol(w.dtype)
        for b, T in enumerate(tokens):
            if T == 0:
                assert (got[b] == 0).all() and (n_sel[b] == 0).all()         # nothing to attend: zero rows
                assert np.isneginf(gl.lse[b].cpu().numpy()).all()
    ctx.close()
