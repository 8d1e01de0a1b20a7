"""Runs the same decode steps through the oracle (CPU, fp64) and through libnosa (GPU) on the
same seeded inputs, and compares them.  Test plumbing: no arithmetic of the method lives here.

Margin rule: selection indices must match bit-exactly, so a query whose Kq-th and (Kq+1)-th
query-aware candidate scores are closer than ``margin`` (fp64 oracle scores) is redrawn for that
unit with the next retry counter before either side sees it.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from helpers import from_np, gpu_params, oracle_params, out_tol, to_np
from nosa_inputs import QueryStream, Workload, make_layer


class OracleLayer:
    """Oracle-side state of one layer: host cache, pooled arrays, pool, maps."""

    def __init__(self, w: Workload, host_k, host_v, host_bias, n_tokens: np.ndarray):
        self.w, self.p = w, oracle_params(w)
        self.hk, self.hv, self.hb = host_k, host_v, host_bias
        self.n_tok = n_tokens.astype(np.int32)
        B, H, C, nb, d = w.batch, w.n_kv_heads, w.gpu_slots, w.block_size, w.head_dim
        self.pk = np.zeros((B, H, C, nb, d), host_k.dtype)
        self.pv = np.zeros((B, H, C, nb, d), host_v.dtype)
        self.pb = np.zeros((B, H, C, nb), np.float32)
        self.sob = np.full((B, H, w.max_blocks), -1, np.int32)
        self.bos = np.full((B, H, C), -1, np.int32)
        self.kc, self.sec = oracle.pool(self.p, self.hk, self.hb, self.n_tok)

    def scores(self, q: np.ndarray):
        return oracle.block_score(self.p, q, self.kc, self.sec, self.n_tok)

    def step(self, q: np.ndarray, attention: bool = True):
        sq, se = self.scores(q)
        sel, n_sel = oracle.select(self.p, sq, se, self.n_tok)
        ll, n_load = oracle.load(self.p, sel, n_sel, self.sob, self.bos, se, self.n_tok)
        oracle.fetch(self.p, self.hk, self.hv, self.hb, self.pk, self.pv, self.pb, ll, n_load)
        out = lse = None
        if attention:
            out, lse = oracle.attention(self.p, q, self.pk, self.pv, self.pb, sel, n_sel, self.sob, self.n_tok)
        return dict(sq=sq, se=se, sel=sel, n_sel=n_sel, load_list=ll, n_load=n_load, out=out, lse=lse)


def query_margin(w: Workload, sq: np.ndarray, n_tok: np.ndarray) -> np.ndarray:
    """Gap between the Kq-th and (Kq+1)-th best query-aware candidate score per unit [B, Hkv]."""
    B, H = sq.shape[:2]
    gap = np.full((B, H), np.inf)
    for b in range(B):
        T = int(n_tok[b])
        N, Nc = -(-T // w.block_size), T // w.block_size
        lo, hi = w.sink_blocks, min(Nc, N - w.window_blocks)
        if hi - lo <= w.kq_blocks or w.kq_blocks == 0:
            continue
        for h in range(H):
            s = np.sort(sq[b, h, lo:hi])[::-1]
            gap[b, h] = s[w.kq_blocks - 1] - s[w.kq_blocks]
    return gap


def draw_with_margin(w: Workload, qs: QueryStream, ol: OracleLayer, step: int, margin: float = 1e-3, max_retry: int = 8):
    """Next query of the stream, with units redrawn until the selection margin holds."""
    d = qs.draw(step, 0)
    retries = 0
    for r in range(1, max_retry + 1):
        q = to_np(d["q32"].to(w.torch_dtype))
        gap = query_margin(w, ol.scores(q)[0], ol.n_tok)
        bad = np.argwhere(gap < margin)
        if len(bad) == 0:
            break
        retries += len(bad)
        alt = qs.draw(step, r)
        G = w.group
        for b, h in bad:
            for key in ("q32", "x", "m"):
                if d[key] is not None:
                    d[key][b, h * G:(h + 1) * G] = alt[key][b, h * G:(h + 1) * G]
    else:
        raise AssertionError("selection margin not reached")
    return qs.commit(d), retries


def run_parity(w: Workload, seed: int, steps: int, device="cuda:0", overlap=True, check_attention=True,
               residency=None, poison=True, margin=1e-3, layer_index=0, n_tokens=None):
    """Drives ``steps`` decode steps of one layer through both sides; asserts parity at each step.

    ``n_tokens`` [B] gives every batch element its own token count (default: ``w.context`` for all).
    Returns per-step records (n_load, retries, max abs error)."""
    import paper_2510_13602_amd as nosa
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like

    layer = make_layer(w, seed, layer_index)
    n_tok = np.full((w.batch,), w.context, np.int32) if n_tokens is None else np.asarray(n_tokens, np.int32)
    ol = OracleLayer(w, to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"]), n_tok)
    ctx = nosa.Nosa(gpu_params(w), device=device)
    ctx.set_overlap(overlap)
    hk, hv, hb = pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"])
    gl = LayerCache(ctx, hk, hv, hb, torch.from_numpy(n_tok))
    # both sides read the same pooled bytes (the oracle's); the library's own pooling is checked too
    gl.rebuild_pooled()
    torch.cuda.synchronize()
    assert to_np(gl.k_pooled).tobytes() == ol.kc.tobytes()
    assert to_np(gl.se_pooled).tobytes() == ol.sec.tobytes()
    if poison:                      # stale slots must never reach an output
        gl.pool_k.fill_(float("nan"))
        gl.pool_v.fill_(float("nan"))
        gl.pool_bias.fill_(float("nan"))
        ol.pk[...] = 0x7fc0 if ol.pk.dtype == np.uint16 else np.nan
        ol.pv[...] = 0x7fc0 if ol.pv.dtype == np.uint16 else np.nan
        ol.pb[...] = np.nan
    if residency is not None:
        sob, bos = residency
        gl.set_residency(sob, bos)
        ol.sob[...], ol.bos[...] = sob.numpy(), bos.numpy()
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                for s, J in enumerate(ol.bos[b, h]):
                    if J >= 0:
                        ol.pk[b, h, s], ol.pv[b, h, s], ol.pb[b, h, s] = ol.hk[b, h, J], ol.hv[b, h, J], ol.hb[b, h, J]
    qs = QueryStream(w, seed, layer_index)
    records = []
    for t in range(steps):
        q, retries = draw_with_margin(w, qs, ol, t, margin)
        ref = ol.step(to_np(q), attention=check_attention)
        out = gl.step(q.to(device))
        torch.cuda.synchronize()
        assert (gl.sel_idx.cpu().numpy() == ref["sel"]).all(), f"step {t}: selected blocks differ"
        assert (gl.n_sel.cpu().numpy() == ref["n_sel"]).all()
        assert (gl.n_load.cpu().numpy() == ref["n_load"]).all(), f"step {t}: miss counts differ"
        assert (gl.load_list.cpu().numpy() == ref["load_list"]).all()
        assert (gl.slot_of_block.cpu().numpy() == ol.sob).all() and (gl.block_of_slot.cpu().numpy() == ol.bos).all()
        err = None
        if check_attention:
            got = out.double().cpu().numpy()
            assert np.isfinite(got).all(), f"step {t}: non-finite output"
            err = float(np.abs(got - ref["out"]).max())
            assert err <= out_tol(w.dtype), f"step {t}: max abs err {err}"
        if t > 0 and w.gpu_slots == w.k_blocks:
            assert ref["n_load"].max() <= w.kq_blocks          # Theorem 1 on the measured run
        records.append(dict(step=t, n_load_max=int(ref["n_load"].max()), n_load_mean=float(ref["n_load"].mean()),
                            retries=retries, err=err))
    # the selected slots hold the host bytes
    sob = gl.slot_of_block.cpu().numpy()
    sel, n_sel = gl.sel_idx.cpu().numpy(), gl.n_sel.cpu().numpy()
    pk, pv, pb = to_np(gl.pool_k), to_np(gl.pool_v), to_np(gl.pool_bias)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            for J in sel[b, h, :n_sel[b, h]]:
                s = sob[b, h, J]
                assert pk[b, h, s].tobytes() == ol.hk[b, h, J].tobytes()
                assert pv[b, h, s].tobytes() == ol.hv[b, h, J].tobytes()
                assert pb[b, h, s].tobytes() == ol.hb[b, h, J].tobytes()
    ctx.close()
    return records


def run_fullsize_sampled(w: Workload, seed: int, steps: int, n_samples: int, device="cuda:0", margin=1e-3):
    """A workload at its full size with the library's default stream order (default splits, fetch on the
    side stream, attention in two launches around it, cold start through the real path), checked two ways
    (``run_fullsize_all_units`` covers the one-stream order that ``bench.py`` times):

    * sampled units: each is re-run by the oracle as a one-unit problem on the same bytes, with its
      residency state carried along; Gamma, miss count and the attention rows must match;
    * all units: properties that hold at any size (Gamma ascending and unique, forced blocks inside,
      miss count <= Kq after the first step, maps inverse to each other, finite outputs).
    """
    import paper_2510_13602_amd as nosa
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like

    print(f"fullsize {w.name}: drawing the layer on the GPU", flush=True)
    layer = make_layer(w, seed, 0, device=device)
    hk, hv, hb = pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"])
    del layer
    torch.cuda.empty_cache()
    ctx = nosa.Nosa(gpu_params(w), device=device)
    gl = LayerCache(ctx, hk, hv, hb, torch.full((w.batch,), w.context, dtype=torch.int32))
    gl.rebuild_pooled()
    gl.pool_k.fill_(float("nan")); gl.pool_v.fill_(float("nan")); gl.pool_bias.fill_(float("nan"))
    torch.cuda.synchronize()

    rng = np.random.default_rng(seed + 99)
    units = [(0, 0), (w.batch - 1, w.n_kv_heads - 1)]
    while len(units) < n_samples:
        u = (int(rng.integers(w.batch)), int(rng.integers(w.n_kv_heads)))
        if u not in units:
            units.append(u)
    G = w.group
    w1 = w.replace(batch=1, n_q_heads=G, n_kv_heads=1)
    n1 = np.array([w.context], np.int32)
    oracles = {}
    for (b, h) in units:
        ol = OracleLayer(w1, to_np(hk[b:b + 1, h:h + 1]), to_np(hv[b:b + 1, h:h + 1]), to_np(hb[b:b + 1, h:h + 1]), n1)
        assert to_np(gl.k_pooled[b:b + 1, h:h + 1]).tobytes() == ol.kc.tobytes()     # the library's pooled keys
        assert to_np(gl.se_pooled[b:b + 1, h:h + 1]).tobytes() == ol.sec.tobytes()
        ol.pk[...] = 0x7fc0 if ol.pk.dtype == np.uint16 else np.nan
        ol.pv[...] = 0x7fc0 if ol.pv.dtype == np.uint16 else np.nan
        ol.pb[...] = np.nan
        oracles[(b, h)] = ol
    qs = QueryStream(w, seed, 0, device=device)
    N, Nc = w.max_blocks, w.context // w.block_size
    forced = sorted(set(range(min(w.sink_blocks, N))) | set(range(max(0, N - w.window_blocks), N)))
    worst = 0.0
    for t in range(steps):
        d = qs.draw(t, 0)
        for r in range(1, 9):                         # margin rule on the sampled units only
            q = d["q32"].to(w.torch_dtype)
            bad = []
            for (b, h), ol in oracles.items():
                gap = query_margin(w1, ol.scores(to_np(q[b:b + 1, h * G:(h + 1) * G]))[0], n1)[0, 0]
                if gap < margin:
                    bad.append((b, h))
            if not bad:
                break
            alt = qs.draw(t, r)
            for b, h in bad:
                for key in ("q32", "x", "m"):
                    if d[key] is not None:
                        d[key][b, h * G:(h + 1) * G] = alt[key][b, h * G:(h + 1) * G]
        q = qs.commit(d)
        out = gl.step(q)
        torch.cuda.synchronize()
        sel, n_sel, n_load = gl.sel_idx.cpu().numpy(), gl.n_sel.cpu().numpy(), gl.n_load.cpu().numpy()
        sob, bos = gl.slot_of_block.cpu().numpy(), gl.block_of_slot.cpu().numpy()
        got = out.double().cpu().numpy()
        # properties over all units
        assert np.isfinite(got).all()
        assert (n_sel == min(w.k_blocks, N)).all()
        assert (np.diff(sel, axis=-1) > 0).all() and sel.min() >= 0 and sel.max() < N
        assert all((sel == J).any(-1).all() for J in forced)
        if t == 0:
            assert (n_load == w.k_blocks).all()
        elif w.gpu_slots == w.k_blocks:
            assert n_load.max() <= w.kq_blocks
        slots = np.take_along_axis(sob, sel, axis=-1)
        assert (slots >= 0).all() and (np.take_along_axis(bos, slots, axis=-1) == sel).all()
        assert (np.sort(slots, axis=-1)[..., 1:] != np.sort(slots, axis=-1)[..., :-1]).all()
        # sampled units against the oracle
        for (b, h), ol in oracles.items():
            ref = ol.step(to_np(q[b:b + 1, h * G:(h + 1) * G]))
            assert (sel[b, h] == ref["sel"][0, 0]).all(), f"step {t} unit {(b, h)}: selected blocks differ"
            assert n_load[b, h] == ref["n_load"][0, 0], f"step {t} unit {(b, h)}: miss count differs"
            err = float(np.abs(got[b, h * G:(h + 1) * G] - ref["out"][0]).max())
            worst = max(worst, err)
            assert err <= out_tol(w.dtype), f"step {t} unit {(b, h)}: max abs err {err}"
        print(f"fullsize {w.name} step {t}: n_load mean {n_load.mean():.2f} max {n_load.max()}, worst err so far {worst:.2e}", flush=True)
    ctx.close()
    return worst


def run_fullsize_all_units(w: Workload, seed: int, layer_index: int, steps: int, attention_steps, mode: str,
                           device="cuda:0", margin=1e-3):
    """A workload at its full size, EVERY unit against the oracle at EVERY step: Gamma, its length, the miss
    count, the load list and both residency maps bit for bit; the attention output of every unit on the steps
    in ``attention_steps``; at the end the whole GPU pool byte for byte against the oracle's.

    ``mode`` picks the launch configuration: "fused" is what ``bench.py`` times (everything on one stream
    through the single ``nosa_decode_step`` entry: the plain attention kernel, default splits); "overlap" is
    the library's default order (gather on the side stream, attention in two launches around it).
    The layer (index ``layer_index`` of the workload's stack) is drawn on the GPU and copied to pinned host
    memory once; the oracle reads those very bytes.
    """
    import paper_2510_13602_amd as nosa
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like

    assert mode in ("fused", "overlap")
    attention_steps = set(attention_steps)
    print(f"all units {w.name} layer {layer_index} ({mode}): drawing the layer on the GPU", flush=True)
    layer = make_layer(w, seed, layer_index, device=device)
    hk, hv, hb = pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"])
    del layer
    torch.cuda.empty_cache()
    n_tok = np.full((w.batch,), w.context, np.int32)
    ol = OracleLayer(w, to_np(hk), to_np(hv), to_np(hb), n_tok)
    ctx = nosa.Nosa(gpu_params(w), device=device)
    ctx.set_overlap(mode == "overlap")
    gl = LayerCache(ctx, hk, hv, hb, torch.from_numpy(n_tok))
    gl.rebuild_pooled()
    torch.cuda.synchronize()
    assert to_np(gl.k_pooled).tobytes() == ol.kc.tobytes()
    assert to_np(gl.se_pooled).tobytes() == ol.sec.tobytes()
    gl.pool_k.fill_(float("nan")); gl.pool_v.fill_(float("nan")); gl.pool_bias.fill_(float("nan"))
    ol.pk[...] = 0x7fc0 if ol.pk.dtype == np.uint16 else np.nan
    ol.pv[...] = 0x7fc0 if ol.pv.dtype == np.uint16 else np.nan
    ol.pb[...] = np.nan
    qs = QueryStream(w, seed, layer_index, device=device)
    worst, retries_total, loads = 0.0, 0, []
    for t in range(steps):
        q, retries = draw_with_margin(w, qs, ol, t, margin)
        retries_total += retries
        att = t in attention_steps
        ref = ol.step(to_np(q), attention=att)
        out = gl.step_fused(q) if mode == "fused" else gl.step(q)
        torch.cuda.synchronize()
        assert (gl.sel_idx.cpu().numpy() == ref["sel"]).all(), f"step {t}: selected blocks differ"
        assert (gl.n_sel.cpu().numpy() == ref["n_sel"]).all()
        assert (gl.n_load.cpu().numpy() == ref["n_load"]).all(), f"step {t}: miss counts differ"
        assert (gl.load_list.cpu().numpy() == ref["load_list"]).all(), f"step {t}: load lists differ"
        assert (gl.slot_of_block.cpu().numpy() == ol.sob).all() and (gl.block_of_slot.cpu().numpy() == ol.bos).all()
        if t == 0:
            assert (ref["n_load"] == min(w.k_blocks, w.max_blocks)).all()
        elif w.gpu_slots == w.k_blocks:
            assert ref["n_load"].max() <= w.kq_blocks, f"step {t}: fetch bound broken"          # Theorem 1
        if t > 0:
            loads.append(float(ref["n_load"].mean()))
        if att:
            got = out.double().cpu().numpy()
            assert np.isfinite(got).all(), f"step {t}: non-finite output"
            err = float(np.abs(got - ref["out"]).max())
            worst = max(worst, err)
            assert err <= out_tol(w.dtype), f"step {t}: max abs err {err}"
            lerr = float(np.abs(gl.lse.double().cpu().numpy() - ref["lse"]).max())
            assert lerr <= 1e-3, f"step {t}: lse err {lerr}"
        if t % 16 == 0 or t == steps - 1:
            print(f"all units {w.name} layer {layer_index} ({mode}) step {t}: n_load mean {ref['n_load'].mean():.2f} "
                  f"max {ref['n_load'].max()}, worst attention err so far {worst:.2e}", flush=True)
    assert to_np(gl.pool_k).tobytes() == ol.pk.tobytes() and to_np(gl.pool_v).tobytes() == ol.pv.tobytes()
    assert to_np(gl.pool_bias).tobytes() == ol.pb.tobytes()
    ctx.close()
    return dict(worst=worst, retries=retries_total, mean_load=float(np.mean(loads)) if loads else 0.0)


def run_growing(w: Workload, seed: int, steps: int, device="cuda:0", margin=1e-3, check_every=1, attention_steps=None,
                progress=0):
    """Growing context: every step after the first appends one token per unit (key, value, bias)
    before scoring, on both sides; the integer state (token counts, Gamma, miss counts, load lists, both
    maps) is compared at EVERY step.  Pooled arrays and the attention output are compared on the steps
    of ``attention_steps`` (default: every ``check_every``-th step and the steps around block boundaries).
    Also asserts the fetch bound n_load <= Kq at every step after the first, block boundaries included.
    """
    import paper_2510_13602_amd as nosa
    from nosa_inputs import append_token
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like

    assert w.generated >= steps - 1          # step 0 appends nothing
    layer = make_layer(w, seed, 0)
    n_tok = np.full((w.batch,), w.context, np.int32)
    ol = OracleLayer(w, to_np(layer["host_k"]).copy(), to_np(layer["host_v"]).copy(), to_np(layer["host_bias"]).copy(), n_tok)
    ctx = nosa.Nosa(gpu_params(w), device=device)
    ctx.set_overlap(True)                        # whatever the shape's default: the two-launch order is the one under test here
    gl = LayerCache(ctx, pinned_like(layer["host_k"]), pinned_like(layer["host_v"]), pinned_like(layer["host_bias"]),
                    torch.from_numpy(n_tok))
    gl.rebuild_pooled()
    qs = QueryStream(w, seed, 0)
    prev_se = np.full((w.batch, w.n_kv_heads, w.max_blocks), -np.inf)
    boundary_loads, worst, checked = [], 0.0, 0

    def n_sub(T):                     # complete sub-blocks of a cache of T tokens
        return 0 if T < w.pool_kernel else (T - w.pool_kernel) // w.pool_stride + 1

    for t in range(steps):
        if t > 0:
            tok = append_token(w, seed, 0, t)
            before = n_sub(int(ol.n_tok[0]))
            oracle.append(ol.p, to_np(tok["k_new"]), to_np(tok["v_new"]), to_np(tok["b_new"]), ol.pk, ol.pv, ol.pb,
                          ol.hk, ol.hv, ol.hb, prev_se, ol.n_tok, ol.sob, ol.bos)
            if n_sub(int(ol.n_tok[0])) != before:       # the pooled arrays only change when a sub-block completes
                ol.kc, ol.sec = oracle.pool(ol.p, ol.hk, ol.hb, ol.n_tok)
            gl.append(tok["k_new"].to(device), tok["v_new"].to(device), tok["b_new"].to(device))
        q, _ = draw_with_margin(w, qs, ol, t, margin)
        if attention_steps is None:
            check = t % check_every == 0 or (w.context + t) % w.block_size in (0, 1, w.block_size - 1)
        else:
            check = t in attention_steps
        ref = ol.step(to_np(q), attention=check)
        prev_se = ref["se"]
        out = gl.step(q.to(device))
        torch.cuda.synchronize()
        assert (gl.n_tokens.cpu().numpy() == ol.n_tok).all(), f"step {t}: token counts differ"
        assert (gl.sel_idx.cpu().numpy() == ref["sel"]).all(), f"step {t}: selected blocks differ"
        assert (gl.n_load.cpu().numpy() == ref["n_load"]).all(), f"step {t}: miss counts differ"
        assert (gl.load_list.cpu().numpy() == ref["load_list"]).all()
        assert (gl.slot_of_block.cpu().numpy() == ol.sob).all() and (gl.block_of_slot.cpu().numpy() == ol.bos).all()
        if t > 0 and w.gpu_slots == w.k_blocks:
            assert ref["n_load"].max() <= w.kq_blocks, f"step {t}: fetch bound broken ({ref['n_load'].max()})"
        if (w.context + t) % w.block_size == 0:
            boundary_loads.append(int(ref["n_load"].max()))
        if progress and t % progress == 0:
            print(f"growing {w.name}: step {t} of {steps}, {int(ol.n_tok[0])} tokens, n_load max {int(ref['n_load'].max())}, "
                  f"{checked} attention checks, worst err {worst:.2e}", flush=True)
        if check:
            checked += 1
            assert to_np(gl.k_pooled).tobytes() == ol.kc.tobytes(), f"step {t}: pooled keys differ"
            assert to_np(gl.se_pooled).tobytes() == ol.sec.tobytes(), f"step {t}: pooled importance differs"
            got = out.double().cpu().numpy()
            assert np.isfinite(got).all()
            err = float(np.abs(got - ref["out"]).max())
            worst = max(worst, err)
            assert err <= out_tol(w.dtype), f"step {t}: max abs err {err}"
    # the host pool received every appended token
    torch.cuda.synchronize()
    assert to_np(gl.host_k).tobytes() == ol.hk.tobytes() and to_np(gl.host_v).tobytes() == ol.hv.tobytes()
    assert to_np(gl.host_bias).tobytes() == ol.hb.tobytes()
    # ... and the pooled arrays and the GPU pool ended up identical to the oracle's
    assert to_np(gl.k_pooled).tobytes() == ol.kc.tobytes() and to_np(gl.se_pooled).tobytes() == ol.sec.tobytes()
    assert to_np(gl.pool_k).tobytes() == ol.pk.tobytes() and to_np(gl.pool_v).tobytes() == ol.pv.tobytes()
    assert to_np(gl.pool_bias).tobytes() == ol.pb.tobytes()
    ctx.close()
    return dict(worst=worst, boundary_loads=boundary_loads, checked=checked)


# ---- sparse prefill --------------------------------------------------------------------------------

def prefill_inputs(w: Workload, seed: int, p0: int, lq: int, positions=None, margin: float = 1e-3, max_retry: int = 8):
    """Cache, pooled arrays and the chunk's queries.  Positions (all, or the sample) whose query-aware selection
    margin is below ``margin`` get the query of an independent redraw, unit by unit."""
    from nosa_inputs import chunk_queries
    p = oracle_params(w)
    layer = make_layer(w, seed, 0)
    hk, hv, hb = to_np(layer["host_k"]), to_np(layer["host_v"]), to_np(layer["host_bias"])
    n_full = np.full((w.batch,), p0 + lq, np.int32)
    kc, sec = oracle.pool(p, hk, hb, n_full)
    q32 = chunk_queries(w, seed, 0, lq)
    pos = list(range(lq)) if positions is None else list(positions)
    G = w.group
    todo = pos
    for r in range(1, max_retry + 1):
        q = to_np(q32.to(w.torch_dtype))
        bad = []
        for t in todo:
            n_tok = np.full((w.batch,), p0 + t + 1, np.int32)
            sq, _ = oracle.block_score(p, np.ascontiguousarray(q[:, t]), kc, sec, n_tok)
            for b, h in np.argwhere(query_margin(w, sq, n_tok) < margin):
                bad.append((t, b, h))
        if not bad:
            break
        alt = chunk_queries(w, seed, 0, lq, retry=r)
        for t, b, h in bad:
            q32[b, t, h * G:(h + 1) * G] = alt[b, t, h * G:(h + 1) * G]
        todo = sorted({t for t, _, _ in bad})
    else:
        raise AssertionError("selection margin not reached")
    return dict(p=p, hk=hk, hv=hv, hb=hb, kc=kc, sec=sec, q=q32.to(w.torch_dtype), layer=layer)


def run_prefill_parity(w: Workload, seed: int, p0: int, lq: int, positions=None, device="cuda:0"):
    """One chunk through oracle.prefill and through nosa_prefill_select / nosa_prefill_attend: selections
    bit-exact, outputs within the dtype's tolerance, at all positions or at the sample."""
    import paper_2510_13602_amd as nosa
    inp = prefill_inputs(w, seed, p0, lq, positions)
    p = inp["p"]
    q_np = to_np(inp["q"])
    sel_o, nsel_o, out_o, lse_o = oracle.prefill(p, q_np, inp["hk"], inp["hv"], inp["hb"], inp["kc"], inp["sec"], p0,
                                                 positions)
    B, H, d = w.batch, w.n_kv_heads, w.head_dim
    td = w.torch_dtype
    ctx = nosa.Nosa(gpu_params(w), device=device)
    ck, cv = inp["layer"]["host_k"].to(device), inp["layer"]["host_v"].to(device)
    cb = inp["layer"]["host_bias"].to(device)
    n_full = torch.full((B,), p0 + lq, dtype=torch.int32, device=device)
    kc = torch.zeros((B, H, w.n_sub_max, d), dtype=td, device=device)
    sec = torch.zeros((B, H, w.n_sub_max), dtype=torch.float32, device=device)
    ctx.nosa_pool_blocks(ck, cb, n_full, kc, sec)
    q = inp["q"].to(device)
    n_tok_s = torch.empty((B * lq,), dtype=torch.int32, device=device)
    sq_s = torch.empty((B, lq, H, w.max_blocks), dtype=torch.float32, device=device)
    se_s = torch.empty_like(sq_s)
    sel = torch.full((B, lq, H, w.k_blocks), -7, dtype=torch.int32, device=device)
    n_sel = torch.full((B, lq, H), -7, dtype=torch.int32, device=device)
    out = torch.full((B, lq, w.n_q_heads, d), float("nan"), dtype=td, device=device)
    lse = torch.full((B, lq, w.n_q_heads), float("nan"), dtype=torch.float32, device=device)
    ctx.nosa_prefill_select(q, kc, sec, p0, lq, n_tok_s, sq_s, se_s, sel, n_sel)
    ctx.nosa_prefill_attend(q, ck, cv, cb, sel, n_sel, p0, lq, out, lse)
    torch.cuda.synchronize()
    sel_g = sel.cpu().numpy().transpose(0, 2, 1, 3)          # -> [B,H,lq,K]
    nsel_g = n_sel.cpu().numpy().transpose(0, 2, 1)
    out_g, lse_g = out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    pos = np.arange(lq) if positions is None else np.asarray(sorted(positions))
    np.testing.assert_array_equal(n_tok_s.cpu().numpy().reshape(B, lq), np.tile(p0 + np.arange(lq) + 1, (B, 1)))
    np.testing.assert_array_equal(nsel_g[:, :, pos], nsel_o[:, :, pos])
    np.testing.assert_array_equal(sel_g[:, :, pos], sel_o[:, :, pos])
    tol = out_tol(w.dtype)
    err = np.abs(out_g[:, pos] - out_o[:, pos]).max()
    assert np.isfinite(out_g).all() and err <= tol, f"prefill attention: max abs err {err} > {tol}"
    lerr = np.abs(lse_g[:, pos] - lse_o[:, pos]).max()
    assert lerr <= 1e-2, f"prefill lse: max abs err {lerr}"
    ctx.close()
    return dict(err=err, lse_err=lerr, n_pos=len(pos))
