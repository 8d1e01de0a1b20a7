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
        ll, n_load = oracle.load(self.p, sel, n_sel, self.sob, self.bos)
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
               residency=None, poison=True, margin=1e-3, layer_index=0):
    """Drives ``steps`` decode steps of one layer through both sides; asserts parity at each step.

    Returns per-step records (n_load, retries, max abs error)."""
    import paper_2510_13602_amd as nosa
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like

    layer = make_layer(w, seed, layer_index)
    n_tok = np.full((w.batch,), w.context, np.int32)
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
