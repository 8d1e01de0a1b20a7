#!/usr/bin/env python3
"""Benchmark of the NOSA decode-step hot path on one MI355X.

A "step" is one pass of the whole path (block score -> constrained selection + load positions ->
fetch of missed blocks from pinned host memory -> block-sparse attention) over one batch of one
layer of the 8B-shaped workload (batch 64, 32 query / 8 KV heads, d 128, 32768 tokens, block 64,
K = 64 blocks, fetch budget Kq = 8, bf16).  Successive steps cycle through distinct layers, so no
step finds its KV pool in cache.  The metric counts (batch x KV head x layer) units per second.

Prints ONE JSON line.  `value` counts units per second over the timed steps (inputs resident before the
timed region); `roofline` prices the attention kernel's algorithmic HBM bytes per launch, timed with HIP
events inside the same region, against the 8 TB/s peak; `cpu_baseline` is the fp64 CPU oracle on a bounded
sample of the same tensors.  `--study prefill` and `--study transfer` print lines of their own.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="8b", choices=["tiny", "1b", "3b", "8b", "longgen"])
    ap.add_argument("--layers", type=int, default=0, help="distinct GPU layer states to cycle (0 = workload default, max 32)")
    ap.add_argument("--host-layers", type=int, default=2, help="distinct pinned host pools (each 8 GiB at the 8B shape)")
    ap.add_argument("--splits", type=int, default=0, help="override the number of attention splits")
    ap.add_argument("--fetch-wgs", type=int, default=0, help="override the gather kernel's grid size")
    ap.add_argument("--no-overlap", action="store_true", help="run the fetch on the main stream")
    ap.add_argument("--resident", action="store_true", help="kernel-only mode: same queries every step, so nothing is fetched")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-batch", type=int, default=16)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU work the oracle baseline is given")
    ap.add_argument("--no-kernel-timing", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--kq", type=int, default=0, help="override the query-aware budget Kq (blocks); Ke shrinks accordingly")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--heads", default="", help="override the head counts: 'Hq,Hkv' (e.g. 32,2 for the paper's own 8B model)")
    ap.add_argument("--slots", type=int, default=0,
                    help="GPU pool slots C per unit (default: the workload's, C = K for the 8B shape); C > K keeps blocks beyond the selection resident")
    ap.add_argument("--victim-policy", type=int, default=-1, choices=[-1, 0, 1],
                    help="which free slot a missed block overwrites: 0 lowest slot, 1 least important block (default: the workload's)")
    ap.add_argument("--xcd-shift-kib", type=int, default=0, help="xcd study: place the pools of odd layer states this many KiB further into their allocations")
    ap.add_argument("--gen-tokens", type=int, default=16384, help="long-generation workload: tokens generated per layer state")
    ap.add_argument("--no-fused-select", action="store_true",
                    help="run block score and selection as two kernels inside nosa_decode_step (default: one kernel, scores stay on chip)")
    ap.add_argument("--attention-kernel", type=int, default=0, choices=[0, 1, 2],
                    help="0 chosen from the shape, 1 vector-ALU attention kernel, 2 matrix-core attention kernel (bf16)")
    ap.add_argument("--gap-cycles", type=int, default=0,
                    help="experiment: a one-thread spin kernel of this many clock ticks before every step (the GPU is as good as idle meanwhile)")
    ap.add_argument("--no-larger-pool", action="store_true",
                    help="skip the second measurement of the headline workload with C = 96 slots and importance-ranked victims")
    ap.add_argument("--locality-steps", type=int, default=64, help="untimed steps after the timed regions that record the miss count of every step")
    ap.add_argument("--study", default="", choices=["", "transfer", "prefill", "xcd"],
                    help="transfer: block-wise versus element-wise host-to-device gather over miss fractions (prints one JSON line per point); "
                         "prefill: sparse prefill of one chunk at the end of the 8B-shaped context (one JSON line); "
                         "xcd: per-XCD timing of the attention kernel's workgroups over several layer states (one JSON line)")
    ap.add_argument("--prefill-batch", type=int, default=4)
    ap.add_argument("--prefill-chunk", type=int, default=2048, help="query positions per chunk (multiple of 64)")
    ap.add_argument("--prefill-all", action="store_true",
                    help="prefill study: also time every chunk of the context from position 0 and report the whole-prompt rate")
    ap.add_argument("--mode", default="fused", choices=["calls", "fused", "graph"],
                    help="how a step crosses the C ABI: four calls, the single nosa_decode_step entry, or a HIP graph replay")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run five plain 1 GiB device copies (known traffic, for scaling rocprofv3 counters)")
    return ap.parse_args()


def decode_bytes_per_unit(w) -> int:
    """Algorithmic HBM bytes one unit costs the attention kernel per step: the K and V rows and the
    bias of the K selected blocks, q in, o out, the selection list and its slots."""
    e = w.elem_size
    kv = w.k_blocks * w.block_size * (2 * w.head_dim * e + 4)
    qo = 2 * w.group * w.head_dim * e
    idx = 2 * w.k_blocks * 4
    return kv + qo + idx


def step_bytes_per_unit(w) -> int:
    """Algorithmic HBM bytes of the whole step per unit: attention + pooled keys and importance."""
    e = w.elem_size
    return decode_bytes_per_unit(w) + w.n_sub_max * (w.head_dim * e + 4)


def cpu_baseline(w, host, queries, sample_batch, seconds):
    """The fp64 oracle, as it stands, timed on this machine's host cores on a slice (the first
    ``sample_batch`` batch elements) of the very tensors the GPU run used."""
    import numpy as np
    import oracle
    to_np = oracle.to_np
    ws = w.replace(batch=sample_batch)
    p = oracle.params_from_workload(ws)
    hk, hv, hb = (to_np(t[:sample_batch]) for t in host)
    n_tok = np.full((ws.batch,), ws.context, np.int32)
    kc, sec = oracle.pool(p, hk, hb, n_tok)
    B, H, C, nb, d = ws.batch, ws.n_kv_heads, ws.gpu_slots, ws.block_size, ws.head_dim
    pk, pv = np.zeros((B, H, C, nb, d), hk.dtype), np.zeros((B, H, C, nb, d), hv.dtype)
    pb = np.zeros((B, H, C, nb), np.float32)
    sob = np.full((B, H, ws.max_blocks), -1, np.int32)
    bos = np.full((B, H, C), -1, np.int32)
    qs = [to_np(q[:sample_batch]) for q in queries]

    def one(t):
        q = qs[t % len(qs)]
        sq, se = oracle.block_score(p, q, kc, sec, n_tok)
        sel, n_sel = oracle.select(p, sq, se, n_tok)
        ll, n_load = oracle.load(p, sel, n_sel, sob, bos)
        oracle.fetch(p, hk, hv, hb, pk, pv, pb, ll, n_load)
        oracle.attention(p, q, pk, pv, pb, sel, n_sel, sob, n_tok)

    one(0)                                   # cold start (fills the pool), untimed
    threads = oracle.num_threads()

    def timed(budget, first):
        n, t0 = 0, time.perf_counter()
        while n < 2 or time.perf_counter() - t0 < budget:
            n += 1
            one(first + n)
        return n, time.perf_counter() - t0

    # one thread first (a quarter of the budget), then every thread the oracle's OpenMP runtime gives it
    oracle.set_threads(1)
    n1, dt1 = timed(0.25 * seconds, 0)
    oracle.set_threads(threads)
    steps, dt = timed(0.75 * seconds, n1)
    what = (f"whole steps (score, select, load, fetch, attention) of {ws.units} units = batch {sample_batch} of {w.batch} "
            f"of the {w.name}-shaped workload, same tensors as the GPU run, fp64")
    return {"value": ws.units * steps / dt, "unit": "unit-steps/s", "cores": threads, "kind": "oracle",
            "sample": f"{steps} {what}, OpenMP over units on {threads} threads, {dt:.1f} s",
            "single_thread": {"value": ws.units * n1 / dt1, "unit": "unit-steps/s", "cores": 1,
                              "sample": f"{n1} {what}, one thread, {dt1:.1f} s"}}


def transfer_study(args):
    """Block-wise versus element-wise host-to-device gather (Sec. 3.2 "Comparison with DMA"; Sec. 4
    "Offloading Communication") at the paper's micro-benchmark shape: batch 64, 2 KV heads, d 128, a budget of
    4096 tokens (64 blocks of 64) per head, of which a fraction 1 - gamma is fetched from pinned host memory."""
    import numpy as np
    import torch
    import paper_2510_13602_amd as nosa
    from nosa_inputs import Workload
    dev = "cuda:0"
    w = Workload("transfer", 64, 2, 2, 128, 16384, 64, 16, 1, 16, 64, "bf16", 1, 1, "key_offset")
    params = nosa.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
                              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
                              n_sub_max=w.n_sub_max, dtype=w.dtype)
    ctx = nosa.Nosa(params, device=dev)
    ctx.set_overlap(False)
    B, H, N, C, nb, d = w.batch, w.n_kv_heads, w.max_blocks, w.gpu_slots, w.block_size, w.head_dim
    g = torch.Generator(device=dev).manual_seed(args.seed)
    host = []
    for shape, dt in (((B, H, N, nb, d), torch.bfloat16), ((B, H, N, nb, d), torch.bfloat16), ((B, H, N, nb), torch.float32)):
        t = torch.empty(shape, dtype=dt, pin_memory=True)
        t.copy_(torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(dt))
        host.append(t)
    pool_k = torch.zeros((B, H, C, nb, d), dtype=torch.bfloat16, device=dev)
    pool_v = torch.zeros_like(pool_k)
    pool_b = torch.zeros((B, H, C, nb), dtype=torch.float32, device=dev)
    rng = np.random.default_rng(args.seed)
    reps = 20
    for gamma in (0.5, 0.6, 0.7, 0.75, 0.8, 0.9, 0.95):
        n_blk = round((1 - gamma) * C)
        n_tok = n_blk * nb
        # block-wise: n_blk random blocks into random slots; element-wise: n_tok random tokens into random rows
        ll = np.full((B, H, w.k_blocks, 2), -1, np.int32)
        tl = np.full((B, H, n_tok, 2), -1, np.int32)
        for b in range(B):
            for h in range(H):
                ll[b, h, :n_blk, 0] = np.sort(rng.choice(N, n_blk, replace=False))
                ll[b, h, :n_blk, 1] = rng.choice(C, n_blk, replace=False)
                tl[b, h, :, 0] = rng.choice(N * nb, n_tok, replace=False)
                tl[b, h, :, 1] = rng.choice(C * nb, n_tok, replace=False)
        ll_d, tl_d = torch.from_numpy(ll).to(dev), torch.from_numpy(tl).to(dev)
        nl_d = torch.full((B, H), n_blk, dtype=torch.int32, device=dev)
        nt_d = torch.full((B, H), n_tok, dtype=torch.int32, device=dev)
        nbytes = B * H * n_tok * (2 * d * 2 + 4)
        for pattern in ("block", "element"):
            def go():
                if pattern == "block":
                    ctx.nosa_fetch(host[0], host[1], host[2], pool_k, pool_v, pool_b, ll_d, nl_d)
                else:
                    ctx.nosa_fetch_tokens(host[0], host[1], host[2], pool_k, pool_v, pool_b, tl_d, nt_d)
            go()
            torch.cuda.synchronize()
            ctx.timing_enable(True)
            ctx.timing_read(nosa.KERNEL_FETCH)
            for _ in range(reps):
                go()
            torch.cuda.synchronize()
            ms, n = ctx.timing_read(nosa.KERNEL_FETCH)
            ctx.timing_enable(False)
            print(json.dumps({"study": "transfer", "pattern": pattern, "gamma": gamma, "fetched_per_head": n_blk if pattern == "block" else n_tok,
                              "unit": "blocks" if pattern == "block" else "tokens", "bytes": nbytes, "avg_us": 1e3 * ms / n,
                              "host_link_GBps": nbytes / (ms / n * 1e-3) / 1e9}), flush=True)
    ctx.close()


def longgen_bench(args):
    """Long-generation 8B-shaped workload: prompt 4096, then ``--gen-tokens`` tokens (default: all 16384) are
    generated per layer state.  A step is split_qkv_evict -> append (host pool, GPU slot, pooled arrays) ->
    score + select -> fetch -> attention of one layer; ``--layers`` layer states (default 2) take turns.
    With ``--mode graph`` the whole step is one HIP graph replay per layer.  Three windows of 256 steps per
    layer -- at the start (N = 64 blocks), in the middle and at the end (N = 320 at full length) -- are timed on
    their own, with per-kernel HIP-event durations when the step is not a graph."""
    import torch
    import paper_2510_13602_amd as nosa
    from nosa_inputs import CONFIGS, QueryStream, append_token, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    dev = "cuda:0"
    gen = args.gen_tokens
    w = CONFIGS["longgen"].replace(generated=gen)
    if args.slots:
        w = w.replace(gpu_slots=args.slots)
    if args.victim_policy >= 0:
        w = w.replace(victim_policy=args.victim_policy)
    L = args.layers or 2
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.set_stream(stream)
    params = nosa.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
                              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
                              n_sub_max=w.n_sub_max, dtype=w.dtype, victim_policy=w.victim_policy)
    ctx = nosa.Nosa(params, stream=stream, device=dev)
    ctx.set_fused_select(not args.no_fused_select)
    ctx.set_attention_kernel(args.attention_kernel)
    if args.fetch_wgs:
        ctx.set_fetch_workgroups(args.fetch_wgs)
    layers, streams = [], []
    for l in range(L):
        lay = make_layer(w, args.seed, l, device=dev)
        lc = LayerCache(ctx, pinned_like(lay["host_k"]), pinned_like(lay["host_v"]), pinned_like(lay["host_bias"]),
                        torch.full((w.batch,), w.context, dtype=torch.int32))
        lc.rebuild_pooled()
        layers.append(lc)
        streams.append(QueryStream(w, args.seed, l, device=dev))
        del lay
    B, Hq, H, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    g = torch.Generator(device=dev).manual_seed(args.seed + 5)
    w1 = (torch.randn((d, H), generator=g, device=dev) / d ** 0.5).float()
    w2 = torch.randn((H,), generator=g, device=dev).float()
    # fused activations of every step: drifting queries | appended keys | appended values
    qkv = [torch.empty((gen + 1, B, (Hq + 2 * H) * d), dtype=w.torch_dtype, device=dev) for _ in range(L)]
    for l in range(L):
        for t in range(gen + 1):
            tok = append_token(w, args.seed, l, t + 1, device=dev)
            qkv[l][t, :, :Hq * d] = streams[l].next(t).reshape(B, Hq * d)
            qkv[l][t, :, Hq * d:(Hq + H) * d] = tok["k_new"].reshape(B, H * d)
            qkv[l][t, :, (Hq + H) * d:] = tok["v_new"].reshape(B, H * d)
    td = w.torch_dtype
    q_out = [torch.empty((B, Hq, d), dtype=td, device=dev) for _ in range(L)]
    k_new = [torch.empty((B, H, d), dtype=td, device=dev) for _ in range(L)]
    v_new = [torch.empty((B, H, d), dtype=td, device=dev) for _ in range(L)]
    b_new = [torch.empty((B, H), dtype=torch.float32, device=dev) for _ in range(L)]
    qkv_static = [torch.empty((B, (Hq + 2 * H) * d), dtype=td, device=dev) for _ in range(L)]
    for l, lc in enumerate(layers):                     # step 0: the prompt's last token is already cached
        lc.step_fused(qkv[l][0][:, :Hq * d].reshape(B, Hq, d).contiguous())
    torch.cuda.synchronize()
    graph = args.mode == "graph"
    if graph:
        for l, lc in enumerate(layers):
            lc.capture_generation(qkv_static[l], w1, w2, 0, q_out[l], k_new[l], v_new[l], b_new[l])
        torch.cuda.synchronize()

    def do_step(l, t):                                   # token t (1-based) of layer l
        if graph:
            qkv_static[l].copy_(qkv[l][t])
            layers[l].replay()
        else:
            ctx.nosa_split_qkv_evict(qkv[l][t], w1, w2, 0, q_out[l], k_new[l], v_new[l], b_new[l])
            layers[l].append(k_new[l], v_new[l], b_new[l])
            layers[l].step_fused(q_out[l])

    win = min(256, max(1, gen // 3))
    starts = sorted({1, max(1, gen // 2 - win // 2), gen - win + 1})
    windows = []
    hist = torch.zeros((win, L, B, H), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    t_all = time.perf_counter()
    t = 1
    in_windows = 0.0
    while t <= gen:
        if t in starts:                                  # a window: synchronise, time it on its own, read the kernel timers
            torch.cuda.synchronize()
            ctx.timing_enable(not graph and not args.no_kernel_timing)
            for k in range(len(nosa.KERNEL_NAMES)):
                ctx.timing_read(k)
            t0 = time.perf_counter()
            for i in range(win):
                for l in range(L):
                    do_step(l, t + i)
                    hist[i, l].copy_(layers[l].n_load)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            ctx.timing_enable(False)
            kern = {}
            for k, name in enumerate(nosa.KERNEL_NAMES):
                ms, n = ctx.timing_read(k)
                if n:
                    kern[name] = 1e3 * ms / n
            tokens = w.context + t + win - 1
            windows.append({"tokens_at_end": tokens, "blocks": (tokens + w.block_size - 1) // w.block_size,
                            "ms_per_step": 1e3 * dt / (win * L), "unit_steps_per_s": w.units * win * L / dt,
                            "kernels_avg_us": kern or None, "mean_blocks_fetched": float(hist.float().mean().item()),
                            "max_blocks_fetched": int(hist.max().item())})
            t += win
            in_windows += dt
        else:
            nxt = min([x for x in starts if x > t] + [gen + 1])
            for tt in range(t, nxt):
                for l in range(L):
                    do_step(l, tt)
            t = nxt
    torch.cuda.synchronize()
    dt_all = time.perf_counter() - t_all
    steps = gen * L
    line = {
        "metric": "sparse decode steps/sec (batch x KV heads x layer units), growing context", "value": w.units * steps / dt_all,
        "unit": "unit-steps/s", "n_gpus": 1, "steps": steps, "warmup": 0, "ms_per_step": 1e3 * dt_all / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "long-generation 8b-shaped", "batch": B, "n_q_heads": Hq, "n_kv_heads": H, "head_dim": d,
                   "prompt": w.context, "generated_per_layer": gen, "tokens_at_end": int(layers[0].n_tokens[0].item()),
                   "k_blocks": w.k_blocks, "kq_blocks": w.kq_blocks, "gpu_slots": w.gpu_slots, "victim_policy": w.victim_policy,
                   "layers_cycled": L, "step_entry": args.mode,
                   "upstream": "split_qkv_evict + append every step" + (", inside the graph" if graph else "")},
        "windows": windows,
        "note": "value covers all steps; the windows are timed between their own synchronisations (with HIP-event pairs around "
                "every kernel unless the step is a graph replay), the steps between windows run without any timing",
    }
    ctx.close()
    print(json.dumps(line), flush=True)


def xcd_study(args):
    """Where the attention kernel's time goes across the chip: per-workgroup start / end stamps (nosa_set_trace) of
    the stand-alone attention launch on the 8B-shaped workload, grouped by the XCD a workgroup ran on, for several
    layer states (distinct pool allocations) visited several times each.  One JSON line."""
    import numpy as np
    import torch
    import paper_2510_13602_amd as nosa
    from nosa_inputs import CONFIGS, QueryStream, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    dev = "cuda:0"
    w = CONFIGS[args.workload if args.workload in ("3b", "8b") else "8b"]
    L = args.layers or 6
    params = nosa.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
                              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
                              n_sub_max=w.n_sub_max, dtype=w.dtype)
    ctx = nosa.Nosa(params, device=dev)
    ctx.set_overlap(False)
    ctx.set_attention_kernel(args.attention_kernel)
    if args.splits:
        ctx.set_splits(args.splits)
    lay = make_layer(w, args.seed, 0, device=dev)
    host = (pinned_like(lay["host_k"]), pinned_like(lay["host_v"]), pinned_like(lay["host_bias"]))
    del lay
    n_tok = torch.full((w.batch,), w.context, dtype=torch.int32)
    layers = []
    for l in range(L):
        lc = LayerCache(ctx, *host, n_tok)
        if l % 2 == 1 and args.xcd_shift_kib:
            # odd layer states: the same pools, placed args.xcd_shift_kib further into their allocations, so that every
            # unit's blocks sit at different physical-address bits while the workgroup-to-XCD assignment stays the same
            for name in ("pool_k", "pool_v"):
                t = getattr(lc, name)
                shift = args.xcd_shift_kib * 1024 // t.element_size()
                big = torch.zeros(t.numel() + shift, dtype=t.dtype, device=dev)
                setattr(lc, name, big[shift:].view(t.shape))
        if l == 0:
            lc.rebuild_pooled()
        else:
            lc.k_pooled.copy_(layers[0].k_pooled)
            lc.se_pooled.copy_(layers[0].se_pooled)
        layers.append(lc)
    q = QueryStream(w, args.seed, 0, device=dev).next(0)
    for lc in layers:                      # cold start: every layer state ends up with the same selection in its own pool
        lc.step(q)
    torch.cuda.synchronize()
    n_wg = ctx.splits * w.units
    trace = torch.zeros((n_wg, 4), dtype=torch.int64, device=dev)
    ctx.set_trace(trace)
    visits = 4
    per_layer = []
    for l, lc in enumerate(layers):
        durs, ends, xcds = [], [], None
        for v in range(visits + 1):
            for other in layers:           # touch every other pool in between, so that no visit finds its pool in a cache
                if other is not lc:
                    other.decode(q)
            lc.decode(q)
            torch.cuda.synchronize()
            t = trace.cpu().numpy()
            if v == 0:
                continue                   # warm-up visit
            t0 = t[:, 0].min()
            durs.append((t[:, 1] - t[:, 0]) / 100.0)      # us
            ends.append((t[:, 1] - t0) / 100.0)
            xcds = t[:, 2]
        dur, end = np.mean(durs, axis=0), np.mean(ends, axis=0)
        by = []
        for x in range(8):
            m = xcds == x
            by.append({"xcd": x, "workgroups": int(m.sum()), "dur_mean_us": float(dur[m].mean()) if m.any() else None,
                       "dur_min_us": float(dur[m].min()) if m.any() else None, "dur_max_us": float(dur[m].max()) if m.any() else None,
                       "last_end_us": float(end[m].max()) if m.any() else None})
        per_layer.append({"layer_state": l, "pool_shift_kib": args.xcd_shift_kib if l % 2 == 1 else 0, "kernel_span_us": float(end.max()), "workgroup_dur_mean_us": float(dur.mean()),
                          "round_robin_matches_xcc_id": bool(((np.arange(n_wg) % 8) == xcds).all()), "by_xcd": by})
    ctx.set_trace(None)
    ctx.close()
    print(json.dumps({"study": "xcd", "workload": w.name, "attention_kernel": "vector" if args.attention_kernel == 1 else "matrix-core", "workgroups": n_wg, "splits": n_wg // w.units, "visits_averaged": visits,
                      "layers": per_layer}), flush=True)


def prefill_study(args):
    """Sparse prefill of the last chunk of an 8B-shaped context: every query position selects its blocks
    (score + selection kernels on a virtual batch of positions) and attends to them on the matrix cores.
    A step is one chunk (batch x chunk positions) of one layer; two cache copies alternate."""
    import torch
    import paper_2510_13602_amd as nosa
    from nosa_inputs import CONFIGS, chunk_queries, make_layer
    dev = "cuda:0"
    B, lq = args.prefill_batch, args.prefill_chunk
    w = CONFIGS[args.workload if args.workload in ("1b", "3b", "8b") else "8b"].replace(batch=B)
    w = w.replace(gpu_slots=w.max_blocks)
    lq = min(lq, w.context)
    p0 = w.context - lq
    H, Hq, d, K = w.n_kv_heads, w.n_q_heads, w.head_dim, w.k_blocks
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.set_stream(stream)
    params = nosa.make_params(batch=B, n_q_heads=Hq, n_kv_heads=H, head_dim=d, k_blocks=K, kq_blocks=w.kq_blocks,
                              sink_blocks=w.sink_blocks, window_blocks=w.window_blocks, gpu_slots=w.gpu_slots,
                              max_blocks=w.max_blocks, n_sub_max=w.n_sub_max, dtype=w.dtype)
    ctx = nosa.Nosa(params, stream=stream, device=dev)
    td = w.torch_dtype
    L = 2
    caches, qs = [], []
    n_full = torch.full((B,), w.context, dtype=torch.int32, device=dev)
    for l in range(L):
        lay = {k: v.to(dev) for k, v in make_layer(w, args.seed, l).items() if k.startswith("host_")}
        kc = torch.zeros((B, H, w.n_sub_max, d), dtype=td, device=dev)
        sec = torch.zeros((B, H, w.n_sub_max), dtype=torch.float32, device=dev)
        ctx.nosa_pool_blocks(lay["host_k"], lay["host_bias"], n_full, kc, sec)
        caches.append((lay["host_k"], lay["host_v"], lay["host_bias"], kc, sec))
        qs.append(chunk_queries(w, args.seed, l, lq).to(td).to(dev))
    n_tok_s = torch.empty((B * lq,), dtype=torch.int32, device=dev)
    sq_s = torch.empty((B, lq, H, w.max_blocks), dtype=torch.float32, device=dev)
    se_s = torch.empty_like(sq_s)
    sel = torch.empty((B, lq, H, K), dtype=torch.int32, device=dev)
    n_sel = torch.empty((B, lq, H), dtype=torch.int32, device=dev)
    out = torch.empty((B, lq, Hq, d), dtype=td, device=dev)
    lse = torch.empty((B, lq, Hq), dtype=torch.float32, device=dev)

    def do_step(i):
        ck, cv, cb, kc, sec = caches[i % L]
        q = qs[i % L]
        ctx.nosa_prefill_select(q, kc, sec, p0, lq, n_tok_s, sq_s, se_s, sel, n_sel)
        ctx.nosa_prefill_attend(q, ck, cv, cb, sel, n_sel, p0, lq, out, lse)

    for i in range(args.warmup):
        do_step(i)
    torch.cuda.synchronize()
    ctx.timing_enable(True)
    for k in range(len(nosa.KERNEL_NAMES)):
        ctx.timing_read(k)
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        do_step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx.timing_enable(False)
    kern = {}
    for k, name in enumerate(nosa.KERNEL_NAMES):
        ms, n = ctx.timing_read(k)
        if n:
            kern[name] = 1e3 * ms / n
    # algorithmic work of the attention kernel: 4 d flops per (query head, attended token)
    t_in_blk = (torch.arange(lq, device=dev) % 64).view(1, lq, 1)
    tokens = (n_sel.long() * 64 - (63 - t_in_blk)).sum().item()
    flops = 4.0 * d * w.group * tokens
    s4 = sel.view(B, lq // 64, 64, H, K).permute(0, 1, 3, 2, 4).reshape(B, lq // 64, H, 64 * K).long()
    member = torch.zeros((B, lq // 64, H, w.max_blocks + 1), dtype=torch.bool, device=dev)
    member.scatter_(3, torch.where(s4 >= 0, s4, torch.full_like(s4, w.max_blocks)), True)
    union = member[..., :w.max_blocks].sum(-1).float()
    t_att = kern["prefill_attend"] * 1e-6
    line = {
        "metric": "sparse prefill tokens/sec (selection + attention of one layer)", "value": B * lq * args.steps / dt,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}-shaped sparse prefill, last chunk", "batch": B, "chunk": lq, "p0": p0, "n_q_heads": Hq,
                   "n_kv_heads": H, "head_dim": d, "context": w.context, "k_blocks": K, "kq_blocks": w.kq_blocks,
                   "sink_blocks": w.sink_blocks, "window_blocks": w.window_blocks},
        "roofline": {"bound": "mfma", "achieved": flops / t_att / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": flops / t_att / 2.5e15, "traffic": None,
                     "kernel": "prefill_attend", "kernel_avg_us": kern["prefill_attend"], "flops_per_launch": flops},
        "kernels_avg_us": kern,
        "union_blocks_per_workgroup": {"mean": float(union.mean().item()), "max": float(union.max().item()), "budget": K},
    }
    if args.prefill_all:
        # the whole prompt, chunk by chunk (the cache already holds it; a chunk sees only its own prefix)
        per_chunk = []
        ck, cv, cb, kc, sec = caches[0]
        q = qs[0]
        for c0 in range(0, w.context, lq):
            ctx.nosa_prefill_select(q, kc, sec, c0, lq, n_tok_s, sq_s, se_s, sel, n_sel)
            ctx.nosa_prefill_attend(q, ck, cv, cb, sel, n_sel, c0, lq, out, lse)
        torch.cuda.synchronize()
        for c0 in range(0, w.context, lq):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(4):
                ctx.nosa_prefill_select(q, kc, sec, c0, lq, n_tok_s, sq_s, se_s, sel, n_sel)
                ctx.nosa_prefill_attend(q, ck, cv, cb, sel, n_sel, c0, lq, out, lse)
            e1.record(stream)
            e1.synchronize()
            per_chunk.append(e0.elapsed_time(e1) / 4)
        total_ms = sum(per_chunk)
        line["whole_prompt"] = {"chunks": len(per_chunk), "ms_per_chunk": [round(x, 3) for x in per_chunk], "ms_per_layer": total_ms,
                                "tokens_per_s_per_layer": B * w.context / (total_ms * 1e-3)}
    ctx.close()
    print(json.dumps(line), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the path on ONE GPU (no collectives, no sharding); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2510_13602_amd as nosa
    from nosa_inputs import CONFIGS, QueryStream, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like

    if not torch.cuda.is_available():
        print("bench.py: no GPU; the NOSA hot path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "copies": 5}))
        return
    if args.study == "transfer":
        return transfer_study(args)
    if args.study == "prefill":
        return prefill_study(args)
    if args.study == "xcd":
        return xcd_study(args)
    if args.workload == "longgen":
        return longgen_bench(args)
    w = CONFIGS[args.workload]
    if args.kq:
        w = w.replace(kq_blocks=args.kq)
    if args.slots:
        w = w.replace(gpu_slots=args.slots)
    if args.victim_policy >= 0:
        w = w.replace(victim_policy=args.victim_policy)
    if args.batch:
        w = w.replace(batch=args.batch)
    if args.heads:
        hq, hkv = (int(x) for x in args.heads.split(","))
        w = w.replace(n_q_heads=hq, n_kv_heads=hkv)
    line = measure(args, w)
    headline = (args.workload == "8b" and not args.kq and not args.slots and args.victim_policy < 0 and not args.resident
                and not args.batch and not args.heads)
    if headline and not args.no_larger_pool:
        # The same workload with half as many slots again per unit and importance-ranked victims: the paper's
        # pool holds exactly the selection (C = K, the headline above); a larger pool keeps recently used
        # blocks, the misses all but vanish and the step is bound by HBM instead of the host link.
        a2 = argparse.Namespace(**vars(args))
        a2.layers, a2.warmup, a2.no_cpu_baseline, a2.no_overlap = 8, max(args.warmup, 8 * 48), True, True
        sub = measure(a2, w.replace(gpu_slots=96, victim_policy=1))
        line["larger_pool"] = {k: sub[k] for k in ("value", "unit", "ms_per_step", "steps", "warmup", "config", "roofline", "kernels_avg_us",
                                                    "step_hbm_GBps", "step_roofline", "locality", "fetch")}
        if args.mode != "graph":
            # ... and the same steps as one HIP graph replay each (no event pairs, no launch gaps)
            a3 = argparse.Namespace(**vars(a2))
            a3.mode, a3.locality_steps = "graph", 0
            g = measure(a3, w.replace(gpu_slots=96, victim_policy=1))
            line["larger_pool"]["graph_replay"] = {k: g[k] for k in ("value", "unit", "ms_per_step", "step_hbm_GBps", "step_roofline")}
    print(json.dumps(line), flush=True)


def measure(args, w):
    """Sets the workload up, runs the timed regions and returns the JSON line as a dict."""
    import torch
    import paper_2510_13602_amd as nosa
    from nosa_inputs import CONFIGS, QueryStream, make_layer
    from paper_2510_13602_amd.runtime import LayerCache, pinned_like
    dev = "cuda:0"
    L = args.layers or min(w.layers, 32)
    LH = max(1, min(args.host_layers, L))
    t_setup = time.perf_counter()

    params = nosa.make_params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                              k_blocks=w.k_blocks, kq_blocks=w.kq_blocks, sink_blocks=w.sink_blocks,
                              window_blocks=w.window_blocks, gpu_slots=w.gpu_slots, max_blocks=w.max_blocks,
                              n_sub_max=w.n_sub_max, dtype=w.dtype, victim_policy=w.victim_policy)
    stream = torch.cuda.Stream(device=dev)          # a real stream (the NULL stream cannot be captured into a graph)
    torch.cuda.set_stream(stream)
    ctx = nosa.Nosa(params, stream=stream, device=dev)
    if args.splits:
        ctx.set_splits(args.splits)
    if args.fetch_wgs:
        ctx.set_fetch_workgroups(args.fetch_wgs)
    ctx.set_overlap(False)      # the timed region runs every kernel alone on one stream; see below
    ctx.set_fused_select(not args.no_fused_select)
    ctx.set_attention_kernel(args.attention_kernel)

    # host pools: every block of the cache, pinned; drawn on the GPU (seeded) and copied out
    hosts = []
    for hl in range(LH):
        lay = make_layer(w, args.seed, hl, device=dev)
        hosts.append((pinned_like(lay["host_k"]), pinned_like(lay["host_v"]), pinned_like(lay["host_bias"])))
        del lay
        torch.cuda.empty_cache()
    # what the runtime's own copy engine moves from one of these pinned pools (the practical ceiling of the host link)
    link_copy_GBps = None
    if not args.resident:
        src = hosts[0][0].view(-1)[:1 << 29]                       # up to 1 GiB of bf16 (or 2 GiB of fp32)
        dst = torch.empty(src.shape, dtype=src.dtype, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src, non_blocking=True)
        e0.record(stream)
        dst.copy_(src, non_blocking=True)
        e1.record(stream)
        e1.synchronize()
        link_copy_GBps = src.numel() * src.element_size() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del dst
    n_tok = torch.full((w.batch,), w.context, dtype=torch.int32)
    layers = []
    for l in range(L):
        hk, hv, hb = hosts[l % LH]
        lc = LayerCache(ctx, hk, hv, hb, n_tok)
        lc.keep_scores = args.no_fused_select      # fused Stage 1: nobody reads the block scores, so they are not written
        if l < LH:
            lc.rebuild_pooled()
        else:                                   # same host pool -> same pooled arrays
            lc.k_pooled.copy_(layers[l % LH].k_pooled)
            lc.se_pooled.copy_(layers[l % LH].se_pooled)
        layers.append(lc)
    # queries: one stream per host pool (the planted directions belong to the pool)
    streams = [QueryStream(w, args.seed, hl, device=dev) for hl in range(LH)]
    total = args.warmup + args.steps
    n_q = 1 if args.resident else (3 * total + 32 + args.locality_steps) // L + 4
    queries = [[streams[hl].next(t) for t in range(n_q)] for hl in range(LH)]

    def q_of(l, i):
        # a layer's own query stream advances by one per visit of that layer (keeps the step-to-step
        # correlation of the AR(1) workloads); i counts steps over all layers
        return queries[l % LH][0 if args.resident else (i + L - 1) // L]

    q_static = [torch.zeros_like(queries[0][0]) for _ in range(L)]    # what a layer's graph reads its query from

    def do_step(l, q):
        if args.gap_cycles:                         # experiment: an almost idle GPU for a while before every step
            torch.cuda._sleep(args.gap_cycles)
        if args.mode == "calls":
            layers[l].step(q)
        elif args.mode == "fused":
            layers[l].step_fused(q)
        else:
            q_static[l].copy_(q)                    # the query lands in the buffer the graph reads
            layers[l].replay()

    # cold start of every layer (fills the pool through the real path), then W warm-up steps
    for l, lc in enumerate(layers):
        lc.step(q_of(l, 0))
    torch.cuda.synchronize()
    cold_loads = float(sum(lc.n_load.float().mean().item() for lc in layers) / L)
    if args.mode == "graph":
        for l, lc in enumerate(layers):
            lc.capture(q_static[l])
        torch.cuda.synchronize()
    for i in range(args.warmup):
        do_step(i % L, q_of(i % L, 1 + i))
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    names = ["block_score", "select", "fetch", "sparse_decode", "combine"]
    step_no = [args.warmup]

    def timed_region(n_steps):
        """n_steps steps between two synchronisations; returns (seconds, per-kernel mean durations)."""
        ctx.timing_enable(not args.no_kernel_timing)
        for k in range(5):
            ctx.timing_read(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            j = step_no[0]
            do_step(j % L, q_of(j % L, 1 + j))
            step_no[0] += 1
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ctx.timing_enable(False)
        kern = {}
        for k, name in enumerate(names):
            ms, n = ctx.timing_read(k)
            kern[name] = (1e3 * ms / n) if n else None
        return dt, kern

    # The timed region: K steps with every kernel alone on the stream, so that the per-kernel durations (and
    # the roofline figure of the attention kernel) mean what they say.  A second region then repeats K
    # steps in the library's default order -- gather on the side stream, attention over the resident blocks
    # beside it -- which is faster end to end but stretches the attention kernel while host reads are in flight.
    dt, kern = timed_region(args.steps)
    loads = torch.stack([lc.n_load.float() for lc in layers[:min(L, args.steps)]])
    mean_load, max_load = float(loads.mean().item()), float(loads.max().item())
    overlap = None
    if not args.no_overlap:
        mode = args.mode
        if mode == "graph":                      # the graphs were recorded in one-stream order; run eagerly here
            args.mode = "fused"
        ctx.set_overlap(True)
        for _ in range(min(8, args.warmup)):
            j = step_no[0]
            do_step(j % L, q_of(j % L, 1 + j))
            step_no[0] += 1
        dt_ov, kern_ov = timed_region(args.steps)
        # ... and the same order as one HIP graph replay per step: the cross-stream waits become graph edges
        for l, lc in enumerate(layers):
            lc.capture(q_static[l])
        torch.cuda.synchronize()
        args.mode = "graph"
        for _ in range(min(8, args.warmup)):
            j = step_no[0]
            do_step(j % L, q_of(j % L, 1 + j))
            step_no[0] += 1
        dt_og, _ = timed_region(args.steps)
        ctx.set_overlap(False)
        if mode == "graph":                      # back to the graphs of the one-stream order
            for l, lc in enumerate(layers):
                lc.capture(q_static[l])
            torch.cuda.synchronize()
        args.mode = mode
        overlap = {"ms_per_step": 1e3 * dt_ov / args.steps, "value": w.units * args.steps / dt_ov, "kernels_avg_us": kern_ov,
                   "graph_replay": {"ms_per_step": 1e3 * dt_og / args.steps, "value": w.units * args.steps / dt_og},
                   "note": "gather on the side stream; sparse_decode = attention over resident blocks (runs beside the gather), "
                           "combine = attention over fetched blocks + merge; graph_replay = the same steps as one graph launch each"}

    # locality gamma(t) = #(Gamma(t) ^ Gamma(t-1)) / #Gamma(t): with the pool holding the previous selection
    # (and whatever else fits) the blocks NOT fetched are exactly the ones found resident, so
    # gamma(t) >= 1 - n_load / n_sel.  An untimed pass records the miss count of every unit at every step.
    locality = None
    if args.locality_steps > 0 and not args.resident:
        n_loc = args.locality_steps
        hist = torch.zeros((n_loc, w.batch, w.n_kv_heads), dtype=torch.int32, device=dev)
        mode = args.mode
        if mode == "graph":
            args.mode = "fused"
        for i in range(n_loc):
            j = step_no[0]
            do_step(j % L, q_of(j % L, 1 + j))
            hist[i].copy_(layers[j % L].n_load)
            step_no[0] += 1
        args.mode = mode
        torch.cuda.synchronize()
        hit = 1.0 - hist.float() / float(min(w.k_blocks, w.max_blocks))
        locality = {"definition": "gamma(t) = 1 - blocks fetched / blocks selected, per unit and step",
                    "mean": float(hit.mean().item()), "min": float(hit.min().item()),
                    "guaranteed_when_C_equals_K": (w.k_blocks - w.kq_blocks) / w.k_blocks,
                    "steps": n_loc, "units": w.units,
                    "mean_blocks_fetched": float(hist.float().mean().item()), "max_blocks_fetched": int(hist.max().item())}

    units = w.units
    dec_us = kern["sparse_decode"]
    dec_bytes = decode_bytes_per_unit(w) * units
    achieved = dec_bytes / (dec_us * 1e-6) / 1e9 if dec_us else None
    peak = 8000.0
    # HBM bytes per launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE): a stored measurement of this
    # kernel on this workload, not taken during this run (counters need the profiler attached)
    traffic, traffic_source = None, None
    tfile = os.path.join(ROOT, "profiles", f"sparse_decode_{w.name}_hbm_traffic.json")
    if os.path.exists(tfile) and w == CONFIGS[w.name] and args.attention_kernel != 1:
        with open(tfile) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
        traffic_source = f"profiles/sparse_decode_{w.name}_hbm_traffic.md (rocprofv3 --pmc run of this command, stored; not measured in this run)"
    blk_bytes = 2 * w.block_size * w.head_dim * w.elem_size + w.block_size * 4
    fetch_us = kern["fetch"]
    line = {
        "metric": "sparse decode steps/sec (batch x KV heads x layer units) at fixed ctx",
        "value": units * args.steps / dt,
        "unit": "unit-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}-shaped", "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "context": w.context, "block_size": w.block_size, "k_blocks": w.k_blocks,
                   "kq_blocks": w.kq_blocks, "sink_blocks": w.sink_blocks, "window_blocks": w.window_blocks,
                   "gpu_slots": w.gpu_slots, "victim_policy": w.victim_policy, "layers_cycled": L,
                   "stage1": "two kernels" if (args.no_fused_select or args.mode == "calls") else "one kernel (scores + selection + load positions)", "host_pools": LH, "splits": ctx.splits, "step_entry": args.mode,
                   "fetch": "resident (no misses)" if args.resident else "main stream (every kernel alone)"},
        "roofline": {"bound": "hbm", "kernel": (f"decode_mfma_kernel<{w.head_dim},false> (matrix-core attention, group {w.group})"
                                                if w.dtype == "bf16" and args.attention_kernel != 1 else
                                                f"decode_partial_kernel<{w.dtype},{w.head_dim},{w.group},false> (vector-ALU attention)"),
                     "achieved": achieved, "peak": peak, "unit": "GB/s",
                     "frac": (achieved / peak) if achieved else None, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": dec_bytes, "avg_launch_us": dec_us,
                     "scope": "the attention kernel alone (the dominant HBM kernel); the whole step is priced in step_roofline"},
        "cpu_baseline": None,
        "kernels_avg_us": kern,
        "overlap": overlap,
        "step_hbm_GBps": step_bytes_per_unit(w) * units * args.steps / dt / 1e9,
        "step_roofline": None,
        "locality": locality,
        "fetch": {"mean_blocks_per_unit": mean_load, "max_blocks_per_unit": max_load, "cold_start_blocks_per_unit": cold_loads,
                  "host_link_GBps": (mean_load * units * blk_bytes / (fetch_us * 1e-6) / 1e9) if fetch_us else None},
        "setup_s": setup_s,
    }
    # What bounds the whole step: its HBM bytes at 8 TB/s, or the bytes it pulls over the host link at the
    # rate the runtime's own copy of pinned memory reaches on this machine.
    step_s = dt / args.steps
    hbm_s = step_bytes_per_unit(w) * units / 8e12
    link_bytes = mean_load * units * blk_bytes
    link_s = link_bytes / (link_copy_GBps * 1e9) if link_copy_GBps else 0.0
    if link_s > hbm_s:
        line["step_roofline"] = {"bound": "host link", "achieved": link_bytes / step_s / 1e9, "peak": link_copy_GBps, "unit": "GB/s",
                                 "frac": link_bytes / step_s / 1e9 / link_copy_GBps, "peak_source": "pinned-to-device copy of 1 GiB by the runtime, measured in this run",
                                 "link_bytes_per_step": link_bytes, "step_hbm_frac": line["step_hbm_GBps"] / peak}
    else:
        line["step_roofline"] = {"bound": "hbm", "achieved": line["step_hbm_GBps"], "peak": peak, "unit": "GB/s",
                                 "frac": line["step_hbm_GBps"] / peak, "link_bytes_per_step": link_bytes,
                                 "link_copy_GBps": link_copy_GBps}
    if not args.no_cpu_baseline:
        layers.clear()
        torch.cuda.empty_cache()
        line["cpu_baseline"] = cpu_baseline(w, hosts[0], queries[0], min(args.cpu_sample_batch, w.batch), args.cpu_seconds)
    ctx.close()
    return line


if __name__ == "__main__":
    main()
