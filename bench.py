#!/usr/bin/env python3
"""SP-KV decode benchmark on one MI355X.

A step is one pass of the whole hot path over one batch: the append of one new token per
sequence (gate, ring write, evict + compact) and the decode attention of that token (work
partition, split-K MFMA decode, log-sum-exp combine), taken through spkv_decode_step (two
launches; --two-call times spkv_append + spkv_decode_attention, three launches, instead).  Inputs are synthetic, seeded and resident in
HBM before the timed region.  The workload is the Llama-3-8B-shaped layer: batch 16,
32 query / 8 KV heads, head_dim 128, context 32768, window 128, tau 0.5, per-head keep
rates U[0.10, 0.33].  Several independent cache instances are rotated so that the working
set is far larger than the 256 MB Infinity Cache and every step reads its K/V from HBM.

Prints ONE JSON line: the metric, its value and unit, the step time, `roofline` (dominant
kernel against the HBM peak) and `cpu_baseline` (the fp64 oracle on a bounded sample).
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2605_14037_amd as spkv  # noqa: E402
from paper_2605_14037_amd.inputs import (TokenStream, Workload, prefill_chunks,  # noqa: E402
                                         to_numpy_f32, workload)

HBM_PEAK_GBPS = 8000.0


PREFILL_TIMING = {}    # filled by build_cache(..., time_prefill=True)


def build_cache(wl: Workload, instance: int, chunk: int, tau=None, oracle=None, oracle_seqs=0,
                time_prefill=False):
    """Prefill one cache instance with its own seeded data; optionally mirror the first
    `oracle_seqs` sequences into an oracle.  With time_prefill the chunks are generated
    first and the bulk appends alone are timed (write path, many tokens per call)."""
    tau = wl.tau if tau is None else tau
    if tau <= 0.0:
        pool = sum(max(0, c + 4096 - wl.window) for c in wl.ctx_lens) * wl.n_kv_heads
    else:
        pool = int(wl.expected_kept_tokens() * 1.08) + wl.batch * wl.n_kv_heads * (chunk + 256)
    cache = spkv.SPKVCache(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim,
                           max_context=max(wl.ctx_lens) + 4096, max_total_kept_tokens=pool,
                           window=wl.window, tau=tau)
    stream = TokenStream(wl, device="cuda", layer=instance)
    if time_prefill:
        chunks = [stream.next_tokens(counts) for counts in prefill_chunks(wl.ctx_lens, chunk)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k, v, f, cu in chunks:
            cache.append(k, v, f, cu)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = cache.stats()
        moved = st.dense_kv_bytes + (st.kept_tokens + st.window_tokens) * 4 * wl.head_dim
        if PREFILL_TIMING and PREFILL_TIMING["ms"] <= dt * 1e3:
            return cache, stream          # keep the faster of the instances timed
        PREFILL_TIMING.update({
            "what": "spkv_append over the whole prompt, inputs resident, chunked (a single pass "
                    "per cache instance: the faster of the last two instances built)",
            "chunk_tokens_per_sequence": chunk, "calls": len(chunks), "ms": dt * 1e3,
            "tokens_per_s": st.total_tokens / dt,
            "GBps_read_new_kv_plus_written_kept": moved / dt / 1e9})
        return cache, stream
    for counts in prefill_chunks(wl.ctx_lens, chunk):
        k, v, f, cu = stream.next_tokens(counts)
        cache.append(k, v, f, cu)
        if oracle is not None:
            n = cu[oracle_seqs]
            oracle.append(to_numpy_f32(k[:n]), to_numpy_f32(v[:n]), to_numpy_f32(f[:n]),
                          cu[:oracle_seqs + 1])
    return cache, stream


MFMA_BF16_PEAK_TFLOPS = 2500.0


def prefill_attention_leg(wl: Workload, chunk: int, timed_calls: int, tau=None, instance=2000):
    """spkv_prefill_attention: the first ctx - timed_calls * chunk tokens of every sequence
    are fed by spkv_append (not timed), the rest in `timed_calls` calls of `chunk` tokens per
    sequence, each timed with events on the launch stream (timed_calls = 0: the whole
    prompt).  Algorithmic flops: 4 D per (query head, attended key) -- q.k and p.v -- with the
    attended keys counted from the gate bits of the same logits (window + gated-on keys at
    least w behind, Eq. 3-4)."""
    tau = wl.tau if tau is None else tau
    ctx = int(min(wl.ctx_lens))
    B, Hkv, D, w = wl.batch, wl.n_kv_heads, wl.head_dim, wl.window
    n_calls = ctx // chunk if timed_calls <= 0 else min(timed_calls, ctx // chunk)
    before = ctx - n_calls * chunk
    if tau <= 0.0:
        pool = B * Hkv * ctx
    else:
        pool = int(B * Hkv * ctx * float(wl.keep.mean()) * 1.1) + B * Hkv * (max(chunk, 4096) + 256)
    cache = spkv.SPKVCache(B, wl.n_q_heads, Hkv, D, max_context=ctx + 64,
                           max_total_kept_tokens=pool, window=w, tau=tau)
    theta = cache.threshold_logit()
    stream = TokenStream(wl, device="cuda", layer=instance)
    gates = []
    done = 0
    while done < before:
        n = min(4096, before - done)
        k, v, f, cu = stream.next_tokens([n] * B)
        cache.append(k, v, f, cu)
        gates.append((f >= theta).view(B, n, Hkv))
        done += n
    calls = []
    for _ in range(n_calls):
        k, v, f, cu = stream.next_tokens([chunk] * B)
        q = stream.next_query(rows=chunk * B)
        calls.append((k, v, f, cache.make_cu(cu), q))
        gates.append((f >= theta).view(B, chunk, Hkv))
    out = torch.empty_like(calls[0][4])
    ws = torch.empty(cache.prefill_workspace_bytes(chunk, chunk * B), dtype=torch.uint8, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_calls + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i, (k, v, f, cu, q) in enumerate(calls):
        cache.prefill_attention(k, v, f, q, cu, workspace=ws, out=out)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(n_calls)]
    st = cache.stats()
    assert st.device_error == 0 and st.total_tokens == B * ctx
    # attended keys of every timed query, per KV head
    cum = torch.cat(gates, dim=1).to(torch.int64).cumsum(dim=1)            # [B, ctx, Hkv]
    t = torch.arange(before, ctx, device="cuda")
    win = torch.clamp(t + 1, max=w).view(1, -1, 1)
    far = torch.where((t >= w).view(1, -1, 1), cum[:, torch.clamp(t - w, min=0), :], 0)
    attended = (win + far).sum(dim=(0, 2)).view(n_calls, chunk).sum(dim=1).double().cpu().numpy()
    flops = attended * 4.0 * D * (wl.n_q_heads // Hkv)
    total_ms = float(sum(ms))
    res = {
        "what": "spkv_prefill_attention: attention of every new token (window or gate, causal) "
                "+ append, chunked; inputs resident",
        "chunk_tokens_per_sequence": chunk, "context_before_timed_calls": before,
        "calls_timed": n_calls, "ms_total": total_ms,
        "ms_per_call_first_last": [ms[0], ms[-1]],
        "tokens_per_s": B * chunk * n_calls / (total_ms * 1e-3),
        "attended_keys_per_query_mean": float(attended.sum() / (B * Hkv * chunk * n_calls)),
        "algorithmic_TFLOP": float(flops.sum() / 1e12),
        "TFLOPs": float(flops.sum() / (total_ms * 1e-3) / 1e12),
        "frac_of_bf16_mfma_peak": float(flops.sum() / (total_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS),
        "TFLOPs_last_call": float(flops[-1] / (ms[-1] * 1e-3) / 1e12),
        "tau": tau,
    }
    cache.close()
    return res


def soft_gated_leg(batch=4, ctx=16384, n_q_heads=32, n_kv_heads=8, head_dim=128, window=128, reps=3):
    """spkv_soft_gated_attention (training-time forward, Eq. 6) on whole sequences: dense
    causal attention with the gate bias; flops = 4 D per (query head, key <= query)."""
    g = torch.Generator(device="cuda").manual_seed(20260514)
    total = batch * ctx
    q = torch.randn(total, n_q_heads, head_dim, generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn(total, n_kv_heads, head_dim, generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn(total, n_kv_heads, head_dim, generator=g, device="cuda").to(torch.bfloat16)
    f = (torch.randn(total, n_kv_heads, generator=g, device="cuda") * 2.0 - 1.0).contiguous()
    cu = [b * ctx for b in range(batch + 1)]
    lib = spkv.load_library()
    ws = torch.empty(int(lib.spkv_soft_gated_workspace_bytes(batch, n_kv_heads, head_dim, window, ctx)),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)
    spkv.soft_gated_attention(q, k, v, f, cu, window=window, out=out, workspace=ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        spkv.soft_gated_attention(q, k, v, f, cu, window=window, out=out, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    flops = 4.0 * head_dim * n_q_heads * batch * (ctx * (ctx + 1) / 2)
    return {"what": "spkv_soft_gated_attention: causal attention with bias log u outside the window",
            "batch": batch, "ctx": ctx, "heads": f"{n_q_heads}q/{n_kv_heads}kv", "head_dim": head_dim,
            "window": window, "ms_per_call": ms, "tokens_per_s": total / (ms * 1e-3),
            "algorithmic_TFLOP": flops / 1e12, "TFLOPs": flops / (ms * 1e-3) / 1e12,
            "frac_of_bf16_mfma_peak": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}


HOST_ISSUE_S = []      # host time spent issuing each timed region (before the final sync)


def timed_steps(caches, steps_in, n_steps, offset, do_append=True, do_decode=True, fused=False):
    """n_steps steps, rotating over the cache instances; returns seconds.  fused: one
    spkv_decode_step per step instead of spkv_append + spkv_decode_attention."""
    R = len(caches)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_steps):
        j = offset + i
        c = caches[j % R]
        k, v, f, cu, q, out = steps_in[j % len(steps_in)]
        if fused:
            c.decode_step(k, v, f, q, out=out)
            continue
        if do_append:
            c.append(k, v, f, cu)
        if do_decode:
            c.decode_attention(q, out=out)
    t1 = time.perf_counter()
    torch.cuda.synchronize()
    HOST_ISSUE_S.append((t1 - t0) / max(1, n_steps))
    return time.perf_counter() - t0


def quick_point(wl, chunk, steps, warmup):
    """Step and split-K kernel time of one workload (rotating cold cache instances)."""
    exp_bytes = (wl.expected_kept_tokens() + wl.batch * wl.n_kv_heads * wl.window) * 4 * wl.head_dim
    R = max(2, int(np.ceil(2.5e9 / exp_bytes)))
    caches, streams = [], []
    for r in range(R):
        c, s = build_cache(wl, r, chunk)
        caches.append(c)
        streams.append(s)
    steps_in = []
    for j in range(32):
        k, v, f, cu = streams[j % R].next_tokens([1] * wl.batch)
        q = streams[j % R].next_query()
        steps_in.append((k, v, f, caches[0].make_cu(cu), q, torch.empty_like(q)))
    timed_steps(caches, steps_in, max(warmup, 2 * R), 0, fused=True)    # every instance has run twice
    dt = timed_steps(caches, steps_in, steps, warmup, fused=True)
    host_us = HOST_ISSUE_S[-1] * 1e6
    stats = [c.stats() for c in caches]
    kept = float(np.mean([s.kept_kv_bytes for s in stats]))
    # the same step forced into one launch (merge and append by the last workgroup of every
    # pair) and into two (the library picks per call by default)
    forced = {}
    for n_launch in (1, 2):
        for c in caches:
            c.set_option(spkv.OPT_STEP_LAUNCHES, n_launch)
        timed_steps(caches, steps_in, max(warmup, R), 0, fused=True)
        forced[n_launch] = timed_steps(caches, steps_in, steps, warmup, fused=True)
    dt_one = forced[1]
    for c in caches:
        c.set_option(spkv.OPT_STEP_LAUNCHES, 0)
        c.set_option(spkv.OPT_SPLIT_ONLY, 1)
    timed_steps(caches, steps_in, max(warmup, R), 0, do_append=False)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        caches[i % R].decode_attention(steps_in[i % 32][4], out=steps_in[i % 32][5])
    e1.record()
    torch.cuda.synchronize()
    kern_us = e0.elapsed_time(e1) / steps * 1e3
    for c in caches:
        c.set_option(spkv.OPT_SPLIT_ONLY, 0)
    # and replayed from a HIP graph (one captured step per cache instance): no host work per call
    graph_us = None
    n_rep = max(1, steps // R)
    if min(c.safe_steps() for c in caches) > n_rep + 2:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for r in range(R):
                k, v, f, cu, q, out = steps_in[r % 32]
                caches[r].decode_step(k, v, f, q, out=out)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_rep):
            for c in caches:
                c.advance(1)
            g.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / (n_rep * R) * 1e6
        del g
    res = {"ctx": max(wl.ctx_lens), "keep": float(wl.keep.mean()), "instances": R,
           "kept_kv_MB": kept / 1e6, "dense_kv_MB": float(np.mean([s.dense_kv_bytes for s in stats])) / 1e6,
           "us_per_step": dt / steps * 1e6, "us_per_step_one_launch": dt_one / steps * 1e6,
           "us_per_step_two_launches": forced[2] / steps * 1e6,
           "us_per_step_graph_replay": graph_us, "host_issue_us": host_us,
           "kernel_us": kern_us,
           "kernel_GBps": kept / kern_us / 1e3, "step_GBps": kept / (dt / steps) / 1e9}
    for c in caches:
        c.close()
    torch.cuda.empty_cache()
    return res


def scaling_sweep(args):
    """Step time against kept bytes at fixed context, and against context at fixed kept
    length (batch 16, 32q/8kv heads, head_dim 128, window 128, tau 0.5)."""
    from paper_2605_14037_amd.inputs import small_workload
    rows = []
    for keep in (0.02, 0.05, 0.10, 0.20, 0.33, 0.50, 1.00):
        wl = small_workload(f"keep{keep}", 16, 32, 8, 128, [32768] * 16, keep, seed=int(keep * 100))
        rows.append(dict(sweep="keep at ctx 32768", **quick_point(wl, args.chunk, 60, 10)))
        print(json.dumps(rows[-1]), flush=True)
    for ctx in (8192, 16384, 32768, 65536, 131072):
        keep = 3264.0 / (ctx - 128)
        wl = small_workload(f"ctx{ctx}", 16, 32, 8, 128, [ctx] * 16, keep, seed=ctx)
        rows.append(dict(sweep="ctx at ~3264 kept pairs per head", **quick_point(wl, args.chunk, 60, 10)))
        print(json.dumps(rows[-1]), flush=True)
    return rows


def predictor_step_leg(caches, steps_in, wl, K):
    """The step with the utility predictor of the paper's appendix (Linear d_model -> 256,
    SiLU, Linear 256 -> H_kv; d_model 4096, random weights, logits centred on the workload's
    mean): spkv_decode_step_predict, and the same predictor as a call of its own followed by
    spkv_decode_step."""
    B, Hkv, DM, DH, R = wl.batch, wl.n_kv_heads, 4096, 256, len(caches)
    g = torch.Generator(device="cuda").manual_seed(wl.seed + 77)
    w1 = (torch.randn(DH, DM, generator=g, device="cuda") / DM ** 0.5).to(torch.bfloat16)
    w2 = (torch.randn(Hkv, DH, generator=g, device="cuda") / (0.36 * DH) ** 0.5).to(torch.bfloat16)
    b1 = torch.zeros(DH, device="cuda")
    b2 = torch.full((Hkv,), float(wl.mu.mean()), device="cuda")
    hs = [torch.randn(B, DM, generator=g, device="cuda").to(torch.bfloat16) for _ in range(8)]
    f = torch.empty(B, Hkv, device="cuda")
    ws = torch.empty(spkv.load_library().spkv_decode_step_predict_workspace_bytes(B, DH),
                     dtype=torch.uint8, device="cuda")
    act = torch.empty(B * DH, dtype=torch.float32, device="cuda")

    def run(n, inside):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            k, v, _, cu, q, out = steps_in[i % len(steps_in)]
            if inside:
                caches[i % R].decode_step_predict(hs[i % 8], w1, b1, w2, b2, k, v, q, out=out,
                                                  util_logits=f, workspace=ws)
            else:
                spkv.utility_logits(hs[i % 8], w1, b1, w2, b2, out=f, workspace=act)
                caches[i % R].decode_step(k, v, f, q, out=out)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    run(max(R, 10), True)
    t_in = run(K, True)
    run(max(R, 10), False)
    t_sep = run(K, False)
    return {"what": f"predictor {DM}->{DH}->{Hkv} + append + decode per step",
            "us_per_step_predictor_inside_the_step": t_in * 1e6,
            "us_per_step_predictor_as_its_own_call": t_sep * 1e6, "steps_timed": K}


def layered_bench(wl, args):
    """The 32-layer configuration: one cache per layer; a step runs, for every layer, the
    utility predictor on the new tokens' hidden states, the append and the decode attention:
    spkv_decode_step_predict.  Also timed: the same predictor as a call of its own, and the
    linear stand-in (logits = h W_l + b, one torch product) before spkv_decode_step.  The
    layers' caches (10.8 GB of kept K/V) are the cold rotation.  Dense baseline: the same loop over
    tau = 0 caches of `dense_layers` layers, scaled to all layers (stated in the output)."""
    Lyr, B, Hkv = wl.n_layers, wl.batch, wl.n_kv_heads
    caches, streams = [], []
    for l in range(Lyr):
        c, s = build_cache(wl, l, args.chunk)
        caches.append(c)
        streams.append(s)
    g = torch.Generator(device="cuda").manual_seed(wl.seed)
    W = [torch.randn(4096, Hkv, generator=g, device="cuda") / 64.0 for _ in range(Lyr)]
    bias = torch.full((B, Hkv), float(wl.mu.mean()), device="cuda")
    ring = []
    for j in range(4):
        per_layer = []
        for l in range(Lyr):
            k, v, _, cu = streams[l].next_tokens([1] * B)
            h = torch.randn(B, 4096, generator=g, device="cuda")
            q = streams[l].next_query()
            per_layer.append((k, v, h, caches[0].make_cu(cu), q, torch.empty_like(q),
                              torch.empty(B, Hkv, device="cuda")))
        ring.append(per_layer)

    # The predictor of the paper's appendix (Linear 4096 -> 256, SiLU, Linear 256 -> H_kv) per
    # layer, random weights; the output layer is rescaled so that the logits of random hidden
    # states have the workload's mean and unit spread (the keep rate of the configuration).
    DH = 256
    mlp = []
    for l in range(Lyr):
        w1 = (torch.randn(DH, 4096, generator=g, device="cuda") / 64.0).to(torch.bfloat16)
        w2 = torch.randn(Hkv, DH, generator=g, device="cuda") / 16.0
        probe = torch.randn(2048, 4096, generator=g, device="cuda").to(torch.bfloat16)
        f0 = spkv.utility_logits(probe, w1, None, w2.to(torch.bfloat16), None)
        w2 = (w2 / f0.std(dim=0)[:, None]).to(torch.bfloat16)
        f1 = spkv.utility_logits(probe, w1, None, w2, None)
        b2 = (float(wl.mu.mean()) - f1.mean(dim=0)).contiguous()
        mlp.append((w1, torch.zeros(DH, device="cuda"), w2, b2))
    hb = [[t[2].to(torch.bfloat16) for t in per_layer] for per_layer in ring]
    pws = torch.empty(spkv.load_library().spkv_decode_step_predict_workspace_bytes(B, DH),
                      dtype=torch.uint8, device="cuda")
    act_ws = torch.empty(B * DH, dtype=torch.float32, device="cuda")

    def run(cs, n_steps, offset, layers, mode="linear"):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_steps):
            for l in range(layers):
                k, v, h, cu, q, out, f = ring[(offset + i) % 4][l]
                if mode == "linear":        # stand-in predictor: one torch product per layer
                    torch.addmm(bias, h, W[l], out=f)
                    cs[l].decode_step(k, v, f, q, out=out)
                elif mode == "mlp_separate":
                    w1, b1, w2, b2 = mlp[l]
                    spkv.utility_logits(hb[(offset + i) % 4][l], w1, b1, w2, b2, out=f, workspace=act_ws)
                    cs[l].decode_step(k, v, f, q, out=out)
                else:                       # the predictor inside the step's two launches
                    w1, b1, w2, b2 = mlp[l]
                    cs[l].decode_step_predict(hb[(offset + i) % 4][l], w1, b1, w2, b2, k, v, q,
                                              out=out, util_logits=f, workspace=pws)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n_steps

    W_, K_ = max(2, args.warmup // 10), max(5, args.steps // 10)
    run(caches, W_, 0, Lyr)
    dt_linear = run(caches, K_, W_, Lyr)
    run(caches, 1, 0, Lyr, "mlp_separate")
    dt_sep = run(caches, K_, 1, Lyr, "mlp_separate")
    run(caches, 1, 0, Lyr, "fused")
    dt = run(caches, K_, 1, Lyr, "fused")
    # The same step captured once into a HIP graph (all layers) and replayed: no per-launch
    # host work, no gaps between the 2 x layers launches.
    graph_us = None
    n_rep = K_
    if min(c.safe_steps() for c in caches) > n_rep + 1:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for l in range(Lyr):
                k, v, h, cu, q, out, f = ring[0][l]
                w1, b1, w2, b2 = mlp[l]
                caches[l].decode_step_predict(hb[0][l], w1, b1, w2, b2, k, v, q, out=out,
                                              util_logits=f, workspace=pws)
        graph.replay()                       # the step the captured calls accounted for
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_rep):
            for c in caches:
                c.advance(1)
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / n_rep * 1e6
        del graph
    for c in caches:
        c.set_option(spkv.OPT_SPLIT_ONLY, 1)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for l in range(Lyr):
        caches[l].decode_attention(ring[0][l][4], out=ring[0][l][5])
    e0.record()
    for i in range(K_):
        for l in range(Lyr):
            caches[l].decode_attention(ring[i % 4][l][4], out=ring[i % 4][l][5])
    e1.record()
    torch.cuda.synchronize()
    kern_us = e0.elapsed_time(e1) / (K_ * Lyr) * 1e3
    for c in caches:
        c.set_option(spkv.OPT_SPLIT_ONLY, 0)
    stats = [c.stats() for c in caches]
    kept = float(sum(s.kept_kv_bytes for s in stats))
    dense_bytes = float(sum(s.dense_kv_bytes for s in stats))
    arena = float(sum(s.arena_bytes for s in stats))
    dense = None
    if not args.no_dense:
        DL = 8
        dcs = [build_cache(wl, 1000 + l, args.chunk, tau=0.0)[0] for l in range(DL)]
        run(dcs, 1, 0, DL, "fused")
        ddt = run(dcs, max(3, K_ // 2), 1, DL, "fused")
        dense = {"what": f"same loop over tau = 0 caches of {DL} layers, scaled x{Lyr // DL} to {Lyr} layers",
                 "us_per_step": ddt * Lyr / DL * 1e6, "kv_bytes_per_step": dense_bytes,
                 "GBps": dense_bytes / (ddt * Lyr / DL) / 1e9, "speedup_of_spkv": ddt * Lyr / DL / dt}
        for c in dcs:
            c.close()
    result = {
        "metric": "sp-kv decode step (append + decode attention): achieved HBM GB/s on kept-KV bytes",
        "value": kept / dt / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": K_, "warmup": W_,
        "ms_per_step": dt * 1e3, "us_per_step": dt * 1e6, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {Lyr} layers x (batch {B}, {wl.n_q_heads}q/{Hkv}kv heads, "
                               f"head_dim {wl.head_dim}, ctx {max(wl.ctx_lens)}, window {wl.window}, "
                               f"tau {wl.tau}), utility predictor 4096->{DH}->{Hkv} per layer, inside the step",
                   "kept_kv_bytes_per_step": kept, "dense_kv_bytes_per_step": dense_bytes,
                   "cache_arena_bytes": arena,
                   "density_evicted": float(np.mean([s.density_evicted for s in stats]))},
        "frac_of_hbm_peak_step": kept / dt / 1e9 / HBM_PEAK_GBPS,
        "step_entry": "spkv_decode_step_predict (predictor + append + decode, 2 launches per layer)",
        "other_predictor_paths": {
            "mlp_by_spkv_utility_logits_then_decode_step": {"us_per_step": dt_sep * 1e6,
                                                            "GBps": kept / dt_sep / 1e9},
            "linear_stand_in_by_torch_then_decode_step": {"us_per_step": dt_linear * 1e6,
                                                          "GBps": kept / dt_linear / 1e9}},
        "hip_graph_replay": None if graph_us is None else {
            "what": "the same step captured once (all layers) and replayed; host bookkeeping by "
                    "spkv_cache_advance", "us_per_step": graph_us, "replays_timed": n_rep,
            "GBps": kept / (graph_us * 1e-6) / 1e9,
            "frac_of_hbm_peak_step": kept / (graph_us * 1e-6) / 1e9 / HBM_PEAK_GBPS},
        "dense_cache": dense,
        "roofline": {"bound": "hbm", "kernel": "spkv_decode_split<128>",
                     "achieved": kept / Lyr / kern_us / 1e3, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": kept / Lyr / kern_us / 1e3 / HBM_PEAK_GBPS, "traffic": None,
                     "algorithmic_bytes_per_launch": kept / Lyr, "kernel_avg_us": kern_us,
                     "launches_timed": K_ * Lyr,
                     "timing": "HIP events around back-to-back launches of the split-K kernel alone"},
        "cpu_baseline": None,
    }
    print(json.dumps(result))


def read_traffic_summary(wl_name):
    """HBM bytes per launch of the decode kernel of this workload from the committed rocprofv3
    --pmc summary (FETCH_SIZE / WRITE_SIZE scaled by a copy kernel of known size); None when
    no summary of this workload is committed."""
    path = os.path.join(ROOT, "profiles", f"decode_step_{wl_name}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, oracle, q, seqs, kept_bytes_sample, repeats=2):
    from oracle.spkv_oracle import SPKVOracle  # noqa: F401  (the oracle is only used here)
    workers = max(1, min(16, os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16"))))
    qn = to_numpy_f32(q[:seqs])
    best = None
    for _ in range(repeats):
        t0 = time.perf_counter()
        oracle.decode(qn, workers=workers)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    return {
        "value": kept_bytes_sample / best / 1e9, "unit": "GB/s", "cores": workers,
        "kind": "oracle",
        "sample": (f"fp64 oracle (numpy, {workers} threads over (sequence, KV head) pairs), one decode "
                   f"step (attention over the dense history under the explicit mask) for the first "
                   f"{seqs} of {wl.batch} sequences x {wl.n_kv_heads} KV heads of instance 0, best of "
                   f"{repeats}; GB/s counts the same kept-KV bytes as the GPU figure for those sequences"),
        "seconds_per_step_sample": best,
        "us_per_step_extrapolated_from_sample_x%d" % (wl.batch // seqs): best * wl.batch / seqs * 1e6,
    }


def events_per_launch(fn, n):
    """Average milliseconds of n calls of fn issued back to back, by HIP events on the
    launch stream (torch's current stream is the stream the binding launches on)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def read_ceiling_leg(nbytes, n_workgroups, launches):
    """A plain streaming read (spkv_debug_read) of the same number of bytes, in scattered 32 KB
    runs (the cache's page size), by as many one-wave workgroups as the decode launch has work
    items, back to back over a region of at least 3 GiB (twice the bytes of a launch) so that
    every launch reads cold memory."""
    run_bytes = 32768
    region = max(3 << 30, (2 * int(nbytes) + (1 << 30)) // run_bytes * run_bytes)
    src = torch.empty(region, dtype=torch.uint8, device="cuda")
    src.zero_()
    sink = torch.empty(max(1, n_workgroups) * 1024, dtype=torch.uint8, device="cuda")
    total_runs = region // run_bytes
    n_runs = max(1, min(int(nbytes) // run_bytes, total_runs // 2))
    state = {"first": 0}

    def launch(_):
        spkv.debug_read(src, run_bytes, state["first"], n_runs, 1000003, n_workgroups, sink)
        state["first"] = (state["first"] + n_runs) % (total_runs - n_runs)

    for i in range(5):
        launch(i)
    ms = events_per_launch(launch, launches)
    del src, sink          # (no empty_cache here: handing gigabytes back to the driver right before
    #                         the next timed leg was measured to slow that leg by 3-4 %)
    gbps = n_runs * run_bytes / (ms * 1e-3) / 1e9
    return {"what": "spkv_debug_read: non-temporal 16 KB chunk reads in scattered 32 KB runs, one-wave "
                    "workgroups, no arithmetic; same bytes and workgroup count as the decode launch",
            "bytes_per_launch": n_runs * run_bytes, "workgroups": n_workgroups, "us_per_launch": ms * 1e3,
            "GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS, "launches_timed": launches}


def decode_leg(wl, args, K, W, with_dense=True, cpu_seqs=0, keep_caches=False, cpu_repeats=2):
    """One workload through the decode path: fused step (host clock and HIP events), the same
    step replayed from a HIP graph, the split-K part alone, the other launch count, the read
    ceiling, the dense-cache baseline and the CPU oracle.  Kept bytes are counted right before
    and right after the timed steps (mean of the two)."""
    exp_bytes = (wl.expected_kept_tokens() + wl.batch * wl.n_kv_heads * wl.window) * 4 * wl.head_dim
    R = args.instances or max(2, int(np.ceil(2.5e9 / exp_bytes)))
    cpu_seqs = min(cpu_seqs, max(1, wl.batch // 4))      # a bounded sample: a quarter of the batch at most
    oracle = None
    if cpu_seqs > 0:
        from oracle.spkv_oracle import SPKVOracle
        oracle = SPKVOracle(cpu_seqs, wl.n_q_heads, wl.n_kv_heads, wl.head_dim,
                            window=wl.window, tau=wl.tau)
    caches, streams = [], []
    for r in range(R):
        c, s = build_cache(wl, r, args.chunk, oracle=oracle if r == 0 else None,
                           oracle_seqs=cpu_seqs, time_prefill=(keep_caches and r >= max(1, R - 2)))
        if args.item_target:
            c.set_option(spkv.OPT_ITEM_TARGET, args.item_target)
        if args.merge_waves:
            c.set_option(spkv.OPT_MERGE_WAVES, args.merge_waves)
        if args.step_launches:
            c.set_option(spkv.OPT_STEP_LAUNCHES, args.step_launches)
        caches.append(c)
        streams.append(s)

    # Per-step inputs, resident before timing (a ring of distinct steps).
    steps_in = []
    for j in range(max(64, R)):
        k, v, f, cu = streams[j % R].next_tokens([1] * wl.batch)
        q = streams[j % R].next_query()
        steps_in.append((k, v, f, caches[0].make_cu(cu), q, torch.empty_like(q)))

    fused = not args.two_call
    timed_steps(caches, steps_in, max(W, 2 * R), 0, fused=fused)        # every instance has run twice
    before = [c.stats() for c in caches]
    dt = timed_steps(caches, steps_in, K, W, fused=fused)
    after = [c.stats() for c in caches]
    host_issue_us = HOST_ISSUE_S[-1] * 1e6
    assert all(s.device_error == 0 for s in after)
    kept_bytes = float(np.mean([s.kept_kv_bytes for s in before + after]))
    dense_bytes = float(np.mean([s.dense_kv_bytes for s in before + after]))
    density = float(np.mean([s.density_evicted for s in after]))
    work_items = int(after[0].n_work_items)

    # K back-to-back steps between two HIP events on the launch stream.  (One event pair per
    # launch would put a ~5 us barrier packet in front of every kernel.)
    def step(i):
        k, v, f, cu, q, out = steps_in[i % len(steps_in)]
        caches[i % R].decode_step(k, v, f, q, out=out)
    for i in range(R):
        step(i)
    Kk = max(K, 100)       # the legs below time single kernels: enough launches for a stable mean
    step_events_ms = events_per_launch(step, Kk)

    # both launch counts forced (the default picks per call), and the split-K part alone
    forced = {}
    for n_launch in (1, 2):
        for c in caches:
            c.set_option(spkv.OPT_STEP_LAUNCHES, n_launch)
        timed_steps(caches, steps_in, max(W, R), 0, fused=True)
        forced[n_launch] = timed_steps(caches, steps_in, K, W, fused=True) / K * 1e6
    for c in caches:
        c.set_option(spkv.OPT_STEP_LAUNCHES, args.step_launches)
        c.set_option(spkv.OPT_SPLIT_ONLY, 1)
    timed_steps(caches, steps_in, max(W, R), 0, do_append=False)
    split_ms = events_per_launch(
        lambda i: caches[i % R].decode_attention(steps_in[i % len(steps_in)][4],
                                                 out=steps_in[i % len(steps_in)][5]), Kk)
    for c in caches:
        c.set_option(spkv.OPT_SPLIT_ONLY, 0)

    # With two launches per step the dominant kernel is the split-K launch, timed alone above;
    # with one launch it is the step itself.
    kern_avg_ms = step_events_ms if args.step_launches == 1 else split_ms
    achieved = kept_bytes / (kern_avg_ms * 1e-3) / 1e9
    res = {
        "workload": f"{wl.name}: batch {wl.batch}, {wl.n_q_heads}q/{wl.n_kv_heads}kv heads, "
                    f"head_dim {wl.head_dim}, ctx {min(wl.ctx_lens)}..{max(wl.ctx_lens)}, "
                    f"window {wl.window}, tau {wl.tau}, target keep rates "
                    f"{wl.keep.min():.2f}..{wl.keep.max():.2f} ({wl.note})",
        "cache_instances_rotated": R,
        "kept_kv_bytes_per_step": kept_bytes, "dense_kv_bytes_per_step": dense_bytes,
        "density_evicted": density, "work_items": work_items,
        "us_per_step": dt / K * 1e6, "steps_timed": K,
        "GBps_step": kept_bytes / (dt / K) / 1e9,
        "frac_of_hbm_peak_step": kept_bytes / (dt / K) / 1e9 / HBM_PEAK_GBPS,
        "host_issue_us_per_step": host_issue_us,
        "hip_graph_replay": None,
        "us_per_step_forced_one_launch": forced[1], "us_per_step_forced_two_launches": forced[2],
        "roofline": {
            "bound": "hbm",
            "kernel": (f"spkv_decode_split<{wl.head_dim}>: split-K over the kept lists (the first of the "
                       "step's two launches; the second, spkv_combine_append, merges and appends)"
                       if args.step_launches != 1 else
                       f"spkv_decode_split<{wl.head_dim}, step>: split-K + merge + append in one launch"),
            "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": read_traffic_summary(wl.name),
            "algorithmic_bytes_per_launch": kept_bytes,
            "kernel_avg_us": kern_avg_ms * 1e3, "launches_timed": Kk,
            "timing": "HIP events around K back-to-back launches of this kernel alone on the launch stream",
            "us_per_step_by_events": step_events_ms * 1e3,
        },
    }
    ceiling = read_ceiling_leg(kept_bytes, work_items, Kk)
    ceiling["kernel_over_read_ceiling"] = ceiling["us_per_launch"] / (kern_avg_ms * 1e3)
    ceiling["step_over_read_ceiling"] = ceiling["us_per_launch"] / (dt / K * 1e6)
    res["read_ceiling"] = ceiling

    # The same step captured once per cache instance into one HIP graph and replayed: what a
    # serving loop sees when the host's per-call work (argument checks, the capacity bound, the
    # launch itself) is off the path.
    graph = None
    n_rep = max(1, Kk // R)
    if min(c.safe_steps() for c in caches) > n_rep + 2:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for r in range(R):
                k, v, f, cu, q, out = steps_in[r]
                caches[r].decode_step(k, v, f, q, out=out)
        g.replay()                                   # the step the captured calls accounted for
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_rep):
            for c in caches:
                c.advance(1)
            g.replay()
        torch.cuda.synchronize()
        gus = (time.perf_counter() - t0) / (n_rep * R) * 1e6
        graph = {"what": f"one graph of {R} captured steps (one per cache instance), replayed {n_rep} "
                         "times; host bookkeeping by spkv_cache_advance",
                 "us_per_step": gus, "GBps": kept_bytes / gus / 1e3,
                 "frac_of_hbm_peak_step": kept_bytes / gus / 1e3 / HBM_PEAK_GBPS}
        del g      # (last in the leg: giving a graph's memory pool back slows what is timed next)

    res["hip_graph_replay"] = graph

    state = (caches, streams, steps_in, R, dt)
    if not keep_caches:
        for c in caches:
            c.close()
        caches, streams = [], []
        state = None
        torch.cuda.empty_cache()
    if with_dense and not args.no_dense:
        dc, ds = build_cache(wl, 1000, args.chunk, tau=0.0)
        Kd = max(10, K // 4)
        timed_steps([dc], steps_in, 5, 0, fused=fused)
        ddt = timed_steps([dc], steps_in, Kd, 5, fused=fused)
        dst = dc.stats()
        res["dense_cache"] = {
            "what": "same library, tau = 0 (every pair kept): dense-cache decode on the same GPU",
            "us_per_step": ddt / Kd * 1e6, "kv_bytes_per_step": dst.kept_kv_bytes,
            "GBps": dst.kept_kv_bytes / (ddt / Kd) / 1e9,
            "speedup_of_spkv": (ddt / Kd) / (dt / K)}
        dc.close()
        del dc, ds
        torch.cuda.empty_cache()
    res["_oracle"] = (oracle, steps_in[0], cpu_seqs, cpu_repeats)
    return res, state


def finish_cpu(res, wl):
    """CPU baseline of a leg, run after every GPU timing (a long host-only phase lets the GPU
    clocks drop): the oracle mirrors the first sequences of instance 0 up to the end of the
    prefill; give it one more step of instance 0 and time its decode."""
    oracle, step0, cpu_seqs, repeats = res.pop("_oracle")
    if oracle is None:
        res["cpu_baseline"] = None
        return
    k, v, f, cu, q, out = step0
    n = cu[cpu_seqs]
    oracle.append(to_numpy_f32(k[:n]), to_numpy_f32(v[:n]), to_numpy_f32(f[:n]), list(cu[:cpu_seqs + 1]))
    res["cpu_baseline"] = cpu_baseline(wl, oracle, q, cpu_seqs, oracle.stats()["kept_kv_bytes"], repeats)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--configs", default=None,
                    help="further configurations measured into the line's `configs` object, comma "
                         "separated (default: cfg3,cfg4,cfg5 beside cfg2, none beside any other "
                         "workload; cfg5 here is one of its 32 layers); 'none' for none")
    ap.add_argument("--instances", type=int, default=0, help="cache instances to rotate (0 = auto)")
    ap.add_argument("--item-target", type=int, default=0)
    ap.add_argument("--merge-waves", type=int, default=0,
                    help="work items per workgroup of the split-K kernel (0 = chosen per call)")
    ap.add_argument("--step-launches", type=int, default=0,
                    help="kernel launches per step: 1 (merge and append by the last workgroup of "
                         "every pair), 2 (a merge launch), 0 = chosen by the library")
    ap.add_argument("--chunk", type=int, default=1024, help="prefill chunk (tokens per sequence)")
    ap.add_argument("--two-call", action="store_true",
                    help="time spkv_append + spkv_decode_attention as the step instead of the fused "
                         "spkv_decode_step")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the legs beyond the decode step (predictor, multi-token, prefill)")
    ap.add_argument("--cpu-seqs", type=int, default=4)
    ap.add_argument("--scaling", action="store_true",
                    help="run the keep-rate and context sweeps instead of the benchmark")
    ap.add_argument("--prefill", action="store_true",
                    help="run only the prefill-attention leg over the whole prompt "
                         "(--prefill-chunk tokens per sequence per call, --prefill-tau)")
    ap.add_argument("--prefill-chunk", type=int, default=2048)
    ap.add_argument("--prefill-tau", type=float, default=None)
    ap.add_argument("--prefill-calls", type=int, default=0, help="timed calls (0 = whole prompt)")
    ap.add_argument("--soft-gated", action="store_true",
                    help="run only the soft-gated attention forward leg (batch 4 x 16384 tokens)")
    ap.add_argument("--copy-reference", action="store_true",
                    help="run only the plain 1 GiB copy kernel 20 times (profiler calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (every sequence and "
              "KV head is independent, so the path shards by sequence or by head without exchange). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    spkv.load_library()

    if args.copy_reference:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            spkv.debug_copy(dst, src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 20
        print(json.dumps({"copy_reference_bytes_read": 1 << 30, "bytes_written": 1 << 30,
                          "us_per_copy": dt * 1e6, "GBps_read_plus_write": 2 * (1 << 30) / dt / 1e9}))
        return

    if args.scaling:
        scaling_sweep(args)
        return

    if args.soft_gated:
        print(json.dumps({"soft_gated_attention": soft_gated_leg()}))
        return

    wl = workload(args.workload)
    if args.prefill:
        print(json.dumps({"prefill_attention": prefill_attention_leg(
            wl, args.prefill_chunk, args.prefill_calls, tau=args.prefill_tau),
            "config": {"workload": wl.name + ": " + wl.note}}))
        return
    if wl.n_layers > 1:
        layered_bench(wl, args)
        return

    W, K = args.warmup, args.steps
    cpu_seqs = 0 if args.no_cpu else args.cpu_seqs
    extras = not args.no_extras
    res, state = decode_leg(wl, args, K, W, cpu_seqs=cpu_seqs, keep_caches=extras)
    fused = not args.two_call

    extra = {}
    if extras:
        caches, streams, steps_in, R, dt = state
        # the step as two calls (spkv_append + spkv_decode_attention), and its halves
        timed_steps(caches, steps_in, max(W, R, 200), 0, fused=not fused)
        dt_other = timed_steps(caches, steps_in, K, W, fused=not fused)
        dt_dec = timed_steps(caches, steps_in, K, W + K, do_append=False)
        dt_app = timed_steps(caches, steps_in, K, W + 2 * K, do_decode=False)
        # The same step on ONE cache instance, step after step, as a serving loop runs it: what
        # the chip's last-level cache (256 MB) holds of the kept K/V from the step before is not
        # fetched from HBM again.  The headline figure is the cold one (rotation).
        timed_steps(caches[:1], steps_in, max(W, 10), 0, fused=fused)
        dt_hot = timed_steps(caches[:1], steps_in, K, W, fused=fused)
        extra["us_per_step_other_entry"] = dt_other / K * 1e6
        extra["us_per_step_one_instance_warm_cache"] = dt_hot / K * 1e6
        extra["decode_only_us"] = dt_dec / K * 1e6
        extra["append_only_us"] = dt_app / K * 1e6
        extra["step_with_predictor"] = predictor_step_leg(caches, steps_in, wl, K)

        # Multi-token steps: 4 and 16 new tokens per sequence per call, through
        # spkv_decode_chunk and through spkv_prefill_attention (which hands the shortest chunks
        # to the former itself).
        chunk_legs = {}
        for n_tok in (4, 16):
            if n_tok * (wl.n_q_heads // wl.n_kv_heads) > 64:
                continue
            ins = []
            for j in range(2 * R):
                k, v, f, cu = streams[j % R].next_tokens([n_tok] * wl.batch)
                q = streams[j % R].next_query(rows=n_tok * wl.batch)
                ins.append((k, v, f, caches[0].make_cu(cu), q, torch.empty_like(q)))
            ws = torch.empty(caches[0].prefill_workspace_bytes(n_tok, n_tok * wl.batch),
                             dtype=torch.uint8, device="cuda")
            Kc = max(R, K // 8)
            leg = {"calls_timed": Kc}
            for name in ("decode_chunk", "prefill_attention"):
                def call(j):
                    k, v, f, cu, q, o = ins[j % len(ins)]
                    if name == "decode_chunk":
                        caches[j % R].decode_chunk(k, v, f, q, cu, out=o)
                    else:
                        caches[j % R].prefill_attention(k, v, f, q, cu, workspace=ws, out=o)
                for j in range(R):
                    call(j)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for j in range(Kc):
                    call(j)
                torch.cuda.synchronize()
                leg[f"us_per_call_{name}"] = (time.perf_counter() - t0) / Kc * 1e6
            leg["us_per_token_position"] = min(leg["us_per_call_decode_chunk"],
                                               leg["us_per_call_prefill_attention"]) / n_tok
            chunk_legs[f"{n_tok}_tokens_per_sequence"] = leg
        extra["multi_token_step"] = chunk_legs
        extra["prefill_append"] = dict(PREFILL_TIMING)
        for c in caches:
            c.close()
        caches, state = [], None
        del streams
        torch.cuda.empty_cache()
        # Prefill attention: the last two 2048-token chunks of the prompt on a fresh cache.
        if min(wl.ctx_lens) >= 4096:
            extra["prefill_attention"] = prefill_attention_leg(wl, 2048, 2)

    # further configurations, each a decode leg of its own
    names = args.configs
    if names is None:
        names = "cfg3,cfg4,cfg5" if args.workload == "cfg2" else "none"
    others = {}
    other_wl = {}
    if names != "none":
        import dataclasses
        for name in [n for n in names.split(",") if n and n != args.workload]:
            w2 = workload(name)
            label = name
            if w2.n_layers > 1:       # one layer of the layered configuration, gate logits passed in
                w2 = dataclasses.replace(w2, n_layers=1, note=w2.note + "; ONE of its 32 layers")
                label = name + "_one_layer"
            K2 = max(20, K // 2) if w2.expected_kept_tokens() * 4 * w2.head_dim > 1.5e9 else K
            others[label], _ = decode_leg(w2, args, K2, W, cpu_seqs=cpu_seqs, cpu_repeats=1)
            other_wl[label] = w2

    # CPU baselines last
    finish_cpu(res, wl)
    for label, r in others.items():
        finish_cpu(r, other_wl[label])

    result = {
        "metric": "sp-kv decode step (append + decode attention): achieved HBM GB/s on kept-KV bytes",
        "value": res["GBps_step"],
        "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": res["us_per_step"] / 1e3,
        "us_per_step": res["us_per_step"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": res["workload"],
            "cache_instances_rotated": res["cache_instances_rotated"],
            "kept_kv_bytes_per_step": res["kept_kv_bytes_per_step"],
            "dense_kv_bytes_per_step": res["dense_kv_bytes_per_step"],
            "density_evicted": res["density_evicted"],
            "work_items": res["work_items"],
        },
        "step_entry": ("spkv_decode_step (fused append + decode)" if fused else
                       "spkv_append + spkv_decode_attention"),
        "frac_of_hbm_peak_step": res["frac_of_hbm_peak_step"],
        "host_issue_us_per_step": res["host_issue_us_per_step"],
        "hip_graph_replay": res["hip_graph_replay"],
    }
    for key in res:
        if key.startswith("us_per_step_forced_"):
            result[key] = res[key]
    result.update(extra)
    result["dense_cache"] = res.get("dense_cache")
    result["roofline"] = res["roofline"]
    result["read_ceiling"] = res["read_ceiling"]
    result["cpu_baseline"] = res["cpu_baseline"]
    if others:
        result["configs"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
