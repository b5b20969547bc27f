"""Drives the HIP library and the fp64 oracle with the same seeded tensors."""

from __future__ import annotations

import math

import numpy as np
import torch

import paper_2605_14037_amd as spkv
from oracle.spkv_oracle import SPKVOracle
from paper_2605_14037_amd.inputs import TokenStream, prefill_chunks, to_numpy_f32

ATOL, RTOL = 1e-2, 1e-2          # bf16 in / fp32 accumulate tolerance of the benchmark spec
REL_L2_MAX = 6e-3                # bf16 output rounding (2^-9) + bf16 softmax weights (2^-9)


def make_cache(wl, pool_tokens=None, extra_context=0):
    if pool_tokens is None:
        ev = sum(max(0, c + wl.decode_steps - wl.window) for c in wl.ctx_lens) * wl.n_kv_heads
        pool_tokens = ev                                    # worst case: everything kept
    return spkv.SPKVCache(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim,
                          max_context=wl.max_context + extra_context,
                          max_total_kept_tokens=int(pool_tokens), window=wl.window, tau=wl.tau)


def make_oracle(wl):
    return SPKVOracle(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, window=wl.window,
                      tau=wl.tau)


def feed(cache, oracle, k, v, f, cu):
    cache.append(k, v, f, cu)
    if oracle is not None:
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)


def check_output(out_gpu, ref, label=""):
    """Elementwise |gpu - ref| <= ATOL + RTOL |ref| against the unrounded fp64 oracle,
    plus a bound on the relative L2 error so that small outputs cannot hide a gross error."""
    got = out_gpu.detach().to(torch.float32).cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{label}: non-finite output"
    err = np.abs(got - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    rel_l2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
    assert not bad.any(), f"{label}: {int(bad.sum())} elements out of tolerance, max err {err.max():.3e}"
    assert rel_l2 <= REL_L2_MAX, f"{label}: relative L2 error {rel_l2:.3e}"
    return dict(max_abs=float(err.max()), rel_l2=rel_l2)


def check_lse(lse_gpu, ref, label=""):
    got = lse_gpu.detach().cpu().numpy().astype(np.float64)
    err = np.abs(got - np.asarray(ref))
    assert err.max() <= 2e-3 + 1e-3 * np.abs(ref).max(), f"{label}: lse max err {err.max():.3e}"


def check_state(cache, oracle, wl, pairs=None, label=""):
    """Bit-exact long-term lengths for all (seq, head) and positions for `pairs`."""
    st, kept = cache.stats(with_kept_len=True)
    assert st.device_error == 0
    want = oracle.kept_len()
    assert np.array_equal(np.array(kept, dtype=np.int32), want), f"{label}: kept lengths differ"
    if pairs is None:
        pairs = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    for (b, h) in pairs:
        got = cache.kept_positions(b, h)
        assert got == oracle.kept_positions(b, h).tolist(), f"{label}: kept positions differ at {(b, h)}"
    o = oracle.stats()
    for key in ("total_tokens", "evicted_tokens", "window_tokens", "kept_tokens",
                "gate_on_tokens", "kept_kv_bytes", "dense_kv_bytes"):
        assert getattr(st, key) == o[key], f"{label}: stats.{key} {getattr(st, key)} != {o[key]}"
    assert math.isclose(st.density_evicted, o["density_evicted"], rel_tol=1e-12, abs_tol=1e-15)
    assert math.isclose(st.density_all, o["density_all"], rel_tol=1e-12, abs_tol=1e-15)
    return st


def prefill(cache, oracle, stream, wl, chunk):
    for counts in prefill_chunks(wl.ctx_lens, chunk):
        k, v, f, cu = stream.next_tokens(counts)
        feed(cache, oracle, k, v, f, cu)


def run_workload(wl, chunk=4096, q_gain=1.0, check_every=1, pool_tokens=None, item_target=None,
                 state_pairs=None, fused=False):
    """Prefill, then wl.decode_steps steps of append + decode, checking against the oracle.
    fused: use the two-launch spkv_decode_step instead of spkv_append + spkv_decode_attention."""
    stream = TokenStream(wl, device="cuda", q_gain=q_gain)
    cache = make_cache(wl, pool_tokens)
    if item_target is not None:
        cache.set_option(spkv.OPT_ITEM_TARGET, item_target)
    oracle = make_oracle(wl)
    prefill(cache, oracle, stream, wl, chunk)
    check_state(cache, oracle, wl, state_pairs, "after prefill")
    metrics = []
    for step in range(wl.decode_steps):
        k, v, f, cu = stream.next_tokens([1] * wl.batch)
        q = stream.next_query()
        if fused:
            out, lse = cache.decode_step(k, v, f, q, want_lse=True)
            oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        else:
            feed(cache, oracle, k, v, f, cu)
            out, lse = cache.decode_attention(q, want_lse=True)
        if step % check_every == 0 or step == wl.decode_steps - 1:
            ref_out, ref_lse = oracle.decode(to_numpy_f32(q))
            metrics.append(check_output(out, ref_out, f"step {step}"))
            check_lse(lse, ref_lse, f"step {step}")
            check_state(cache, oracle, wl, state_pairs, f"step {step}")
    cache.close()
    return metrics
