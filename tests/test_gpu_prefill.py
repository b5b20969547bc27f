"""GPU parity of spkv_prefill_attention (chunks of any length: attention of every new token
under the availability rule of Eq. 3-5, then the append) against the fp64 oracle's
decode_chunk, which takes the masked attention row by row over the dense history."""

import numpy as np
import pytest
import torch

from tests import harness as H
import paper_2605_14037_amd as spkv
from paper_2605_14037_amd.inputs import TokenStream, small_workload, to_numpy_f32

pytestmark = pytest.mark.gpu


def _run_prefill(wl, chunk_counts, pre_chunk=4096, q_gain=1.0, sample=None, seed=0, decode_after=0,
                 shared_workspace=False):
    """Feeds wl.ctx_lens through spkv_append, then every entry of chunk_counts through
    spkv_prefill_attention; compares all rows (or `sample` random rows per call).
    shared_workspace: one workspace, sized once for the longest chunk, serves every call."""
    stream = TokenStream(wl, device="cuda", q_gain=q_gain)
    extra = sum(max(c) for c in chunk_counts) + decode_after + 8
    pool = sum(c + extra for c in wl.ctx_lens) * wl.n_kv_heads      # room for "everything kept"
    cache = H.make_cache(wl, pool_tokens=pool, extra_context=extra)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, pre_chunk)
    rng = np.random.default_rng(seed)
    ws = None
    if shared_workspace:
        n_top = max(max(c) for c in chunk_counts)
        ws = torch.empty(cache.prefill_workspace_bytes(n_top, n_top * wl.batch), dtype=torch.uint8,
                         device="cuda")
    for counts in chunk_counts:
        total = sum(counts)
        k, v, f, cu = stream.next_tokens(counts)
        q = stream.next_query(rows=total)
        res = cache.prefill_attention(k, v, f, q, cu, workspace=ws, want_lse=True)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        if total:
            out, lse = res
            rows = None
            if sample is not None and sample < total:
                # always include the first and last row of every sequence's chunk
                edge = [cu[b] for b in range(wl.batch) if counts[b]] + \
                       [cu[b + 1] - 1 for b in range(wl.batch) if counts[b]]
                rows = sorted(set(rng.choice(total, size=sample, replace=False).tolist() + edge))
            ref_out, ref_lse = oracle.decode_chunk(to_numpy_f32(q), counts,
                                                   rows=None if rows is None else set(rows))
            if rows is None:
                H.check_output(out, ref_out, f"prefill {counts}")
                H.check_lse(lse, ref_lse, f"prefill {counts}")
            else:
                idx = torch.tensor(rows, device=out.device)
                H.check_output(out[idx], ref_out[rows], f"prefill {counts} (sampled rows)")
                H.check_lse(lse[idx], ref_lse[rows], f"prefill {counts} (sampled rows)")
        H.check_state(cache, oracle, wl, label=f"prefill {counts}")
    for _ in range(decode_after):          # the cache left behind decodes like any other
        k, v, f, cu = stream.next_tokens([1] * wl.batch)
        q = stream.next_query()
        out = cache.decode_step(k, v, f, q)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "decode after prefill")
    cache.close()


@pytest.mark.parametrize("ctx,w", [(0, 128), (0, 16), (5, 128), (100, 128), (128, 128), (129, 128),
                                   (300, 16), (300, 17), (700, 100), (64, 33), (1000, 256)])
def test_prefill_window_edges(ctx, w):
    wl = small_workload("pedge", 2, 8, 2, 64, [ctx, ctx // 2], [[0.5, 0.2]], window=w,
                        seed=ctx * 100 + w + 5)
    _run_prefill(wl, [[40, 7], [1, 100], [w, w + 1], [0, 3], [130, 65], [0, 0], [2 * w + 3, 1]],
                 decode_after=2)


@pytest.mark.parametrize("D,Hq,Hkv", [(128, 32, 8), (128, 8, 8), (64, 4, 2), (128, 16, 2),
                                      (128, 16, 1), (64, 6, 2), (64, 32, 2)])
def test_prefill_head_shapes(D, Hq, Hkv):
    """Group sizes 4, 1, 2, 8, 16, 3, 16: 16, 64, 32, 8, 4, 21, 4 tokens per wave."""
    wl = small_workload("pheads", 3, Hq, Hkv, D, [600, 130, 0], 0.3, seed=D + Hq + Hkv)
    _run_prefill(wl, [[150, 64, 300], [65, 1, 17], [20, 260, 129]], sample=96, decode_after=1)


def test_prefill_whole_prompt_from_empty_then_decode():
    wl = small_workload("pwhole", 2, 8, 2, 128, [0, 0], [[0.3, 0.1]], seed=77)
    _run_prefill(wl, [[1500, 700]], sample=160, decode_after=4)


@pytest.mark.parametrize("tau", [0.0, 1.0, 0.3, 0.9])
def test_prefill_thresholds(tau):
    """tau = 0: dense causal attention; tau = 1: sliding window only."""
    wl = small_workload("ptau", 2, 8, 2, 64, [200, 0], 0.5, tau=tau, seed=int(tau * 10) + 40)
    _run_prefill(wl, [[300, 150], [129, 128]], sample=128)


def test_prefill_peaked_scores():
    wl = small_workload("ppeak", 2, 8, 2, 128, [2000, 500], 0.25, seed=23)
    _run_prefill(wl, [[200, 333]], q_gain=4.0, sample=128)


def test_prefill_many_pairs_pinned_mapping():
    """128 (sequence, head) pairs and 512-token chunks: the grid mapping that keeps a pair's
    workgroups on one XCD; ragged chunk lengths leave some spans empty."""
    ctx = [1024 + 37 * b for b in range(16)]
    wl = small_workload("ppin", 16, 32, 8, 128, ctx, 0.2, seed=31)
    counts = [512 - 29 * (b % 5) for b in range(16)]
    _run_prefill(wl, [counts], sample=64)


def test_prefill_same_state_and_outputs_as_chunk_calls():
    """One 48-token prefill call equals three 16-token spkv_decode_chunk calls."""
    wl = small_workload("pcmp", 2, 8, 2, 128, [900, 300], 0.3, seed=5)
    sa, sb = TokenStream(wl, device="cuda"), TokenStream(wl, device="cuda")
    ca, cb = (H.make_cache(wl, pool_tokens=4000, extra_context=64) for _ in range(2))
    H.prefill(ca, None, sa, wl, 4096)
    H.prefill(cb, None, sb, wl, 4096)
    k, v, f, cu = sa.next_tokens([48, 48])
    q = sa.next_query(rows=96)
    out_a = ca.prefill_attention(k, v, f, q, cu)
    kk = k.view(2, 48, 2, 128); vv = v.view(2, 48, 2, 128); ff = f.view(2, 48, 2); qq = q.view(2, 48, 8, 128)
    outs = []
    for j in range(3):
        sl = slice(16 * j, 16 * j + 16)
        outs.append(cb.decode_chunk(kk[:, sl].reshape(32, 2, 128).contiguous(),
                                    vv[:, sl].reshape(32, 2, 128).contiguous(),
                                    ff[:, sl].reshape(32, 2).contiguous(),
                                    qq[:, sl].reshape(32, 8, 128).contiguous(), [0, 16, 32]).view(2, 16, 8, 128))
    out_b = torch.cat(outs, dim=1).reshape(96, 8, 128)
    assert torch.allclose(out_a.float(), out_b.float(), atol=2e-2, rtol=2e-2)
    sta, kla = ca.stats(with_kept_len=True)
    stb, klb = cb.stats(with_kept_len=True)
    assert list(kla) == list(klb) and sta.gate_on_tokens == stb.gate_on_tokens
    for b in range(2):
        for h in range(2):
            assert ca.kept_positions(b, h) == cb.kept_positions(b, h)
    ca.close(); cb.close()


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 8, 128), (16, 8, 128), (32, 8, 128), (8, 2, 64), (6, 2, 128)])
def test_prefill_one_workspace_for_every_chunk_length(Hq, Hkv, D):
    """Chunk lengths across the workgroup shapes (2, 4 or 8 waves of one or two column
    groups) and across the split counts (the lists are long enough to be cut into ranges),
    all in a workspace sized once for the longest chunk."""
    wl = small_workload("pws", 2, Hq, Hkv, D, [2500, 900], 0.6, seed=41 + Hq)
    lens = [520, 300, 130, 70, 40, 33, 24, 17, 12, 7, 5]
    _run_prefill(wl, [[n, max(1, n // 3)] for n in lens], sample=24, seed=Hq, shared_workspace=True)


def test_prefill_calls_with_the_shortest_chunks():
    """One token for every sequence (handed to the fused decode step), one or two tokens for
    some (the multi-token step), then lengths just above the hand-over."""
    wl = small_workload("ptiny", 3, 8, 2, 128, [300, 40, 0], 0.5, seed=23)
    _run_prefill(wl, [[1, 1, 1], [1, 0, 2], [1, 1, 1], [4, 3, 1], [5, 4, 4], [1, 1, 1]])


def test_prefill_rejects_small_workspace_and_leaves_cache_unchanged():
    wl = small_workload("pbad", 1, 8, 2, 64, [0], 0.5, seed=2)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=1000, extra_context=400)
    k, v, f, cu = stream.next_tokens([200])
    q = stream.next_query(rows=200)
    need = cache.prefill_workspace_bytes(200, 200)
    assert need > 0
    # the staging area of this call alone is (64 + 200) rows * 2 heads * 64 * 2 * 2 bytes
    ws = torch.empty(128 * 1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(spkv.SPKVError) as e:
        cache.prefill_attention(k, v, f, q, cu, workspace=ws)
    assert e.value.code == -1
    assert cache.stats().total_tokens == 0
    out = cache.prefill_attention(k, v, f, q, cu, workspace=torch.empty(need, dtype=torch.uint8, device="cuda"))
    assert out.shape == (200, 8, 64) and cache.stats().total_tokens == 200
    assert cache.prefill_attention(k[:0], v[:0], f[:0], q[:0], [0, 0]) is None
    cache.close()
