"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element.

Kept positions, lengths and stats must match bit for bit; outputs within
|gpu - ref| <= 1e-2 + 1e-2 |ref| (bf16 inputs, fp32 accumulation, bf16 output)."""

import numpy as np
import pytest
import torch

import paper_2605_14037_amd as spkv
from oracle.spkv_oracle import SPKVOracle, threshold_logit
from paper_2605_14037_amd.inputs import (TokenStream, small_workload, to_numpy_f32, workload)
from tests import harness as H

pytestmark = pytest.mark.gpu


def test_cfg1_every_step():
    """Config 1: prefill 2048 tokens, then 64 append+decode steps, all checked."""
    m = H.run_workload(workload("cfg1"), chunk=512)
    assert len(m) == 64


@pytest.mark.parametrize("ctx,w", [(1, 128), (5, 128), (127, 128), (128, 128), (129, 128),
                                   (200, 128), (31, 32), (33, 32), (700, 100), (90, 1),
                                   (300, 8), (1000, 512), (64, 64), (65, 64)])
def test_window_edges(ctx, w):
    """T < w, T = w, T = w + 1, windows that are not a multiple of the 32-key half-page."""
    wl = small_workload("edge", 2, 8, 2, 64, [ctx, max(1, ctx // 2)], [[0.5, 0.2]], window=w,
                        decode_steps=3, seed=ctx * 1000 + w)
    H.run_workload(wl, chunk=4096)


@pytest.mark.parametrize("D,Hq,Hkv", [(64, 2, 2), (64, 8, 2), (128, 32, 8), (128, 8, 1),
                                      (128, 16, 1), (64, 16, 2)])
def test_head_shapes(D, Hq, Hkv):
    """head_dim 64 / 128 and group sizes 1, 4, 8, 16."""
    wl = small_workload("heads", 3, Hq, Hkv, D, [900, 130, 417], 0.3, decode_steps=2,
                        seed=D + Hq + Hkv)
    H.run_workload(wl, chunk=512)


@pytest.mark.parametrize("tau,keep", [(0.0, 0.5), (1.0, 0.5), (0.3, 0.5), (0.9, 0.6),
                                      (0.5, 1.0), (0.5, 0.0)])
def test_thresholds_all_and_none(tau, keep):
    """tau <= 0 keeps everything (dense cache), tau >= 1 keeps nothing (window only)."""
    wl = small_workload("tau", 2, 8, 2, 128, [1500, 777], keep, tau=tau, decode_steps=2,
                        seed=int(tau * 100) + int(keep * 10))
    H.run_workload(wl, chunk=1024)


def test_threshold_value_matches_oracle_bits():
    for tau in (0.01, 0.1, 0.3, 0.5, 0.7, 0.9, 0.99, 0.0, 1.0):
        c = spkv.SPKVCache(1, 1, 1, 64, 256, 256, tau=tau)
        assert np.float32(c.threshold_logit()).tobytes() == threshold_logit(tau).tobytes(), tau
        c.close()


def test_gate_equality_is_kept():
    """A logit exactly equal to theta passes the gate (Eq. 2 uses >=)."""
    B, Hq, Hkv, D, w = 1, 1, 1, 64, 4
    T = 40
    g = torch.Generator(device="cuda").manual_seed(5)
    k = torch.randn(T, Hkv, D, generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn(T, Hkv, D, generator=g, device="cuda").to(torch.bfloat16)
    f = torch.full((T, Hkv), -1.0, device="cuda")
    f[3] = 0.0
    f[7] = -0.0
    f[9] = float("nan")
    cache = spkv.SPKVCache(B, Hq, Hkv, D, 64, 64, window=w, tau=0.5)
    oracle = SPKVOracle(B, Hq, Hkv, D, window=w, tau=0.5)
    H.feed(cache, oracle, k, v, f, [0, T])
    assert cache.kept_positions(0, 0) == [3, 7] == oracle.kept_positions(0, 0).tolist()
    q = torch.randn(B, Hq, D, generator=g, device="cuda").to(torch.bfloat16)
    H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0])
    cache.close()


def test_incremental_equals_bulk():
    """Appending one token at a time and in bulk build the same cache."""
    wl = small_workload("inc", 2, 8, 2, 64, [333, 150], 0.4, seed=77)
    stream = TokenStream(wl, device="cuda")
    k, v, f, cu = stream.next_tokens(wl.ctx_lens)
    bulk, inc, mixed = H.make_cache(wl), H.make_cache(wl), H.make_cache(wl)
    bulk.append(k, v, f, cu)
    for step in range(max(wl.ctx_lens)):
        rows = [cu[b] + step for b in range(wl.batch) if step < wl.ctx_lens[b]]
        c = np.concatenate([[0], np.cumsum([1 if step < n else 0 for n in wl.ctx_lens])]).tolist()
        inc.append(k[rows].contiguous(), v[rows].contiguous(), f[rows].contiguous(), c)
    # mixed: ragged chunks of 1, 70, 129, 2, rest
    done = [0, 0]
    for n in (1, 70, 129, 2, 10 ** 6):
        counts = [min(n, wl.ctx_lens[b] - done[b]) for b in range(2)]
        rows = [cu[b] + done[b] + i for b in range(2) for i in range(counts[b])]
        c = [0, counts[0], counts[0] + counts[1]]
        if rows:
            mixed.append(k[rows].contiguous(), v[rows].contiguous(), f[rows].contiguous(), c)
        done = [done[b] + counts[b] for b in range(2)]
    q = stream.next_query()
    outs = [c.decode_attention(q, want_lse=True) for c in (bulk, inc, mixed)]
    oracle = H.make_oracle(wl)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    for c in (bulk, inc, mixed):
        H.check_state(c, oracle, wl)
    for o, l in outs:
        assert torch.equal(o, outs[0][0]) and torch.equal(l, outs[0][1])
    H.check_output(outs[0][0], oracle.decode(to_numpy_f32(q))[0])
    for c in (bulk, inc, mixed):
        c.close()


@pytest.mark.parametrize("w", [128, 40, 300])
def test_bulk_append_chunk_sizes_around_the_launch_paths(w):
    """The bulk append has three launch shapes: one launch (chunks within the window and one
    256-token segment), two (up to 16 segments per sequence: the per-pair stage counts for
    itself), three (longer chunks: a count launch first).  Chunks on both sides of every limit,
    ragged across the batch, windows that are no multiple of 8 or 32 (ring rows written as
    whole 16-byte units only where all eight slots are covered), prefill attention on top."""
    B = 3
    wl = small_workload("paths", B, 8, 2, 128, [0, 0, 0], [[0.35, 0.1]], window=w, seed=900 + w)
    stream = TokenStream(wl, device="cuda")
    plan = [[5, 0, 200], [256, 257, 40], [4096, 1000, 4097], [9000, 0, 3], [1, 4100, 5000],
            [w, w + 1, w - 1], [300, 300, 300]]
    total = [sum(c[b] for c in plan) for b in range(B)]
    cache = spkv.SPKVCache(B, 8, 2, 128, max_context=max(total) + 600,
                           max_total_kept_tokens=sum(total) * 2 + 2000, window=w)
    oracle = H.make_oracle(wl)
    for counts in plan:
        k, v, f, cu = stream.next_tokens(counts)
        H.feed(cache, oracle, k, v, f, cu)
        H.check_state(cache, oracle, wl, label=f"after {counts}")
    counts = [500, 17, 300]                        # a prefill-attention call on the same state
    k, v, f, cu = stream.next_tokens(counts)
    q = stream.next_query(rows=sum(counts))
    out, lse = cache.prefill_attention(k, v, f, q, cu, want_lse=True)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    rows = sorted(set(range(0, sum(counts), 37)) | {sum(counts) - 1, 499, 500, 516, 517})
    ref_out, ref_lse = oracle.decode_chunk(to_numpy_f32(q), counts, rows=set(rows))
    H.check_output(out[rows], ref_out[rows], "prefill rows")
    H.check_lse(lse[rows], ref_lse[rows], "prefill rows")
    H.check_state(cache, oracle, wl, label="after prefill attention")
    k, v, f, cu = stream.next_tokens([1] * B)
    qd = stream.next_query()
    o2, l2 = cache.decode_step(k, v, f, qd, want_lse=True)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    ro, rl = oracle.decode(to_numpy_f32(qd))
    H.check_output(o2, ro, "decode after the chunks")
    H.check_lse(l2, rl, "decode after the chunks")
    cache.close()


def test_sequences_that_skip_a_step():
    """cu_seqlens may give a sequence no token in a step."""
    wl = small_workload("skip", 3, 4, 2, 64, [140, 150, 160], 0.5, seed=3)
    stream = TokenStream(wl, device="cuda")
    cache, oracle = H.make_cache(wl, extra_context=16), H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 64)
    for counts in ([1, 0, 1], [0, 0, 1], [1, 1, 0], [0, 0, 0], [1, 1, 1]):
        k, v, f, cu = stream.next_tokens(counts)
        H.feed(cache, oracle, k, v, f, cu)
        q = stream.next_query()
        H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0], str(counts))
        H.check_state(cache, oracle, wl, label=str(counts))
    cache.close()


def test_peaked_scores():
    """Queries scaled x4: a few keys dominate and outputs are O(1)."""
    wl = small_workload("peaked", 2, 8, 2, 128, [3000, 1000], 0.25, decode_steps=2, seed=9)
    m = H.run_workload(wl, chunk=1024, q_gain=4.0)
    assert all(x["rel_l2"] < H.REL_L2_MAX for x in m)


def test_split_count_invariance():
    """The number of split-K work items does not change indices, and changes outputs only
    by fp32 rounding."""
    wl = small_workload("split", 2, 8, 2, 128, [6000, 2500], 0.3, seed=21)
    stream = TokenStream(wl, device="cuda")
    k, v, f, cu = stream.next_tokens(wl.ctx_lens)
    q = stream.next_query()
    oracle = H.make_oracle(wl)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    ref = oracle.decode(to_numpy_f32(q))[0]
    outs = []
    for target in (1, 2, 7, 64, 4096, 32768, 0):
        cache = H.make_cache(wl)
        cache.set_option(spkv.OPT_ITEM_TARGET, target)
        cache.append(k, v, f, cu)
        out = cache.decode_attention(q)
        st = H.check_state(cache, oracle, wl, label=f"target {target}")
        assert st.n_work_items >= wl.batch * wl.n_kv_heads
        if target == 1:      # the fewest: one workgroup of four one-wave items per pair
            assert st.n_work_items == 4 * wl.batch * wl.n_kv_heads
        H.check_output(out, ref, f"target {target}")
        outs.append(out.float())
        cache.close()
    for o in outs[1:]:
        assert (o - outs[0]).abs().max().item() <= 2e-2 * max(1.0, outs[0].abs().max().item())


@pytest.mark.parametrize("launches", [1, 2])
@pytest.mark.parametrize("merge", [1, 2, 4])
@pytest.mark.parametrize("D,Hq,Hk", [(128, 8, 2), (64, 16, 1), (128, 4, 4)])
def test_every_merge_width_in_every_single_token_entry_point(merge, D, Hq, Hk, launches):
    """One, two or four work items per workgroup (forced; by default the library picks per
    call), merged by the last workgroup of every pair inside the launch or by a second launch:
    plain decode, fused step and step with the predictor against the oracle, with lists
    of 1 to about 60 half-pages so that some workgroups have waves without an item, and with
    item targets from one workgroup per pair to one item per half-page."""
    from oracle.spkv_oracle import utility_logits as oracle_logits
    B = 3
    wl = small_workload("merge", B, Hq, Hk, D, [1900, 40, 700], [[0.9] * Hk, [0.5] * Hk, [0.1] * Hk],
                        seed=300 + merge + D + Hq)
    g = torch.Generator(device="cuda").manual_seed(9)
    dm, dh = 128, 16
    w1 = (torch.randn(dh, dm, generator=g, device="cuda") / dm ** 0.5).to(torch.bfloat16)
    w2 = (torch.randn(Hk, dh, generator=g, device="cuda") / dh ** 0.5).to(torch.bfloat16)
    for target in (1, 13, 32768, 0):
        stream = TokenStream(wl, device="cuda")
        cache = H.make_cache(wl, pool_tokens=(2700 + 64) * Hk + 128 * B * Hk, extra_context=16)
        oracle = H.make_oracle(wl)
        cache.set_option(spkv.OPT_MERGE_WAVES, merge)
        cache.set_option(spkv.OPT_ITEM_TARGET, target)
        cache.set_option(spkv.OPT_STEP_LAUNCHES, launches)
        H.prefill(cache, oracle, stream, wl, 1024)
        for i in range(3):
            k, v, f, cu = stream.next_tokens([1] * B)
            q = stream.next_query()
            if i == 0:
                out, lse = cache.decode_step(k, v, f, q, want_lse=True)
            elif i == 1:
                x = torch.randn(B, dm, generator=g, device="cuda").to(torch.bfloat16)
                out, lse, f = cache.decode_step_predict(x, w1, None, w2, None, k, v, q, want_lse=True)
                ref_f = oracle_logits(to_numpy_f32(x), to_numpy_f32(w1), None, to_numpy_f32(w2), None)
                assert np.abs(f.cpu().numpy() - ref_f).max() <= 1e-4 + 1e-4 * np.abs(ref_f).max()
            else:
                cache.append(k, v, f, cu)
                out, lse = cache.decode_attention(q, want_lse=True)
            oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
            ref_out, ref_lse = oracle.decode(to_numpy_f32(q))
            H.check_output(out, ref_out, f"merge {merge} target {target} step {i}")
            H.check_lse(lse, ref_lse, f"merge {merge} target {target} step {i}")
        st = H.check_state(cache, oracle, wl, label=f"merge {merge} target {target}")
        if target == 1:
            assert st.n_work_items <= merge * B * Hk
        cache.close()
    with pytest.raises(spkv.SPKVError):
        c = H.make_cache(wl)
        try:
            c.set_option(spkv.OPT_MERGE_WAVES, 3)
        finally:
            c.close()


@pytest.mark.parametrize("D,G,Hk", [(128, 1, 2), (128, 2, 3), (128, 3, 1), (128, 4, 2), (128, 8, 1),
                                    (128, 16, 1), (64, 1, 1), (64, 4, 2), (64, 5, 1), (64, 16, 2)])
def test_one_launch_merge_for_every_group_size(D, G, Hk):
    """The merge by the last workgroup of a pair maps threads to the pair's G x D outputs in
    units of eight floats: every group size from 1 to 16 at both head sizes, every merge
    width, from one partial per pair to dozens, sequences that start empty, many consecutive
    fused steps (tickets must be back at zero after every launch), then plain decode."""
    B = 3
    wl = small_workload("onelaunch", B, G * Hk, Hk, D, [2100, 0, 333], [[0.8] * Hk, [0.5] * Hk, [0.2] * Hk],
                        window=48, seed=7 * D + G)
    for merge, target in ((1, 0), (2, 40), (4, 0), (1, 1), (4, 3)):
        stream = TokenStream(wl, device="cuda")
        cache = H.make_cache(wl, extra_context=32)
        oracle = H.make_oracle(wl)
        cache.set_option(spkv.OPT_MERGE_WAVES, merge)
        cache.set_option(spkv.OPT_ITEM_TARGET, target)
        cache.set_option(spkv.OPT_STEP_LAUNCHES, 1)
        H.prefill(cache, oracle, stream, wl, 1024)
        for i in range(12):
            k, v, f, cu = stream.next_tokens([1] * B)
            q = stream.next_query()
            if i < 10:
                out, lse = cache.decode_step(k, v, f, q, want_lse=True)
                oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
            else:
                H.feed(cache, oracle, k, v, f, cu)
                out, lse = cache.decode_attention(q, want_lse=True)
            if i in (0, 1, 5, 9, 10, 11):
                ref_out, ref_lse = oracle.decode(to_numpy_f32(q))
                H.check_output(out, ref_out, f"G {G} merge {merge} target {target} step {i}")
                H.check_lse(lse, ref_lse, f"G {G} merge {merge} target {target} step {i}")
        H.check_state(cache, oracle, wl, label=f"G {G} merge {merge} target {target}")
        cache.close()


@pytest.mark.parametrize("D,Hq,Hk,w", [(128, 8, 2, 64), (64, 4, 2, 16), (128, 16, 1, 128)])
def test_prune_after_raising_the_threshold(D, Hq, Hk, w):
    """Lists filled through every write path (bulk append, single steps, multi-token steps,
    prefill attention), then tau raised and spkv_cache_prune: lengths and positions bit for
    bit, outputs, statistics; the pages given back are used again by what follows; a prune
    under a lowered threshold changes nothing; sink positions survive."""
    B = 3
    wl = small_workload("prune", B, Hq, Hk, D, [1500, 333, 70], 0.6, window=w, seed=83 + D)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=(2300 + 64) * Hk * B, extra_context=900)
    oracle = SPKVOracle(B, Hq, Hk, D, window=w, tau=0.5, n_sink=2)
    cache.set_option(spkv.OPT_SINK_TOKENS, 2)
    G = Hq // Hk

    def step(kind, counts):
        k, v, f, cu = stream.next_tokens(counts)
        q = stream.next_query(rows=sum(counts))
        if kind == "bulk":
            cache.append(k, v, f, cu)
        elif kind == "fused":
            cache.decode_step(k, v, f, q)
        elif kind == "chunk":
            cache.decode_chunk(k, v, f, q, cu)
        else:
            cache.prefill_attention(k, v, f, q, cu)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)

    def check(label):
        st = H.check_state(cache, oracle, wl, label=label)
        q = stream.next_query()
        H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0], label)
        return st

    H.prefill(cache, oracle, stream, wl, 512)
    for _ in range(5):
        step("fused", [1] * B)
    step("chunk", [min(4, w, 64 // G), 2, 1])
    step("prefill", [150, 40, 3])
    before = check("filled")
    # the logits travel with the pairs when the cache moves into a larger arena
    cache.grow(max_context=wl.max_context + 2000, max_total_kept_tokens=(4000 + 64) * Hk * B)
    for tau in (0.7, 0.9):                       # two raises in a row
        cache.set_tau(tau)
        oracle.set_tau(tau)
        cache.prune()
        oracle.prune()
        after = check(f"pruned at tau {tau}")
        assert after.kept_tokens < before.kept_tokens
        before = after
    step("bulk", [300, 10, 200])                 # recycled pages come back into use
    for _ in range(w + 3):
        step("fused", [1] * B)
    check("appends after the prune")
    cache.set_tau(0.3)                           # lowering brings nothing back
    oracle.set_tau(0.3)
    cache.prune()
    oracle.prune()
    st = check("prune under a lower threshold")
    assert st.kept_tokens == before.kept_tokens or st.kept_tokens > 0
    step("prefill", [90, 90, 90])
    cache.set_tau(1.0)                           # everything but the sinks goes
    oracle.set_tau(1.0)
    cache.prune()
    oracle.prune()
    st = check("tau = 1")
    assert st.kept_tokens == 2 * B * Hk
    cache.close()


@pytest.mark.parametrize("D,Hq,Hk,w", [(128, 8, 2, 32), (64, 4, 2, 128), (128, 16, 4, 16), (128, 4, 4, 64)])
def test_score_chunk_then_append_of_the_accepted_drafts(D, Hq, Hk, w):
    """Speculative decoding rounds: spkv_score_chunk returns what spkv_decode_chunk would for
    the drafts and leaves the cache bit for bit as it was; the accepted prefixes then go in by
    spkv_append, and the next round (and a plain decode step) see exactly that cache."""
    import copy
    B = 3
    G = Hq // Hk
    wl = small_workload("spec", B, Hq, Hk, D, [700, 90, 0], 0.4, window=w, seed=61 + D + w)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=(900 + 64) * Hk * B, extra_context=200)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 4096)
    rng = np.random.default_rng(D + w)
    n_cap = min(16, w, 64 // G)
    for rnd in range(6):
        counts = [int(rng.integers(0 if rnd else 1, n_cap + 1)) for _ in range(B)]
        total = sum(counts)
        if total == 0:
            continue
        k, v, f, cu = stream.next_tokens(counts)
        q = stream.next_query(rows=total)
        before = cache.stats(with_kept_len=True)
        out, lse = cache.score_chunk(k, v, q, cu, want_lse=True)
        # the oracle's view: what the outputs would be had the drafts been appended
        trial = copy.deepcopy(oracle)
        trial.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        ref_out, ref_lse = trial.decode_chunk(to_numpy_f32(q), counts)
        H.check_output(out, ref_out, f"round {rnd} {counts}")
        H.check_lse(lse, ref_lse, f"round {rnd} {counts}")
        after = cache.stats(with_kept_len=True)
        assert before[1] == after[1] and before[0].total_tokens == after[0].total_tokens
        H.check_state(cache, oracle, wl, label=f"round {rnd}: cache untouched by scoring")
        # accept a prefix of every sequence's drafts
        acc = [int(rng.integers(0, c + 1)) for c in counts]
        if sum(acc):
            rows = torch.cat([torch.arange(cu[b], cu[b] + acc[b]) for b in range(B)]).to(k.device)
            acu = [0]
            for a in acc:
                acu.append(acu[-1] + a)
            ka, va, fa = k[rows].contiguous(), v[rows].contiguous(), f[rows].contiguous()
            cache.append(ka, va, fa, acu)
            oracle.append(to_numpy_f32(ka), to_numpy_f32(va), to_numpy_f32(fa), acu)
        H.check_state(cache, oracle, wl, label=f"round {rnd}: after accepting {acc}")
    k, v, f, cu = stream.next_tokens([1] * B)
    q = stream.next_query()
    out = cache.decode_step(k, v, f, q)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "decode after the rounds")
    H.check_state(cache, oracle, wl, label="end")
    cache.close()


@pytest.mark.parametrize("D,Hq,Hk", [(128, 8, 2), (64, 4, 1), (128, 16, 1)])
def test_fused_steps_with_many_items_per_pair(D, Hq, Hk):
    """More than 64 partials per (sequence, head) for the longer sequence (one work item per
    half-page and per workgroup): the merges run in 16-wave workgroups (fused step, step with
    the predictor, and the plain decode)."""
    from oracle.spkv_oracle import utility_logits as oracle_logits
    B = 2
    wl = small_workload("wide", B, Hq, Hk, D, [12000, 900], 0.5, seed=77 + D + Hq)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=(12900 + 64) * Hk + 128 * B * Hk, extra_context=16)
    oracle = H.make_oracle(wl)
    cache.set_option(spkv.OPT_ITEM_TARGET, 32768)         # one item per half-page
    cache.set_option(spkv.OPT_MERGE_WAVES, 1)
    H.prefill(cache, oracle, stream, wl, 4096)
    g = torch.Generator(device="cuda").manual_seed(3)
    dm, dh = 256, 32
    w1 = (torch.randn(dh, dm, generator=g, device="cuda") / dm ** 0.5).to(torch.bfloat16)
    w2 = (torch.randn(Hk, dh, generator=g, device="cuda") / dh ** 0.5).to(torch.bfloat16)
    for i in range(6):
        k, v, f, cu = stream.next_tokens([1] * B)
        q = stream.next_query()
        if i % 3 == 0:
            out = cache.decode_step(k, v, f, q)
        elif i % 3 == 1:
            x = torch.randn(B, dm, generator=g, device="cuda").to(torch.bfloat16)
            out, f = cache.decode_step_predict(x, w1, None, w2, None, k, v, q)
            ref_f = oracle_logits(to_numpy_f32(x), to_numpy_f32(w1), None, to_numpy_f32(w2), None)
            assert np.abs(f.cpu().numpy() - ref_f).max() <= 1e-4 + 1e-4 * np.abs(ref_f).max()
        else:
            cache.append(k, v, f, cu)
            out = cache.decode_attention(q)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0], f"step {i}")
        st = H.check_state(cache, oracle, wl, label=f"step {i}")
    assert st.n_work_items > 64 * Hk
    cache.close()


def test_errors_from_the_host_side():
    wl = small_workload("err", 2, 4, 2, 64, [10, 10], 1.0, seed=1)
    stream = TokenStream(wl, device="cuda")
    cache = spkv.SPKVCache(2, 4, 2, 64, max_context=300, max_total_kept_tokens=64, window=16,
                           tau=0.0)
    q = stream.next_query()
    with pytest.raises(spkv.SPKVError) as e:                 # nothing appended yet
        cache.decode_attention(q)
    assert e.value.code == -2
    k, v, f, cu = stream.next_tokens([200, 0])
    with pytest.raises(spkv.SPKVError) as e:                 # 184 pairs pushed out, all kept, pool holds 64 (+1 page/pair)
        cache.append(k, v, f, cu)
    assert e.value.code == -3
    k2, v2, f2, cu2 = stream.next_tokens([301, 1])
    with pytest.raises(spkv.SPKVError) as e:                 # beyond max_context
        cache.append(k2, v2, f2, cu2)
    assert e.value.code == -3
    st = cache.stats()
    assert st.total_tokens == 0 and st.kept_tokens == 0      # failed calls changed nothing
    k3, v3, f3, cu3 = stream.next_tokens([40, 30])
    cache.append(k3, v3, f3, cu3)
    oracle = SPKVOracle(2, 4, 2, 64, window=16, tau=0.0)
    oracle.append(to_numpy_f32(k3), to_numpy_f32(v3), to_numpy_f32(f3), cu3)
    H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0])
    with pytest.raises(ValueError):
        cache.decode_attention(q.float())
    cache.close()


def test_capacity_bound_refreshes_from_device():
    """The host's worst-case bound trips long before the pool is full when few pairs are
    kept; it must then re-read the true lengths instead of refusing."""
    wl = small_workload("cap", 2, 4, 2, 64, [0, 0], 0.1, window=16, seed=4)
    wl.ctx_lens = [4000, 3000]
    stream = TokenStream(wl, device="cuda")
    cache = spkv.SPKVCache(2, 4, 2, 64, max_context=4100, max_total_kept_tokens=4096,
                           window=16, tau=0.5)
    oracle = SPKVOracle(2, 4, 2, 64, window=16, tau=0.5)
    H.prefill(cache, oracle, stream, wl, 256)               # 14k pairs pushed out, ~1.4k kept
    for _ in range(50):
        k, v, f, cu = stream.next_tokens([1, 1])
        H.feed(cache, oracle, k, v, f, cu)
    st = H.check_state(cache, oracle, wl)
    assert st.kept_tokens < 4096
    q = stream.next_query()
    H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0])
    cache.close()


def test_reset_reuses_the_arena():
    wl = small_workload("reset", 2, 8, 2, 64, [500, 300], 0.5, seed=6)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl)
    k, v, f, cu = stream.next_tokens(wl.ctx_lens)
    cache.append(k, v, f, cu)
    cache.reset()
    assert cache.stats().total_tokens == 0
    k, v, f, cu = stream.next_tokens([70, 20])
    oracle = H.make_oracle(wl)
    H.feed(cache, oracle, k, v, f, cu)
    q = stream.next_query()
    H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0])
    H.check_state(cache, oracle, wl)
    cache.close()


def test_medium_ragged_batch():
    """Several pages per head, ragged tails, dense and window-only heads side by side."""
    keep = np.array([[1.0, 0.0, 0.3, 0.05], [0.2, 1.0, 0.0, 0.5], [0.1, 0.1, 0.9, 0.0]])
    wl = small_workload("ragged", 3, 16, 4, 128, [9000, 2049, 4500], keep, decode_steps=3, seed=8)
    H.run_workload(wl, chunk=2048)


@pytest.mark.parametrize("trial", range(24))
def test_random_shapes_and_ragged_appends(trial):
    """Seeded random shapes; appends of 0..300 tokens per sequence in random order, mixed
    with single-token steps; state and outputs checked after every call."""
    rng = np.random.default_rng(1000 + trial)
    B = int(rng.integers(1, 5))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 8]))
    D = int(rng.choice([64, 128]))
    w = int(rng.choice([1, 2, 7, 31, 32, 33, 64, 100, 128, 129, 200]))
    tau = float(rng.choice([0.2, 0.5, 0.8]))
    keep = rng.uniform(0.0, 1.0, size=(B, Hkv))
    wl = small_workload("rand", B, G * Hkv, Hkv, D, [0] * B, keep, window=w, tau=tau,
                        seed=5000 + trial)
    stream = TokenStream(wl, device="cuda")
    cache = spkv.SPKVCache(B, G * Hkv, Hkv, D, max_context=4000, max_total_kept_tokens=4000 * B * Hkv,
                           window=w, tau=tau)
    oracle = H.make_oracle(wl)
    for call in range(int(rng.integers(4, 9))):
        kind = rng.integers(0, 3)
        if kind == 0:
            counts = [1] * B
        elif kind == 1:
            counts = rng.integers(0, 2, size=B).tolist()
        else:
            counts = rng.integers(0, 301, size=B).tolist()
        k, v, f, cu = stream.next_tokens(counts)
        H.feed(cache, oracle, k, v, f, cu)
        H.check_state(cache, oracle, wl, label=f"trial {trial} call {call}")
        if all(oracle.seq_len(b) > 0 for b in range(B)):
            q = stream.next_query()
            out, lse = cache.decode_attention(q, want_lse=True)
            ref_out, ref_lse = oracle.decode(to_numpy_f32(q))
            H.check_output(out, ref_out, f"trial {trial} call {call}")
            H.check_lse(lse, ref_lse, f"trial {trial} call {call}")
    cache.close()


# ------------------------------------------------------------ fused step (two launches)
def test_fused_step_cfg1_every_step():
    m = H.run_workload(workload("cfg1"), chunk=512, fused=True)
    assert len(m) == 64


@pytest.mark.parametrize("ctx,w", [(0, 128), (0, 1), (0, 3), (1, 128), (127, 128), (128, 128),
                                   (129, 128), (31, 32), (64, 33), (300, 1), (300, 2), (700, 100),
                                   (1000, 512)])
def test_fused_step_window_edges(ctx, w):
    """From an empty cache, across the window filling up, and with tiny windows where the
    pair leaving the window is the only ring key."""
    wl = small_workload("fedge", 2, 8, 2, 64, [ctx, ctx // 2], [[0.5, 0.2]], window=w,
                        decode_steps=max(6, 2 * w + 3 if w < 40 else 6), seed=ctx * 1000 + w + 7)
    H.run_workload(wl, chunk=4096, fused=True)


@pytest.mark.parametrize("D,Hq,Hkv", [(64, 2, 2), (128, 32, 8), (128, 16, 1), (64, 24, 3)])
def test_fused_step_head_shapes(D, Hq, Hkv):
    wl = small_workload("fheads", 3, Hq, Hkv, D, [900, 130, 417], 0.3, decode_steps=4,
                        seed=D + Hq + Hkv + 1)
    H.run_workload(wl, chunk=512, fused=True)


def test_fused_and_two_call_steps_build_the_same_cache():
    """Alternating the fused entry point with append + decode_attention leaves the same
    kept positions, lengths and statistics as the two-call path alone."""
    wl = small_workload("fmix", 2, 8, 2, 128, [200, 90], 0.5, window=64, seed=12)
    stream = TokenStream(wl, device="cuda")
    a, bcache = H.make_cache(wl, extra_context=300), H.make_cache(wl, extra_context=300)
    oracle = H.make_oracle(wl)
    k, v, f, cu = stream.next_tokens(wl.ctx_lens)
    a.append(k, v, f, cu)
    bcache.append(k, v, f, cu)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    for step in range(200):
        k, v, f, cu = stream.next_tokens([1, 1])
        q = stream.next_query()
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        a.append(k, v, f, cu)
        out_a = a.decode_attention(q)
        if step % 3 == 0:
            bcache.append(k, v, f, cu)
            out_b = bcache.decode_attention(q)
        else:
            out_b = bcache.decode_step(k, v, f, q)
        assert (out_a.float() - out_b.float()).abs().max().item() <= 2e-2
        if step % 25 == 0 or step == 199:
            H.check_state(a, oracle, wl, label=f"two-call step {step}")
            H.check_state(bcache, oracle, wl, label=f"mixed step {step}")
            H.check_output(out_b, oracle.decode(to_numpy_f32(q))[0], f"mixed step {step}")
    a.close()
    bcache.close()


def test_fused_step_capacity_error_leaves_state():
    cache = spkv.SPKVCache(1, 2, 1, 64, max_context=20, max_total_kept_tokens=64, window=4, tau=0.0)
    wl = small_workload("fcap", 1, 2, 1, 64, [0], 1.0, window=4, seed=2)
    stream = TokenStream(wl, device="cuda")
    for _ in range(20):
        k, v, f, _ = stream.next_tokens([1])
        cache.decode_step(k, v, f, stream.next_query())
    k, v, f, _ = stream.next_tokens([1])
    with pytest.raises(spkv.SPKVError) as e:
        cache.decode_step(k, v, f, stream.next_query())
    assert e.value.code == -3
    st = cache.stats()
    assert st.total_tokens == 20 and st.kept_tokens == 16
    cache.close()


def test_largest_batch():
    """SPKV_MAX_BATCH sequences (cu_seqlens fills the kernel-argument block), 8 KV heads:
    4096 (sequence, head) pairs, ragged lengths around the window."""
    B = 512
    rng = np.random.default_rng(99)
    lens = rng.integers(1, 200, size=B).tolist()
    wl = small_workload("bigbatch", B, 8, 8, 64, lens, 0.4, window=64, decode_steps=2, seed=17)
    H.run_workload(wl, chunk=4096, state_pairs=[(0, 0), (511, 7), (255, 3)])
    H.run_workload(wl, chunk=4096, state_pairs=[(1, 1), (510, 6)], fused=True)


def test_multi_token_step_on_thousands_of_pairs():
    """512 sequences x 17 KV heads = 8704 pairs, group size 1: more pairs than a quarter of
    the work-item slots, the shape at which the partial buffers of the multi-token kernels
    were once too small for one slot per pair."""
    B = 512
    rng = np.random.default_rng(5)
    lens = rng.integers(0, 30, size=B).tolist()
    wl = small_workload("manypairs", B, 17, 17, 64, lens, 0.4, window=8, seed=23)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, extra_context=16)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 4096)
    for counts in ([4] * B, rng.integers(0, 5, size=B).tolist()):
        k, v, f, cu = stream.next_tokens(counts)
        q = stream.next_query(rows=sum(counts))
        out, lse = cache.decode_chunk(k, v, f, q, cu, want_lse=True)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        ref_out, ref_lse = oracle.decode_chunk(to_numpy_f32(q), counts)
        H.check_output(out, ref_out, "chunk")
        H.check_lse(lse, ref_lse, "chunk")
        H.check_state(cache, oracle, wl, [(0, 0), (511, 16), (200, 9), (37, 3)], "chunk")
    cache.close()


def test_partition_follows_the_lengths_over_thousands_of_steps():
    """Every single-token step adds one to the host's upper bound of every long-term length
    although only the keep rate's share is kept.  The work partition is derived from that
    bound, so it must be brought back to the device's lengths now and then (without waiting):
    after 3000 fused steps at keep rate 0.1 the partition of the last call must still cut the
    lists into about as many items as the exact lengths would give."""
    wl = small_workload("drift", 2, 8, 2, 128, [600, 300], 0.1, window=64, seed=77)
    stream = TokenStream(wl, device="cuda")
    n_steps = 3000
    cache = H.make_cache(wl, pool_tokens=2 * 2 * (900 + n_steps), extra_context=n_steps + 8)
    cache.set_option(spkv.OPT_ITEM_TARGET, 24)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 4096)
    ins = []
    for _ in range(8):
        k, v, f, cu = stream.next_tokens([1, 1])
        q = stream.next_query()
        ins.append((k, v, f, cache.make_cu(cu), q, to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu))
    out = torch.empty_like(ins[0][4])
    for i in range(n_steps):
        k, v, f, cuc, q, kn, vn, fn, cu = ins[i % 8]
        cache.decode_step(k, v, f, q, out=out)
        oracle.append(kn, vn, fn, cu)
        if i % 500 == 499:
            torch.cuda.synchronize()
            H.check_output(out, oracle.decode(to_numpy_f32(q))[0], f"step {i}")
    st = H.check_state(cache, oracle, wl, label="after the run")
    assert st.kept_tokens < 0.2 * st.evicted_tokens          # the bound would be 5-10x the truth
    assert st.n_work_items_last_call >= 0.85 * st.n_work_items, (st.n_work_items_last_call, st.n_work_items)
    cache.close()


def test_release_and_reuse_sequences():
    """Continuous batching: sequences finish, their slots are released and refilled; pages
    are recycled (the pool would overflow without it) and every state check stays exact."""
    B, Hq, Hkv, D, w = 3, 8, 2, 128, 32
    wl = small_workload("release", B, Hq, Hkv, D, [0] * B, [[0.9, 0.4]] * B, window=w, seed=33)
    stream = TokenStream(wl, device="cuda")
    # room for about two and a half full sequences of 1500 tokens at these keep rates
    cache = spkv.SPKVCache(B, Hq, Hkv, D, max_context=1600, max_total_kept_tokens=5200,
                           window=w, tau=0.5)
    oracle = H.make_oracle(wl)
    rng = np.random.default_rng(5)

    def pages_in_use(kept):
        return sum((L + 63) // 64 for row in kept for L in row)

    def step(fused):
        k, v, f, cu = stream.next_tokens([1] * B)
        q = stream.next_query()
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        if fused:
            out = cache.decode_step(k, v, f, q)
        else:
            cache.append(k, v, f, cu)
            out = cache.decode_attention(q)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0])

    # fill all three, then release / refill one at a time, eleven times
    for b in range(B):
        counts = [0] * B
        counts[b] = int(rng.integers(600, 1500))
        H.feed(cache, oracle, *stream.next_tokens(counts))
    total_pages_ever = 0
    for cycle in range(11):
        step(fused=cycle % 2 == 0)
        b = cycle % B
        cache.release_sequence(b)
        oracle.release_sequence(b)
        st, kept = cache.stats(with_kept_len=True)
        assert kept[b] == [0] * Hkv and st.pool_pages_used == pages_in_use(kept)
        counts = [0] * B
        counts[b] = int(rng.integers(1, 1500))
        for piece in (counts[b] // 3, counts[b] - counts[b] // 3):      # two ragged bulk calls
            c2 = [0] * B
            c2[b] = piece
            if piece:
                H.feed(cache, oracle, *stream.next_tokens(c2))
        st = H.check_state(cache, oracle, wl, label=f"cycle {cycle}")
        _, kept = cache.stats(with_kept_len=True)
        assert st.pool_pages_used == pages_in_use(kept)
        total_pages_ever += sum((L + 63) // 64 for L in kept[b])
        step(fused=cycle % 2 == 1)
    assert total_pages_ever > st.pool_pages_total        # only recycling made this fit
    with pytest.raises(spkv.SPKVError):
        cache.release_sequence(B)
    cache.close()


@pytest.mark.parametrize("n,dm,dh,Hk", [(16, 4096, 256, 8), (1, 128, 16, 1), (37, 1024, 48, 3),
                                        (64, 4096, 512, 8), (300, 512, 64, 2), (63, 256, 64, 2),
                                        (4096 + 17, 1024, 256, 8), (4200, 128, 512, 5),
                                        (4100, 384, 192, 4), (5000, 256, 1024, 3),
                                        (4096, 4096, 256, 8), (4500, 256, 64, 1), (4096 + 33, 384, 128, 3), (4100, 128, 192, 2)])
def test_utility_predictor(n, dm, dh, Hk):
    """The fused two-layer predictor against the fp64 oracle; and fed into the cache, the
    logits it produces gate exactly like the same fp32 values in the oracle."""
    from oracle.spkv_oracle import utility_logits as oracle_logits
    g = torch.Generator(device="cuda").manual_seed(n + dm + dh)
    x = torch.randn(n, dm, generator=g, device="cuda").to(torch.bfloat16)
    w1 = (torch.randn(dh, dm, generator=g, device="cuda") / dm ** 0.5).to(torch.bfloat16)
    b1 = torch.randn(dh, generator=g, device="cuda")
    w2 = (torch.randn(Hk, dh, generator=g, device="cuda") / dh ** 0.5).to(torch.bfloat16)
    b2 = torch.randn(Hk, generator=g, device="cuda")
    got = spkv.utility_logits(x, w1, b1, w2, b2)
    ref = oracle_logits(to_numpy_f32(x), to_numpy_f32(w1), to_numpy_f32(b1), to_numpy_f32(w2),
                        to_numpy_f32(b2))
    err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
    assert err.max() <= 1e-4 + 1e-4 * np.abs(ref).max(), err.max()       # fp32 accumulation
    got_nb = spkv.utility_logits(x, w1, None, w2, None)
    ref_nb = oracle_logits(to_numpy_f32(x), to_numpy_f32(w1), None, to_numpy_f32(w2), None)
    assert np.abs(got_nb.cpu().numpy() - ref_nb).max() <= 1e-4 + 1e-4 * np.abs(ref_nb).max()
    if n == 16:      # one decode step driven by the predictor's logits
        wl = small_workload("pred", n, 32, Hk, 128, [200] * n, 0.5, window=64, seed=5)
        stream = TokenStream(wl, device="cuda")
        cache, oracle = H.make_cache(wl, extra_context=8), H.make_oracle(wl)
        H.prefill(cache, oracle, stream, wl, 4096)
        k, v, _, cu = stream.next_tokens([1] * n)
        q = stream.next_query()
        out = cache.decode_step(k, v, got, q)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(got), cu)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0])
        H.check_state(cache, oracle, wl)
        cache.close()


@pytest.mark.parametrize("B,Hq,Hk,D,dm,dh,bias", [(16, 32, 8, 128, 4096, 256, True),
                                                   (3, 8, 2, 64, 256, 48, True),
                                                   (33, 16, 4, 128, 1024, 64, False),
                                                   (1, 4, 1, 128, 128, 16, True)])
def test_decode_step_with_the_predictor_inside(B, Hq, Hk, D, dm, dh, bias):
    """spkv_decode_step_predict: the logits it computes and stores match the fp64 predictor
    and the standalone call; fed to the oracle as the fp32 values they are, every later gate
    decision (the window is short, so tokens appended here are pushed out within the test)
    and every output match."""
    from oracle.spkv_oracle import utility_logits as oracle_logits
    w = 16
    ctx = [(37 * b) % 90 for b in range(B)]          # includes an empty sequence
    wl = small_workload("predstep", B, Hq, Hk, D, ctx, 0.5, window=w, seed=B + dm)
    stream = TokenStream(wl, device="cuda")
    steps = w + 12
    pool = sum(c + steps for c in ctx) * Hk + 64 * B * Hk
    cache = H.make_cache(wl, pool_tokens=pool, extra_context=steps + 8)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 4096)
    g = torch.Generator(device="cuda").manual_seed(B * 7 + dh)
    w1 = (torch.randn(dh, dm, generator=g, device="cuda") / dm ** 0.5).to(torch.bfloat16)
    w2 = (2.0 * torch.randn(Hk, dh, generator=g, device="cuda") / dh ** 0.5).to(torch.bfloat16)
    b1 = torch.randn(dh, generator=g, device="cuda") if bias else None
    b2 = 0.3 * torch.randn(Hk, generator=g, device="cuda") if bias else None
    n32 = lambda t: None if t is None else to_numpy_f32(t)
    kept_by_gate = 0
    for i in range(steps):
        x = torch.randn(B, dm, generator=g, device="cuda").to(torch.bfloat16)
        k, v, _, cu = stream.next_tokens([1] * B)
        q = stream.next_query()
        out, lse, f = cache.decode_step_predict(x, w1, b1, w2, b2, k, v, q, want_lse=True)
        ref_f = oracle_logits(to_numpy_f32(x), to_numpy_f32(w1), n32(b1), to_numpy_f32(w2), n32(b2))
        err = np.abs(f.cpu().numpy().astype(np.float64) - ref_f).max()
        assert err <= 1e-4 + 1e-4 * np.abs(ref_f).max(), (i, err)
        alone = spkv.utility_logits(x, w1, b1, w2, b2)
        assert (f - alone).abs().max().item() <= 2e-5 * (1.0 + alone.abs().max().item())
        kept_by_gate += int((f >= 0).sum().item())
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        ref_out, ref_lse = oracle.decode(to_numpy_f32(q))
        H.check_output(out, ref_out, f"step {i}")
        H.check_lse(lse, ref_lse, f"step {i}")
        if i % 5 == 4 or i == steps - 1:
            H.check_state(cache, oracle, wl, label=f"step {i}")
    assert 0 < kept_by_gate < steps * B * Hk             # the gate took both decisions
    # bad shapes are refused before anything is launched
    with pytest.raises(spkv.SPKVError):
        cache.decode_step_predict(x, w1, b1, w2, b2, k, v, q,
                                  workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    H.check_state(cache, oracle, wl, label="after the refused call")
    cache.close()


# ---------------------------------------------------- multi-token step (chunks <= 16)
def _run_chunks(wl, chunk_counts, chunk_prefill=4096, q_gain=1.0):
    stream = TokenStream(wl, device="cuda", q_gain=q_gain)
    cache = H.make_cache(wl, extra_context=sum(max(c) for c in chunk_counts) + 8)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, chunk_prefill)
    for counts in chunk_counts:
        k, v, f, cu = stream.next_tokens(counts)
        q = stream.next_query(rows=sum(counts))
        res = cache.decode_chunk(k, v, f, q, cu, want_lse=True)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        if sum(counts):
            out, lse = res
            ref_out, ref_lse = oracle.decode_chunk(to_numpy_f32(q), counts)
            H.check_output(out, ref_out, f"chunk {counts}")
            H.check_lse(lse, ref_lse, f"chunk {counts}")
        H.check_state(cache, oracle, wl, label=f"chunk {counts}")
    cache.close()


@pytest.mark.parametrize("ctx,w", [(0, 128), (0, 16), (5, 128), (120, 128), (128, 128), (129, 128),
                                   (300, 16), (300, 17), (700, 100), (1000, 512), (64, 33)])
def test_chunk_window_edges(ctx, w):
    wl = small_workload("cedge", 2, 8, 2, 64, [ctx, ctx // 2], [[0.5, 0.2]], window=w,
                        seed=ctx * 100 + w + 3)
    n = min(16, w)
    _run_chunks(wl, [[n, n], [1, n], [n, 0], [3, 7 if w >= 7 else 1], [n, n], [0, 0], [n, 1], [n, n]])


@pytest.mark.parametrize("D,Hq,Hkv,n", [(128, 32, 8, 16), (128, 32, 8, 4), (128, 32, 8, 7),
                                        (64, 8, 8, 16), (64, 4, 2, 16), (128, 16, 2, 8),
                                        (128, 16, 1, 4), (64, 6, 2, 16)])
def test_chunk_head_shapes(D, Hq, Hkv, n):
    """Group sizes 1, 2, 3, 4, 8, 16: one, two or four MFMA column groups."""
    wl = small_workload("cheads", 3, Hq, Hkv, D, [900, 130, 2500], 0.3, seed=D + Hq + n)
    _run_chunks(wl, [[n, n, n], [n, 1, n // 2], [n, n, n]])


def test_chunk_equals_single_steps_state_and_peaked_scores():
    wl = small_workload("cpeak", 2, 8, 2, 128, [3000, 1000], 0.25, seed=19)
    _run_chunks(wl, [[16, 16], [16, 9], [2, 16]], q_gain=4.0)


def test_chunk_rejects_long_chunks():
    cache = spkv.SPKVCache(1, 32, 2, 64, 256, 256, window=8)      # group size 16
    wl = small_workload("cbad", 1, 32, 2, 64, [0], 0.5, window=8, seed=1)
    stream = TokenStream(wl, device="cuda")
    for n in (17, 9, 5):          # > 16 tokens; > window; 5 * 16 > 64 columns
        k, v, f, cu = stream.next_tokens([n])
        with pytest.raises(spkv.SPKVError) as e:
            cache.decode_chunk(k, v, f, stream.next_query(rows=n), cu)
        assert e.value.code == -1
    k, v, f, cu = stream.next_tokens([4])
    cache.decode_chunk(k, v, f, stream.next_query(rows=4), cu)
    assert cache.stats().total_tokens == 4
    cache.close()


# ------------------------------------------------------------- live threshold change
def test_set_tau_between_calls_all_entry_points():
    """tau changed between calls: pairs leave the window under the threshold in force at
    that moment, whichever call pushes them out (single append, bulk append, fused step,
    multi-token step, prefill attention); the oracle keeps the threshold history."""
    wl = small_workload("tauchg", 3, 8, 2, 64, [0, 0, 0], 0.5, window=32, seed=77)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=3 * 2 * 1200, extra_context=1200)
    oracle = H.make_oracle(wl)

    def mirror(k, v, f, cu):
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)

    def check(label):
        H.check_state(cache, oracle, wl, label=label)

    k, v, f, cu = stream.next_tokens([200, 40, 3]); cache.append(k, v, f, cu); mirror(k, v, f, cu)
    check("bulk, tau 0.5")
    for tau in (0.8, 0.2):
        cache.set_tau(tau); oracle.set_tau(tau)
        assert cache.threshold_logit() == float(threshold_logit(tau))
        k, v, f, cu = stream.next_tokens([70, 1, 33]); cache.append(k, v, f, cu); mirror(k, v, f, cu)
        check(f"bulk, tau {tau}")
        for _ in range(3):
            k, v, f, cu = stream.next_tokens([1, 1, 1]); q = stream.next_query()
            cache.append(k, v, f, cu); mirror(k, v, f, cu)
            H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0], f"tau {tau}")
    cache.set_tau(0.6); oracle.set_tau(0.6)
    for _ in range(40):                                    # fused steps push old-threshold pairs out
        k, v, f, cu = stream.next_tokens([1, 1, 1]); q = stream.next_query()
        out = cache.decode_step(k, v, f, q); mirror(k, v, f, cu)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "fused, tau 0.6")
    check("fused, tau 0.6")
    cache.set_tau(0.35); oracle.set_tau(0.35)
    for counts in ([16, 5, 9], [16, 16, 16]):
        k, v, f, cu = stream.next_tokens(counts); q = stream.next_query(rows=sum(counts))
        out = cache.decode_chunk(k, v, f, q, cu); mirror(k, v, f, cu)
        H.check_output(out, oracle.decode_chunk(to_numpy_f32(q), counts)[0], "chunk, tau 0.35")
    check("chunk, tau 0.35")
    cache.set_tau(0.7); oracle.set_tau(0.7)
    counts = [150, 64, 1]
    k, v, f, cu = stream.next_tokens(counts); q = stream.next_query(rows=sum(counts))
    out = cache.prefill_attention(k, v, f, q, cu); mirror(k, v, f, cu)
    H.check_output(out, oracle.decode_chunk(to_numpy_f32(q), counts)[0], "prefill, tau 0.7")
    check("prefill, tau 0.7")
    with pytest.raises(spkv.SPKVError):
        cache.set_tau(float("nan"))
    cache.close()


# ------------------------------------------------------------------ capacity growth
def test_grow_after_capacity_error_continues_exactly():
    """A pool sized for a fraction of the tokens: the append that would overflow it is refused
    before any launch; after spkv_cache_grow the same append succeeds and the cache -- kept
    lists, recycled pages, window, statistics, decode output -- is what the oracle says."""
    wl = small_workload("grow", 3, 8, 2, 128, [0, 0, 0], 0.6, window=64, seed=88)
    stream = TokenStream(wl, device="cuda")
    cache = spkv.SPKVCache(3, 8, 2, 128, max_context=700, max_total_kept_tokens=900, window=64)
    oracle = H.make_oracle(wl)

    def feed(counts):
        k, v, f, cu = stream.next_tokens(counts)
        cache.append(k, v, f, cu)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)

    feed([300, 150, 40])
    cache.release_sequence(1); oracle.release_sequence(1)       # some pages on the free stack
    feed([100, 30, 100])
    H.check_state(cache, oracle, wl, label="before growth")
    k, v, f, cu = stream.next_tokens([290, 290, 290])            # 3 * 2 * 290 more pairs could be kept
    with pytest.raises(spkv.SPKVError) as e:
        cache.append(k, v, f, cu)
    assert e.value.code == -3
    H.check_state(cache, oracle, wl, label="after the refused append")
    with pytest.raises(spkv.SPKVError):                          # limits may not shrink
        cache.grow(max_context=600)
    cache.grow(max_context=4000, max_total_kept_tokens=20000)
    assert cache.stats().pool_pages_total >= 20000 // 64
    H.check_state(cache, oracle, wl, label="right after growth")
    cache.append(k, v, f, cu)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    H.check_state(cache, oracle, wl, label="append after growth")
    for _ in range(3):
        k, v, f, cu = stream.next_tokens([1, 1, 1]); q = stream.next_query()
        out = cache.decode_step(k, v, f, q)
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "decode after growth")
    feed([1500, 0, 2000])                                        # beyond the old max_context
    q = stream.next_query()
    H.check_output(cache.decode_attention(q), oracle.decode(to_numpy_f32(q))[0], "long after growth")
    H.check_state(cache, oracle, wl, label="long after growth")
    cache.close()


# ------------------------------------------------------------------ attention sinks
@pytest.mark.parametrize("n_sink,w", [(4, 32), (1, 128), (40, 16)])
def test_sink_tokens_every_entry_point(n_sink, w):
    """SPKV_OPT_SINK_TOKENS: the first n positions of every sequence are kept whatever their
    logit, through every write path (single, bulk, fused step, multi-token step, prefill) and
    after a sequence slot is reused; keep rate 5 % so that the sinks matter."""
    wl = small_workload("sinks", 3, 8, 2, 64, [0, 0, 0], 0.05, window=w, seed=n_sink * 7 + w)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=3 * 2 * 1500, extra_context=1500)
    cache.set_option(spkv.OPT_SINK_TOKENS, n_sink)
    oracle = SPKVOracle(3, 8, 2, 64, window=w, tau=0.5, n_sink=n_sink)

    def mirror(k, v, f, cu):
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)

    k, v, f, cu = stream.next_tokens([1, 0, 0]); cache.append(k, v, f, cu); mirror(k, v, f, cu)
    with pytest.raises(spkv.SPKVError) as e:                 # only on an empty cache
        cache.set_option(spkv.OPT_SINK_TOKENS, 2)
    assert e.value.code == -2
    for _ in range(w + n_sink + 3):                          # single appends push the sinks out
        k, v, f, cu = stream.next_tokens([1, 1, 0]); q = stream.next_query()
        cache.append(k, v, f, cu); mirror(k, v, f, cu)
    H.check_state(cache, oracle, wl, label="single appends")
    k, v, f, cu = stream.next_tokens([200, 3, 2 * w + n_sink + 9]); cache.append(k, v, f, cu); mirror(k, v, f, cu)
    H.check_state(cache, oracle, wl, label="bulk")
    for _ in range(w + 5):                                   # fused steps
        k, v, f, cu = stream.next_tokens([1, 1, 1]); q = stream.next_query()
        out = cache.decode_step(k, v, f, q); mirror(k, v, f, cu)
        H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "fused")
    H.check_state(cache, oracle, wl, label="fused")
    cache.release_sequence(1); oracle.release_sequence(1)
    n = min(16, w)
    for counts in ([n, n, n], [n, n, 0], [n, n, 3]) * 3:     # the reused slot grows by chunks
        k, v, f, cu = stream.next_tokens(counts); q = stream.next_query(rows=sum(counts))
        out = cache.decode_chunk(k, v, f, q, cu); mirror(k, v, f, cu)
        H.check_output(out, oracle.decode_chunk(to_numpy_f32(q), counts)[0], "chunk")
    H.check_state(cache, oracle, wl, label="chunk")
    cache.release_sequence(2); oracle.release_sequence(2)
    counts = [70, 1, w + n_sink + 50]
    k, v, f, cu = stream.next_tokens(counts); q = stream.next_query(rows=sum(counts))
    out = cache.prefill_attention(k, v, f, q, cu); mirror(k, v, f, cu)
    H.check_output(out, oracle.decode_chunk(to_numpy_f32(q), counts)[0], "prefill")
    st = H.check_state(cache, oracle, wl, label="prefill")
    for b in range(3):
        for h in range(2):
            T = oracle.seq_len(b)
            want = [s for s in range(n_sink) if s <= T - 1 - w]
            assert cache.kept_positions(b, h)[:len(want)] == want
    cache.close()


# ------------------------------------------------------------- replay from a HIP graph
@pytest.mark.parametrize("launches", [1, 2])
def test_decode_step_replayed_from_a_hip_graph(launches):
    """The fused step captured once into a HIP graph and replayed with new inputs in the same
    buffers: every replay (with eager copies, checks and synchronisations between them) must
    equal the oracle's step, the host's bookkeeping is carried by spkv_cache_advance, and the
    number of replays stays inside spkv_cache_safe_steps."""
    wl = small_workload("graph", 3, 8, 2, 128, [700, 300, 40], [[0.4, 0.1]], window=64, seed=61)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl, pool_tokens=3 * 2 * 900, extra_context=200)
    cache.set_option(spkv.OPT_STEP_LAUNCHES, launches)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 4096)

    def next_inputs():
        k, v, f, cu = stream.next_tokens([1, 1, 1])
        return k, v, f, cu, stream.next_query()

    k, v, f, cu, q = next_inputs()                    # one eager step: tightens the host's bound
    out = cache.decode_step(k, v, f, q)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "eager step")

    n_safe = cache.safe_steps()
    assert n_safe == 200 + 1 - 1                      # max_context is the binding limit here
    ks, vs, fs, qs = (torch.empty_like(t) for t in (k, v, f, q))
    outs = torch.empty_like(q)
    k, v, f, cu, q = next_inputs()
    for dst, src in ((ks, k), (vs, v), (fs, f), (qs, q)):
        dst.copy_(src)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                     # records the launches; runs nothing
        cache.decode_step(ks, vs, fs, qs, out=outs)
    n_replays = 70                                    # crosses page boundaries of the short lists
    for i in range(n_replays):
        if i > 0:                                     # the captured call itself counted one step
            k, v, f, cu, q = next_inputs()
            for dst, src in ((ks, k), (vs, v), (fs, f), (qs, q)):
                dst.copy_(src)
            cache.advance(1)
        graph.replay()
        oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
        torch.cuda.synchronize()
        H.check_output(outs, oracle.decode(to_numpy_f32(q))[0], f"replay {i}")
    H.check_state(cache, oracle, wl, label="after the replays")
    assert cache.safe_steps() == n_safe - n_replays
    with pytest.raises(spkv.SPKVError) as e:
        cache.advance(n_safe)                         # more than fits: refused, nothing changes
    assert e.value.code == -3
    k, v, f, cu, q = next_inputs()                    # eager calls go on as before
    out = cache.decode_step(k, v, f, q)
    oracle.append(to_numpy_f32(k), to_numpy_f32(v), to_numpy_f32(f), cu)
    H.check_output(out, oracle.decode(to_numpy_f32(q))[0], "eager step after the replays")
    H.check_state(cache, oracle, wl, label="eager after replays")
    cache.close()
