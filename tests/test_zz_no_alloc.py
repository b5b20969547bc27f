"""GPU test of spkv_decode_attention_static, the entry point for callers that cannot
allocate: the split-K partials live in a static device array of the library instead of the
cache's arena.  Its output must equal spkv_decode_attention's (and the oracle's) on two calls
in a row, the second on a smaller cache, and shapes beyond the array are refused."""

import numpy as np
import pytest
import torch

import paper_2605_14037_amd as spkv
from paper_2605_14037_amd.inputs import TokenStream, small_workload, to_numpy_f32
from tests import harness as H

pytestmark = pytest.mark.gpu


def _one_cache(batch, Hq, Hkv, D, ctx, keep, seed, merge=0):
    wl = small_workload("static", batch, Hq, Hkv, D, ctx, keep, decode_steps=2, seed=seed)
    stream = TokenStream(wl, device="cuda")
    cache = H.make_cache(wl)
    if merge:
        cache.set_option(spkv.OPT_MERGE_WAVES, merge)
    oracle = H.make_oracle(wl)
    H.prefill(cache, oracle, stream, wl, 1024)
    k, v, f, cu = stream.next_tokens([1] * batch)
    H.feed(cache, oracle, k, v, f, cu)
    q = stream.next_query()
    out_s = torch.full((batch, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse_s = torch.full((batch, Hq), float("nan"), dtype=torch.float32, device="cuda")
    # the lengths have not been read back since the multi-token appends: refused, no wait
    with pytest.raises(spkv.SPKVError) as e:
        cache.decode_attention_static(q, out_s, lse_s)
    assert e.value.code == spkv.binding.E_STATE
    out_a, lse_a = cache.decode_attention(q, want_lse=True)          # existing entry point
    cache.decode_attention_static(q, out_s, lse_s)
    torch.cuda.synchronize()
    ref_out, ref_lse = oracle.decode(to_numpy_f32(q))
    H.check_output(out_s, ref_out, "static vs oracle")
    H.check_lse(lse_s, ref_lse, "static vs oracle")
    H.check_output(out_s, out_a.to(torch.float32).cpu().numpy(), "static vs arena")
    H.check_lse(lse_s, lse_a.cpu().numpy(), "static vs arena")
    H.check_state(cache, oracle, wl, label="state untouched")
    cache.close()
    return out_s, out_a


@pytest.mark.parametrize("merge", [0, 4])
def test_static_scratch_decode_twice_in_a_row_second_call_smaller(merge):
    big_s, big_a = _one_cache(6, 16, 4, 128, [5000, 2600, 900, 130, 64, 3100], 0.3, seed=1, merge=merge)
    small_s, small_a = _one_cache(1, 8, 2, 64, [300], 0.2, seed=2, merge=merge)
    # same kernels, same partition when the array is not the limit: identical bits
    assert torch.equal(big_s, big_a) and torch.equal(small_s, small_a)


def test_static_scratch_refuses_shapes_beyond_the_array():
    # group size 16 at head_dim 128: 16 MiB hold 2016 partial slots, two per pair are needed
    cache = spkv.SPKVCache(512, 32, 2, 128, max_context=64, max_total_kept_tokens=0, window=8)
    q = torch.zeros(512, 32, 128, dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    with pytest.raises(spkv.SPKVError) as e:
        cache.decode_attention_static(q, out)
    assert e.value.code == spkv.binding.E_CAPACITY
    cache.close()
