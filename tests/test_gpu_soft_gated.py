"""GPU parity of spkv_soft_gated_attention (Eq. 6: causal attention with the bias log u on
keys outside the window) against the fp64 oracle."""

import numpy as np
import pytest
import torch

import paper_2605_14037_amd as spkv
from oracle.spkv_oracle import soft_gated_attention as oracle_soft
from paper_2605_14037_amd.inputs import to_numpy_f32
from tests import harness as H

pytestmark = pytest.mark.gpu


def _inputs(counts, Hq, Hkv, D, seed, mu=0.0, sigma=2.0, q_gain=1.0):
    g = torch.Generator(device="cuda").manual_seed(20260514 + seed)
    total = sum(counts)
    q = (torch.randn(total, Hq, D, generator=g, device="cuda") * q_gain).to(torch.bfloat16)
    k = torch.randn(total, Hkv, D, generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn(total, Hkv, D, generator=g, device="cuda").to(torch.bfloat16)
    f = (torch.randn(total, Hkv, generator=g, device="cuda") * sigma + mu).contiguous()
    cu = [0]
    for c in counts:
        cu.append(cu[-1] + c)
    return q, k, v, f, cu


def _check(counts, Hq, Hkv, D, w, seed, rows=None, **kw):
    q, k, v, f, cu = _inputs(counts, Hq, Hkv, D, seed, **kw)
    out, lse = spkv.soft_gated_attention(q, k, v, f, cu, window=w, want_lse=True)
    ref_out, ref_lse = oracle_soft(to_numpy_f32(q), to_numpy_f32(k), to_numpy_f32(v),
                                   to_numpy_f32(f), cu, w)
    H.check_output(out, ref_out, f"soft {counts} w={w}")
    H.check_lse(lse, ref_lse, f"soft {counts} w={w}")


@pytest.mark.parametrize("w", [1, 16, 33, 128, 512])
def test_soft_gated_window_sizes(w):
    _check([300, 1, 77, 0, 130], 8, 2, 64, w, seed=w)


@pytest.mark.parametrize("D,Hq,Hkv", [(128, 32, 8), (128, 8, 8), (64, 4, 2), (128, 16, 2),
                                      (128, 16, 1), (64, 6, 2)])
def test_soft_gated_head_shapes(D, Hq, Hkv):
    _check([257, 64, 400], Hq, Hkv, D, 128, seed=D + Hq + Hkv)


def test_soft_gated_open_shut_and_peaked():
    """Gates fully open (dense causal), shut (sliding window), and peaked scores."""
    _check([500, 200], 8, 2, 128, 64, seed=1, mu=40.0, sigma=0.0)
    _check([500, 200], 8, 2, 128, 64, seed=2, mu=-60.0, sigma=0.0)
    _check([500, 200], 8, 2, 128, 64, seed=3, q_gain=4.0)


def test_soft_gated_many_pairs_long_sequences():
    """128 (sequence, head) pairs (the XCD-pinned grid mapping) and ragged lengths up to 1500."""
    counts = [1500 - 83 * (b % 7) for b in range(16)]
    q, k, v, f, cu = _inputs(counts, 32, 8, 128, seed=9, mu=-1.0)
    out = spkv.soft_gated_attention(q, k, v, f, cu, window=128)
    # oracle on three sequences only (fp64 dense attention is slow)
    for b in (0, 6, 15):
        rows = slice(cu[b], cu[b + 1])
        ref, _ = oracle_soft(to_numpy_f32(q[rows]), to_numpy_f32(k[rows]), to_numpy_f32(v[rows]),
                             to_numpy_f32(f[rows]), [0, counts[b]], 128)
        H.check_output(out[rows], ref, f"soft sequence {b}")
    assert torch.isfinite(out.float()).all()


def test_soft_gated_rejects_bad_arguments():
    q, k, v, f, cu = _inputs([40], 8, 2, 64, seed=4)
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(spkv.SPKVError) as e:
        spkv.soft_gated_attention(q, k, v, f, cu, window=16, workspace=ws)
    assert e.value.code == -1
    with pytest.raises(spkv.SPKVError):
        spkv.soft_gated_attention(q, k, v, f, cu, window=0)
