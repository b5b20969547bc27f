"""Pins for the fp64 oracle (CPU only).

Each pin checks oracle/spkv_oracle.py against something other than itself:
hand-derived fixtures, pure-Python brute force, a library attention routine,
limiting cases and closed forms.  The last test plants mistakes into copies of
the oracle and requires that the pins catch every one of them.
"""

import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle.spkv_oracle import SPKVOracle, threshold_logit

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rational_weight_cases.json")


# --------------------------------------------------------------------- helpers
def _random_problem(rng, B, Hq, Hkv, D, lens, mu=0.0):
    total = sum(lens)
    k = rng.standard_normal((total, Hkv, D))
    v = rng.standard_normal((total, Hkv, D))
    f = (rng.standard_normal((total, Hkv)) + mu).astype(np.float32)
    q = rng.standard_normal((B, Hq, D))
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    return q, k, v, f, cu


def _build(cls, B, Hq, Hkv, D, w, tau, k, v, f, cu, sm_scale=None):
    o = cls(B, Hq, Hkv, D, window=w, tau=tau, sm_scale=sm_scale, store_dtype=np.float64)
    o.append(k, v, f, cu)
    return o


# ------------------------------------------------- pin 1: hand-derived fixtures
def pin_golden(cls):
    for case in json.load(open(GOLDEN)):
        D, T = case["D"], len(case["weights"])
        scale = case["sm_scale"] if case["sm_scale"] is not None else 1.0 / math.sqrt(D)
        k = np.zeros((T, 1, D))
        v = np.zeros((T, 1, D))
        k[:, 0, 0] = [math.log(wt) / scale for wt in case["weights"]]
        v[:, 0, 0] = case["values"]
        f = np.array(case["logits"], np.float32).reshape(T, 1)
        q = np.zeros((1, 1, D))
        q[0, 0, 0] = 1.0
        o = _build(cls, 1, 1, 1, D, case["window"], case["tau"], k, v, f, [0, T],
                   sm_scale=case["sm_scale"])
        out, lse = o.decode(q)
        want = Fraction(*case["out"])
        assert abs(out[0, 0, 0] - float(want)) < 1e-12, case["name"]
        assert np.all(out[0, 0, 1:] == 0.0), case["name"]
        assert abs(lse[0, 0] - math.log(case["lse_exp"])) < 1e-12, case["name"]
        assert o.kept_positions(0, 0).tolist() == case["kept"], case["name"]
        assert o.kept_len().tolist() == [[len(case["kept"])]], case["name"]


# --------------------------------------------------- pin 2: brute force (loops)
def _brute_force(q, k, v, f, cu, Hq, Hkv, D, w, theta, scale):
    """Hand-written loops over the definition: enumerate the available set of
    the newest query of every sequence and sum exp-weighted values."""
    B = len(cu) - 1
    G = Hq // Hkv
    out = [[[0.0] * D for _ in range(Hq)] for _ in range(B)]
    lse = [[0.0] * Hq for _ in range(B)]
    kept = {}
    for b in range(B):
        rows = list(range(cu[b], cu[b + 1]))
        T = len(rows)
        t = T - 1
        for h in range(Hkv):
            avail = []
            kept[(b, h)] = []
            for s in range(T):
                gate_on = float(f[rows[s]][h]) >= float(theta)
                in_win = 0 <= t - s < w
                if gate_on or in_win:
                    avail.append(s)
                if gate_on and not in_win:
                    kept[(b, h)].append(s)
            for g in range(G):
                j = h * G + g
                scores = [scale * math.fsum(q[b][j][d] * k[rows[s]][h][d] for d in range(D))
                          for s in avail]
                mx = max(scores)
                ws = [math.exp(x - mx) for x in scores]
                z = math.fsum(ws)
                for d in range(D):
                    out[b][j][d] = math.fsum(wt * v[rows[s]][h][d]
                                             for wt, s in zip(ws, avail)) / z
                lse[b][j] = mx + math.log(z)
    return np.array(out), np.array(lse), kept


def pin_brute_force(cls):
    rng = np.random.default_rng(7)
    cases = [  # B, Hq, Hkv, D, w, tau, lens
        (1, 1, 1, 4, 1, 0.5, [9]),
        (2, 4, 2, 4, 2, 0.5, [16, 5]),
        (3, 4, 1, 4, 4, 0.3, [3, 4, 13]),
        (2, 6, 3, 4, 4, 0.7, [5, 16]),
        (1, 2, 2, 4, 16, 0.5, [16]),
    ]
    for (B, Hq, Hkv, D, w, tau, lens) in cases:
        q, k, v, f, cu = _random_problem(rng, B, Hq, Hkv, D, lens)
        o = _build(cls, B, Hq, Hkv, D, w, tau, k, v, f, cu)
        out, lse = o.decode(q)
        theta = math.log(float(np.float32(tau)) / (1.0 - float(np.float32(tau))))
        bo, bl, bkept = _brute_force(q.tolist(), k.tolist(), v.tolist(), f.tolist(), cu,
                                     Hq, Hkv, D, w, np.float32(theta), 1.0 / math.sqrt(D))
        np.testing.assert_allclose(out, bo, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse, bl, rtol=1e-12, atol=1e-13)
        for b in range(B):
            for h in range(Hkv):
                assert o.kept_positions(b, h).tolist() == bkept[(b, h)]


# ------------------------- pin 3: library routine under the paper's mask (SDPA)
def _availability(T, w, gate=None):
    """[T, T] boolean matrix of Eq. 3-4 from the distance d = t - s of every (query, key):
    a key is visible iff it is not in the future (d >= 0) and is either inside the window
    (d < w) or gated on.  gate: None (window only) or bool [T] per key."""
    d = np.subtract.outer(np.arange(T), np.arange(T))
    near = (d >= 0) & (d < w)
    if gate is None:
        return near
    return near | ((d >= 0) & np.asarray(gate, bool)[None, :])


def _sdpa_last_row(q_last, k, v, gate, w, scale, Hq, Hkv, mode):
    """Full T x T masked attention with torch's fp64 SDPA for one sequence;
    returns the last query row.  mode: 'gated' (window OR gate, causal),
    'causal' (is_causal=True, no mask tensor), 'window' (banded causal)."""
    T, D = k.shape[0], k.shape[2]
    G = Hq // Hkv
    kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]  # [1,Hq,T,D]
    vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    gen = torch.Generator().manual_seed(1)
    qt = torch.randn(1, Hq, T, D, dtype=torch.float64, generator=gen)
    qt[0, :, T - 1, :] = torch.from_numpy(q_last)
    if mode == "causal":
        o = F.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=scale)
    else:
        if mode == "window":
            mask = torch.from_numpy(_availability(T, w))[None, None].expand(1, Hq, T, T)
        else:
            per_head = np.stack([_availability(T, w, gate[:, j // G]) for j in range(Hq)])
            mask = torch.from_numpy(per_head)[None]
        o = F.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=scale)
    return o[0, :, T - 1, :].numpy()


def pin_sdpa(cls):
    rng = np.random.default_rng(11)
    B, Hq, Hkv, D, w, tau = 2, 8, 2, 16, 8, 0.5
    lens = [50, 23]
    q, k, v, f, cu = _random_problem(rng, B, Hq, Hkv, D, lens, mu=-0.5)
    o = _build(cls, B, Hq, Hkv, D, w, tau, k, v, f, cu)
    out, _ = o.decode(q)
    for b in range(B):
        sl = slice(cu[b], cu[b + 1])
        sig = 1.0 / (1.0 + np.exp(-f[sl].astype(np.float64)))
        ref = _sdpa_last_row(q[b], k[sl], v[sl], sig >= tau, w, 1.0 / math.sqrt(D),
                             Hq, Hkv, "gated")
        np.testing.assert_allclose(out[b], ref, rtol=1e-10, atol=1e-12)


# ------------------------------------------- pin 4: limiting thresholds (tau)
def pin_tau_limits(cls):
    rng = np.random.default_rng(13)
    B, Hq, Hkv, D, w = 2, 4, 2, 8, 4
    lens = [30, 3]
    q, k, v, f, cu = _random_problem(rng, B, Hq, Hkv, D, lens)
    for tau, mode in ((-math.inf, "causal"), (0.0, "causal"), (math.inf, "window"),
                      (1.0, "window")):
        o = _build(cls, B, Hq, Hkv, D, w, tau, k, v, f, cu)
        out, _ = o.decode(q)
        for b in range(B):
            sl = slice(cu[b], cu[b + 1])
            ref = _sdpa_last_row(q[b], k[sl], v[sl], None, w, 1.0 / math.sqrt(D),
                                 Hq, Hkv, mode)
            np.testing.assert_allclose(out[b], ref, rtol=1e-10, atol=1e-12)
        kl = o.kept_len()
        for b in range(B):
            want = max(0, lens[b] - w) if mode == "causal" else 0
            assert kl[b].tolist() == [want] * Hkv
            if mode == "causal":
                assert o.kept_positions(b, 0).tolist() == list(range(want))


# --------------------------------------------------------- pin 5: closed forms
def pin_closed_forms(cls):
    rng = np.random.default_rng(17)
    # (a) all keys identical, V = identity: out reads off the available set.
    T, w = 12, 3
    f = np.array([1, -1, 1, -1, -1, 1, -1, -1, 1, -1, -1, -1], np.float32).reshape(T, 1)
    k = np.ones((T, 1, T)) * 0.25
    v = np.eye(T).reshape(T, 1, T)
    q = rng.standard_normal((1, 2, T))
    o = _build(cls, 1, 2, 1, T, w, 0.5, k, v, f, [0, T])
    out, lse = o.decode(q)
    avail = [0, 2, 5, 8, 9, 10, 11]         # gated {0,2,5,8} plus window {9,10,11}
    want = np.zeros(T)
    want[avail] = 1.0 / len(avail)
    for j in range(2):
        np.testing.assert_allclose(out[0, j], want, rtol=0, atol=1e-15)
        score = (1.0 / math.sqrt(T)) * 0.25 * q[0, j].sum()
        assert abs(lse[0, j] - (score + math.log(len(avail)))) < 1e-12
    assert o.kept_positions(0, 0).tolist() == [0, 2, 5, 8]
    # (b) constant V rows -> that constant, whatever the weights.
    q, k, v, f, cu = _random_problem(rng, 1, 2, 2, 8, [40])
    v[:] = np.linspace(-1, 1, 8)[None, None, :]
    out, _ = _build(cls, 1, 2, 2, 8, 4, 0.5, k, v, f, cu).decode(q)
    np.testing.assert_allclose(out[0, 0], np.linspace(-1, 1, 8), atol=1e-14)
    # (c) one available key with an overwhelming score -> its V row; the same
    #     key gated off and outside the window -> no influence at all.
    q, k, v, f, cu = _random_problem(rng, 1, 1, 1, 8, [20])
    k[5, 0] = 200.0 * q[0, 0] / np.linalg.norm(q[0, 0])
    f[5, 0] = 3.0
    out, _ = _build(cls, 1, 1, 1, 8, 4, 0.5, k, v, f, cu).decode(q)
    np.testing.assert_allclose(out[0, 0], v[5, 0], atol=1e-9)
    f[5, 0] = -3.0
    out_off, _ = _build(cls, 1, 1, 1, 8, 4, 0.5, k, v, f, cu).decode(q)
    k[5, 0] = 0.0
    out_zero, _ = _build(cls, 1, 1, 1, 8, 4, 0.5, k, v, f, cu).decode(q)
    np.testing.assert_array_equal(out_off, out_zero)


# ------------------------------------- pin 6: counting, via the sigmoid domain
def pin_count_invariant(cls):
    rng = np.random.default_rng(19)
    B, Hkv, D, w = 3, 4, 4, 16
    lens = [300, 16, 17]
    for tau in (0.2, 0.5, 0.8):
        q, k, v, f, cu = _random_problem(rng, B, Hkv, Hkv, D, lens)
        o = _build(cls, B, Hkv, Hkv, D, w, tau, k, v, f, cu)
        u = 1.0 / (1.0 + np.exp(-f.astype(np.float64)))          # Eq. 1
        assert np.all(np.abs(u - tau) > 1e-6)                    # no borderline draws
        kl = o.kept_len()
        gate_on = 0
        for b in range(B):
            ub = u[cu[b]:cu[b + 1]]
            n_out = max(0, lens[b] - w)
            for h in range(Hkv):
                z = ub[:, h] >= tau                                  # Eq. 2
                assert kl[b, h] == int(z[:n_out].sum())
                assert o.kept_positions(b, h).tolist() == np.nonzero(z[:n_out])[0].tolist()
                gate_on += int(z.sum())
        st = o.stats()
        assert st["kept_tokens"] == int(kl.sum())
        assert st["gate_on_tokens"] == gate_on
        assert st["evicted_tokens"] == sum(max(0, n - w) for n in lens) * Hkv
        assert st["window_tokens"] == sum(min(n, w) for n in lens) * Hkv
        assert abs(st["density_all"] - gate_on / (sum(lens) * Hkv)) < 1e-15     # Eq. 8
        # the density the text reports: long-term entries over pairs that have left the window
        assert st["density_evicted"] == float(Fraction(int(kl.sum()), st["evicted_tokens"]))
        assert st["kept_kv_bytes"] == (st["kept_tokens"] + st["window_tokens"]) * 4 * D
        assert st["dense_kv_bytes"] == sum(lens) * Hkv * 4 * D


# ------------------------- pin 7: state machine (incremental == bulk, monotone)
def pin_incremental(cls):
    rng = np.random.default_rng(23)
    B, Hq, Hkv, D, w = 2, 4, 2, 4, 4
    lens = [11, 7]
    q, k, v, f, cu = _random_problem(rng, B, Hq, Hkv, D, lens)
    bulk = _build(cls, B, Hq, Hkv, D, w, 0.5, k, v, f, cu)
    inc = cls(B, Hq, Hkv, D, window=w, tau=0.5, store_dtype=np.float64)
    for step in range(max(lens)):
        rows = [cu[b] + step for b in range(B) if step < lens[b]]
        c = [0] + list(np.cumsum([1 if step < lens[b] else 0 for b in range(B)]))
        inc.append(k[rows], v[rows], f[rows], c)
    o1, l1 = bulk.decode(q)
    o2, l2 = inc.decode(q)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    assert bulk.kept_len().tolist() == inc.kept_len().tolist()
    # raising tau keeps a subset
    lo = _build(cls, B, Hq, Hkv, D, w, 0.3, k, v, f, cu)
    hi = _build(cls, B, Hq, Hkv, D, w, 0.7, k, v, f, cu)
    for b in range(B):
        for h in range(Hkv):
            assert set(hi.kept_positions(b, h)) <= set(lo.kept_positions(b, h))


def pin_threshold(cls=None):
    assert threshold_logit(0.5) == np.float32(0.0)
    assert threshold_logit(0.0) == -np.inf and threshold_logit(-1.0) == -np.inf
    assert threshold_logit(1.0) == np.inf and threshold_logit(math.inf) == np.inf
    for tau in (0.01, 0.1, 0.3, 0.7, 0.9, 0.99):
        th = float(threshold_logit(tau))
        assert abs(1.0 / (1.0 + math.exp(-th)) - tau) < 1e-6      # sigmoid(theta) = tau
        assert threshold_logit(tau).dtype == np.float32


PINS = [pin_golden, pin_brute_force, pin_sdpa, pin_tau_limits, pin_closed_forms,
        pin_count_invariant, pin_incremental]


@pytest.mark.parametrize("pin", PINS + [pin_threshold], ids=lambda p: p.__name__)
def test_pin(pin):
    pin(SPKVOracle)


# ----------------------------------------------------------- planted mistakes
class _WindowOffByOne(SPKVOracle):           # window of w+1 keys
    def available(self, b, h):
        T = self.seq_len(b)
        return ((T - 1 - np.arange(T)) <= self.w) | self.gate(b, h)


class _StrictGate(SPKVOracle):               # u > tau instead of u >= tau
    def gate(self, b, h):
        return self._f(b)[:, h] > self.theta


class _NoScale(SPKVOracle):                  # forgets 1/sqrt(d)
    def __init__(self, *a, **kw):
        super().__init__(*a, **kw)
        if kw.get("sm_scale") is None:
            self.scale = 1.0


class _KeptOffByOne(SPKVOracle):             # long-term list one position early
    def kept_positions(self, b, h):
        n = max(0, self.seq_len(b) - self.w + 1)
        return np.nonzero(self.gate(b, h)[:n])[0].astype(np.int32)


class _GateIgnored(SPKVOracle):              # window only
    def available(self, b, h):
        T = self.seq_len(b)
        return (T - 1 - np.arange(T)) < self.w


class _WrongGroup(SPKVOracle):               # query head j reads KV head j % H_kv
    def decode(self, q, workers=1):
        q = np.asarray(q, np.float64)
        perm = [g * self.Hkv + h for h in range(self.Hkv) for g in range(self.G)]
        out, lse = super().decode(q[:, perm, :])
        inv = np.argsort(perm)
        return out[:, inv, :], lse[:, inv]


class _TransposedPV(SPKVOracle):             # weights applied with K instead of V
    def decode_pair(self, b, h, q_bh):
        out, lse = super().decode_pair(b, h, q_bh)
        K = self._k(b)[:, h, :].astype(np.float64)
        V = self._v(b)[:, h, :].astype(np.float64)
        avail = self.available(b, h)
        x = self.scale * (K @ q_bh.T)
        x[~avail] = -np.inf
        e = np.exp(x - x.max(axis=0))
        return (e.T @ K) / e.sum(axis=0)[:, None], lse


class _ThresholdSignFlipped(SPKVOracle):         # theta with the wrong sign
    def __init__(self, *a, **kw):
        super().__init__(*a, **kw)
        self.theta = np.float32(-self.theta)
        self._theta_hist = [[(0, self.theta)] for _ in range(self.B)]


class _DensityOverAllTokens(SPKVOracle):         # Eq. 8's reported density with the wrong denominator
    def stats(self):
        st = super().stats()
        st["density_evicted"] = st["kept_tokens"] / max(1, st["total_tokens"] * self.Hkv)
        return st


MUTANTS = [_WindowOffByOne, _StrictGate, _NoScale, _KeptOffByOne, _GateIgnored,
           _WrongGroup, _TransposedPV, _ThresholdSignFlipped, _DensityOverAllTokens]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda m: m.__name__)
def test_planted_mistake_is_caught(mutant):
    caught = []
    for pin in PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin catches {mutant.__name__}"


# ------------------------------------------------------- utility predictor (Eq. 1)
def test_utility_logits_against_torch_modules_and_closed_forms():
    """The oracle's predictor against torch's own Linear / SiLU in fp64 (a library routine),
    and against cases whose value is known: zero first layer -> b2 + W2 silu(b1);
    a one-hot path through the network."""
    from oracle.spkv_oracle import utility_logits
    rng = np.random.default_rng(3)
    n, dm, dh, H = 5, 12, 7, 3
    x, w1, b1 = rng.standard_normal((n, dm)), rng.standard_normal((dh, dm)), rng.standard_normal(dh)
    w2, b2 = rng.standard_normal((H, dh)), rng.standard_normal(H)
    net = torch.nn.Sequential(torch.nn.Linear(dm, dh), torch.nn.SiLU(), torch.nn.Linear(dh, H)).double()
    with torch.no_grad():
        net[0].weight.copy_(torch.from_numpy(w1)); net[0].bias.copy_(torch.from_numpy(b1))
        net[2].weight.copy_(torch.from_numpy(w2)); net[2].bias.copy_(torch.from_numpy(b2))
        ref = net(torch.from_numpy(x)).numpy()
    np.testing.assert_allclose(utility_logits(x, w1, b1, w2, b2), ref, rtol=1e-12, atol=1e-12)
    silu = lambda a: a / (1.0 + np.exp(-a))
    got = utility_logits(x, np.zeros_like(w1), b1, w2, b2)
    np.testing.assert_allclose(got, np.tile(b2 + w2 @ silu(b1), (n, 1)), rtol=1e-12)
    # one-hot: x = e_0 scaled by 2, w1 = e_1 e_0^T, w2 = 3 e_2 e_1^T -> logit[2] = 3 silu(2)
    x1 = np.zeros((1, dm)); x1[0, 0] = 2.0
    w1h = np.zeros((dh, dm)); w1h[1, 0] = 1.0
    w2h = np.zeros((H, dh)); w2h[2, 1] = 3.0
    got = utility_logits(x1, w1h, None, w2h, None)
    assert abs(got[0, 2] - 3.0 * 2.0 / (1.0 + math.exp(-2.0))) < 1e-14 and got[0, 0] == 0 and got[0, 1] == 0


# ------------------------------------------------ multi-token step (chunk of queries)
def _sdpa_rows(q_rows, k, v, gate, w, scale, Hq, Hkv, first_row):
    """Rows first_row.. of the full masked attention of one sequence by torch's fp64 SDPA
    under the availability mask of Eq. 3-4 (window or gate, never the future)."""
    T, D = k.shape[0], k.shape[2]
    G = Hq // Hkv
    kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    qt = torch.zeros(1, Hq, T, D, dtype=torch.float64)
    qt[0, :, first_row:, :] = torch.from_numpy(q_rows).permute(1, 0, 2)
    per_head = np.stack([_availability(T, w, gate[:, j // G]) for j in range(Hq)])
    mask = torch.from_numpy(per_head)[None]
    o = F.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=scale)
    return o[0, :, first_row:, :].permute(1, 0, 2).numpy()


def test_decode_chunk_matches_sdpa_rows_and_single_steps():
    rng = np.random.default_rng(29)
    B, Hq, Hkv, D, w, tau = 2, 4, 2, 8, 5, 0.5
    lens, counts = [23, 9], [7, 9]                 # second sequence: the chunk is the whole sequence
    q_all, k, v, f, cu = _random_problem(rng, B, Hq, Hkv, D, lens, mu=-0.3)
    o = _build(SPKVOracle, B, Hq, Hkv, D, w, tau, k, v, f, cu)
    q = rng.standard_normal((sum(counts), Hq, D))
    out, lse = o.decode_chunk(q, counts)
    row = 0
    for b in range(B):
        sl = slice(cu[b], cu[b + 1])
        sig = 1.0 / (1.0 + np.exp(-f[sl].astype(np.float64)))
        ref = _sdpa_rows(q[row:row + counts[b]], k[sl], v[sl], sig >= tau, w, 1.0 / math.sqrt(D),
                         Hq, Hkv, lens[b] - counts[b])
        np.testing.assert_allclose(out[row:row + counts[b]], ref, rtol=1e-10, atol=1e-12)
        row += counts[b]
    # the same outputs from one-token-at-a-time appends and decodes
    inc = SPKVOracle(B, Hq, Hkv, D, window=w, tau=tau, store_dtype=np.float64)
    pre = [lens[b] - counts[b] for b in range(B)]
    rows = [r for b in range(B) for r in range(cu[b], cu[b] + pre[b])]
    inc.append(k[rows], v[rows], f[rows], [0, pre[0], pre[0] + pre[1]])
    qoff = [0, counts[0]]
    for i in range(max(counts)):
        act = [b for b in range(B) if i < counts[b]]
        rows = [cu[b] + pre[b] + i for b in act]
        c = [0] + list(np.cumsum([1 if b in act else 0 for b in range(B)]))
        inc.append(k[rows], v[rows], f[rows], c)
        qq = np.zeros((B, Hq, D))
        for b in act:
            qq[b] = q[qoff[b] + i]
        if all(inc.seq_len(b) > 0 for b in range(B)):
            o1, l1 = inc.decode(qq)
            for b in act:
                np.testing.assert_allclose(o1[b], out[qoff[b] + i], rtol=1e-12, atol=1e-13)
                np.testing.assert_allclose(l1[b], lse[qoff[b] + i], rtol=1e-12, atol=1e-13)


def _cache_process(cls, n_sink=0, release=None, n_steps=34, seed=91):
    """Pin for set_tau, prune, release_sequence and the sinks: the appendix describes the cache
    as a process -- when the window is full, the pair leaving it is kept iff its gate is on
    (here: with the threshold in force at that moment, or when it is one of the first n_sink
    positions of its sequence), otherwise dropped; a prune drops from the kept list what fails
    the threshold of the moment (never a sink); a release empties the slot.  A literal
    simulation of that process (a window list, a kept list, one token at a time, plain Python)
    must give the oracle's kept lists, its counts, both densities of Eq. 8 and, with explicit
    softmax loops over kept + window, its decode output.  release: {step: sequence}."""
    rng = np.random.default_rng(seed)
    release = release or {}
    B, Hq, Hkv, D, w = 2, 4, 2, 4, 3
    taus = {0: 0.5, 7: 0.8, 12: 0.2, 13: 0.65, 20: 0.5, 27: 0.75}    # step -> new tau
    prunes = {8, 14, 15, 21, 28}                                      # steps that begin with a prune
    o = cls(B, Hq, Hkv, D, window=w, tau=taus[0], n_sink=n_sink)
    window = [[[] for _ in range(Hkv)] for _ in range(B)]    # (pos, k, v, f)
    kept = [[[] for _ in range(Hkv)] for _ in range(B)]
    n_tok = [0] * B
    gate_on = [0] * B
    theta = threshold_logit(taus[0])
    scale = 1.0 / math.sqrt(D)
    for step in range(n_steps):
        if step in release:                                   # the request in this slot ends
            b = release[step]
            o.release_sequence(b)
            window[b] = [[] for _ in range(Hkv)]
            kept[b] = [[] for _ in range(Hkv)]
            n_tok[b] = 0
            gate_on[b] = 0
        if step in taus and step > 0:
            o.set_tau(taus[step])
            theta = threshold_logit(taus[step])
        if step in prunes:                                    # what is kept is judged again
            o.prune()
            for b in range(B):
                for h in range(Hkv):
                    kept[b][h] = [e for e in kept[b][h] if e[3] >= theta or e[0] < n_sink]
        counts = [1, 1] if step % 5 else [2, 0]               # sequence 1 lags behind
        total = sum(counts)
        k = rng.standard_normal((total, Hkv, D)).astype(np.float32)
        v = rng.standard_normal((total, Hkv, D)).astype(np.float32)
        f = rng.standard_normal((total, Hkv)).astype(np.float32)
        cu = [0, counts[0], total]
        o.append(k, v, f, cu)
        for b in range(B):
            for r in range(cu[b], cu[b + 1]):
                for h in range(Hkv):
                    if len(window[b][h]) == w:                # window full: one pair leaves
                        old = window[b][h].pop(0)
                        if old[3] >= theta or old[0] < n_sink:
                            kept[b][h].append(old)
                    window[b][h].append((n_tok[b], k[r, h], v[r, h], f[r, h]))
                    gate_on[b] += int(f[r, h] >= theta or n_tok[b] < n_sink)
                n_tok[b] += 1
        for b in range(B):
            assert o.seq_len(b) == n_tok[b]
            for h in range(Hkv):
                assert o.kept_positions(b, h).tolist() == [e[0] for e in kept[b][h]], (step, b, h)
        st = o.stats()
        n_kept = sum(len(kept[b][h]) for b in range(B) for h in range(Hkv))
        n_left = sum(max(0, n - w) for n in n_tok) * Hkv
        assert st["gate_on_tokens"] == sum(gate_on)
        assert st["kept_tokens"] == n_kept and st["evicted_tokens"] == n_left
        assert st["total_tokens"] == sum(n_tok)
        # Eq. 8 as the text reports it (kept over what has left the window) and literally
        assert st["density_evicted"] == (float(Fraction(n_kept, n_left)) if n_left else 0.0)
        assert st["density_all"] == float(Fraction(sum(gate_on), sum(n_tok) * Hkv))
        if all(n_tok):
            q = rng.standard_normal((B, Hq, D)).astype(np.float32)
            out, lse = o.decode(q)
            for b in range(B):
                for h in range(Hkv):
                    entries = kept[b][h] + window[b][h]
                    for g in range(Hq // Hkv):
                        j = h * (Hq // Hkv) + g
                        sc = [scale * math.fsum(float(q[b, j, d]) * float(e[1][d]) for d in range(D))
                              for e in entries]
                        mx = max(sc)
                        wt = [math.exp(x - mx) for x in sc]
                        z = math.fsum(wt)
                        for d in range(D):
                            ref = math.fsum(a * float(e[2][d]) for a, e in zip(wt, entries)) / z
                            assert abs(out[b, j, d] - ref) < 1e-12
                        assert abs(lse[b, j] - (mx + math.log(z))) < 1e-12


def pin_cache_process(cls):
    _cache_process(cls)


def pin_cache_process_with_release(cls):
    # sequence 0 ends after thresholds 0.8 / 0.2 / 0.65 and three prunes have gone by; its
    # successor in the slot lives through a lower threshold, a prune, a higher one, a prune
    _cache_process(cls, release={16: 0, 24: 1})


def pin_cache_process_with_sinks(cls):
    # the sinks' logits are ordinary draws: several fail the thresholds of the prunes
    _cache_process(cls, n_sink=2)
    _cache_process(cls, n_sink=2, release={16: 0}, seed=92)


PROCESS_PINS = [pin_cache_process, pin_cache_process_with_release, pin_cache_process_with_sinks]


@pytest.mark.parametrize("pin", PROCESS_PINS, ids=lambda p: p.__name__)
def test_process_pin(pin):
    pin(SPKVOracle)


# Mistakes in the parts only the process pins reach.
class _ReleaseKeepsThresholdHistory(SPKVOracle):   # a released slot remembers old thresholds
    def release_sequence(self, b):
        hist = self._theta_hist[b]
        super().release_sequence(b)
        self._theta_hist[b] = hist


class _ReleaseKeepsPrunes(SPKVOracle):             # ... or old prunes
    def release_sequence(self, b):
        pr = self._prunes[b]
        super().release_sequence(b)
        self._prunes[b] = pr


class _PruneDropsSinks(SPKVOracle):                # a prune judges the sinks by their logits
    def gate(self, b, h):
        s = np.arange(self.seq_len(b))
        theta = self._theta_when_stored(b, s + self.w)
        theta[s + self.w >= self.seq_len(b)] = self.theta
        z = (self._f(b)[:, h] >= theta) | (s < self.n_sink)
        for n_evicted, theta_p in self._prunes[b]:
            z[:n_evicted] &= self._f(b)[:n_evicted, h] >= theta_p
        return z


class _WrongDensityDenominator(SPKVOracle):        # kept / all tokens instead of kept / evicted
    def stats(self):
        st = super().stats()
        tot = st["total_tokens"] * self.Hkv
        st["density_evicted"] = st["kept_tokens"] / tot if tot else 0.0
        return st


class _PruneIgnored(SPKVOracle):                   # prune does nothing
    def prune(self):
        pass


class _SetTauRewritesHistory(SPKVOracle):          # a new tau re-judges pairs that already left
    def set_tau(self, tau):
        super().set_tau(tau)
        self._theta_hist = [[(0, self.theta)] for _ in range(self.B)]


PROCESS_MUTANTS = {
    _ReleaseKeepsThresholdHistory: "pin_cache_process_with_release",
    _ReleaseKeepsPrunes: "pin_cache_process_with_release",
    _PruneDropsSinks: "pin_cache_process_with_sinks",
    _WrongDensityDenominator: "pin_cache_process",
    _PruneIgnored: "pin_cache_process",
    _SetTauRewritesHistory: "pin_cache_process",
}


@pytest.mark.parametrize("mutant", list(PROCESS_MUTANTS), ids=lambda m: m.__name__)
def test_planted_process_mistake_is_caught_by_its_named_pin(mutant):
    by_name = {p.__name__: p for p in PROCESS_PINS}
    with pytest.raises(AssertionError):
        by_name[PROCESS_MUTANTS[mutant]](mutant)


def test_sinks_pinned_to_sdpa_with_the_sink_columns_unmasked():
    """Pin for n_sink: against torch's fp64 scaled_dot_product_attention with the boolean mask
    causal & (window | gate | first n_sink columns), last row -- the listing's masked
    attention with the ablation's always-visible first positions."""
    rng = np.random.default_rng(5)
    B, Hq, Hkv, D, w, T, ns = 1, 4, 2, 8, 5, 40, 3
    k = rng.standard_normal((T, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((T, Hkv, D)).astype(np.float32)
    f = rng.standard_normal((T, Hkv)).astype(np.float32) - 1.0
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    o = SPKVOracle(B, Hq, Hkv, D, window=w, tau=0.5, n_sink=ns)
    o.append(k, v, f, [0, T])
    out, _ = o.decode(q)
    s = torch.arange(T)
    for h in range(Hkv):
        mask = ((T - 1 - s) < w) | torch.from_numpy(f[:, h] >= 0.0) | (s < ns)
        kept = o.kept_positions(0, h).tolist()
        assert kept == [int(x) for x in s[(torch.from_numpy(f[:, h] >= 0.0) | (s < ns)) & (s <= T - 1 - w)]]
        for g in range(Hq // Hkv):
            j = h * (Hq // Hkv) + g
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(q[0, j]).double().view(1, 1, 1, D),
                torch.from_numpy(k[:, h]).double().view(1, 1, T, D),
                torch.from_numpy(v[:, h]).double().view(1, 1, T, D),
                attn_mask=mask.view(1, 1, 1, T))
            assert np.allclose(out[0, j], ref.view(D).numpy(), atol=1e-12)
    assert set(range(ns)) <= set(o.kept_positions(0, 0).tolist())


def test_soft_gated_attention_pins():
    """Pins for the soft-gated forward (Eq. 6): (i) torch's fp64 scaled_dot_product_attention
    with the listing's additive mask (0 inside the window, log u outside, -inf for the
    future); (ii) gates fully open (f = +40, log u = 0 to 4e-18) = dense causal attention;
    (iii) gates shut (f = -60: weight e^-60) = sliding-window attention within 1e-20;
    (iv) window >= T = dense causal attention whatever the gates; (v) the listing's
    log(u + 1e-8) agrees for moderate logits."""
    from oracle.spkv_oracle import soft_gated_attention
    rng = np.random.default_rng(17)
    Hq, Hkv, D, w = 4, 2, 8, 4
    cu = [0, 19, 19, 30]
    total = cu[-1]
    q = rng.standard_normal((total, Hq, D)).astype(np.float32)
    k = rng.standard_normal((total, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((total, Hkv, D)).astype(np.float32)
    f = (2.0 * rng.standard_normal((total, Hkv))).astype(np.float32)

    def sdpa(fl, window, eps=0.0):
        out = np.zeros((total, Hq, D))
        for b in range(len(cu) - 1):
            lo, hi = cu[b], cu[b + 1]
            T = hi - lo
            if T == 0:
                continue
            dist = np.subtract.outer(np.arange(T), np.arange(T))           # t - s
            for j in range(Hq):
                h = j // (Hq // Hkv)
                # Eq. 6 as an additive bias: nothing inside the window, log u_s behind it,
                # -inf on the future
                with np.errstate(over="ignore", divide="ignore"):      # f = -1e4: u = 0, log u = -inf
                    u = 1.0 / (1.0 + np.exp(-fl[lo:hi, h].astype(np.float64)))
                    bias = np.where(dist >= window, np.log(u + eps)[None, :], 0.0)
                bias[dist < 0] = -np.inf
                mask = torch.from_numpy(bias)
                o = torch.nn.functional.scaled_dot_product_attention(
                    torch.from_numpy(q[lo:hi, j]).double()[None, None],
                    torch.from_numpy(k[lo:hi, h]).double()[None, None],
                    torch.from_numpy(v[lo:hi, h]).double()[None, None], attn_mask=mask[None, None])
                out[lo:hi, j] = o[0, 0].numpy()
        return out

    out, lse = soft_gated_attention(q, k, v, f, cu, w)
    assert np.allclose(out, sdpa(f, w), atol=1e-12)                          # (i)
    assert np.allclose(out, sdpa(f, w, eps=1e-8), atol=1e-5)                 # (v)
    f_open = np.full_like(f, 40.0)
    dense = sdpa(f_open, 10 ** 6)
    assert np.allclose(soft_gated_attention(q, k, v, f_open, cu, w)[0], dense, atol=1e-12)   # (ii)
    f_shut = np.full_like(f, -60.0)
    swa = sdpa(np.full_like(f, -1e4), w)          # log u = -1e4: exactly no weight outside the window
    assert np.allclose(soft_gated_attention(q, k, v, f_shut, cu, w)[0], swa, atol=1e-20 + 1e-12)  # (iii)
    assert np.allclose(soft_gated_attention(q, k, v, f, cu, 64)[0], dense, atol=1e-12)       # (iv)
    # lse: log of the biased partition sum, checked on one row by hand
    t, j, lo = 9, 3, 0
    h = j // (Hq // Hkv)
    xs = [float(q[lo + t, j].astype(np.float64) @ k[lo + s, h].astype(np.float64)) / math.sqrt(D)
          + (0.0 if t - s < w else -math.log1p(math.exp(-float(f[lo + s, h])))) for s in range(t + 1)]
    assert abs(lse[lo + t, j] - math.log(math.fsum(math.exp(x) for x in xs))) < 1e-12
