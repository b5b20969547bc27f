"""fp64 CPU oracle for Self-Pruned KV (SP-KV) decode attention.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
what the SP-KV decode path computes.  It is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg, and by nothing else; the GPU
library shares no code, table or constant with it.

What it follows (paper sections / equations, counted in order of appearance):

* Eq. 1-2 (Sec. 2.1, "Key-wise utility prediction"): every KV pair carries one
  utility per KV head, u = sigmoid(f); the inference gate is z = 1[u >= tau].
  The sigmoid is strictly increasing, so the gate is taken on the pre-sigmoid
  logit: z = 1[f >= theta] with theta = log(tau / (1 - tau)).  theta is
  evaluated once in fp64 and rounded to fp32, and the comparison is an fp32
  comparison on the caller's fp32 logits (tau <= 0 -> theta = -inf, keep all;
  tau >= 1 -> theta = +inf, keep none).  NaN logits compare false (dropped).
* Window indicator (Sec. 2.1, "Sliding-window & gated global attention"):
  key s is in the window of query t iff 0 <= t - s < w, i.e. the window holds
  the w most recent keys including the query's own.
* Eq. 3-4: key s is available to query t iff s <= t and (z_s = 1 or s is in
  the window).
* Eq. 5: o_t = sum_s softmax_s(<q_t, k_s> / sqrt(d) + B_ts) v_s over the
  available keys; computed as a plain two-pass softmax in fp64.
* Reference-implementation appendix: under grouped-query attention there is one
  gate per KV head and query head j reads KV head j // (H_q / H_kv).
* Appendix "Inference Kernels": a pair leaves the window when the token w
  positions later is written; it is then either kept in the long-term cache or
  discarded.  After T tokens the long-term cache of (sequence, KV head) holds
  { s <= T-1-w : z_s = 1 }, listed here in ascending position.
* Eq. 8 ("Measuring sparsity"): gate density; both the literal form (all
  positions) and the form the text reports (long-term entries only) are given.

The oracle never prunes anything: it keeps the whole K/V/logit history and
applies the availability mask explicitly at decode time.

Pins (tests/test_oracle_pins.py): hand-derived rational-weight examples
(tests/golden/), pure-Python brute force on tiny inputs, the library routine
torch.nn.functional.scaled_dot_product_attention in fp64 under the explicit
mask, tau = -inf == dense causal attention, tau = +inf == sliding-window
attention, closed forms (identical keys -> mean of V, constant V, one dominant
key), the count invariant (both densities of Eq. 8 included), a literal
step-by-step simulation of the cache process of the appendix (window list, kept
list; threshold changes, prunes, sequence release and refill, sinks) that pins
set_tau, prune, release_sequence and n_sink, and mutation checks showing that
each planted mistake is caught by at least one pin.
"""

from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np


def threshold_logit(tau: float) -> np.float32:
    """theta = logit(tau) as fp32 (Eq. 2 moved through the sigmoid).

    `tau` is first rounded to fp32 (the width the C ABI carries it in), then
    the logit is evaluated in fp64 and rounded once to fp32.
    """
    t = float(np.float32(tau))
    if math.isnan(t):
        raise ValueError("tau is NaN")
    if t <= 0.0:
        return np.float32(-np.inf)
    if t >= 1.0:
        return np.float32(np.inf)
    return np.float32(math.log(t / (1.0 - t)))


def utility_logits(hidden, w1, b1, w2, b2):
    """Pre-sigmoid output of the utility predictor (Eq. 1; listing appendix: Linear, SiLU,
    Linear), in fp64: f[t, h] = b2[h] + sum_j w2[h, j] silu(b1[j] + sum_k w1[j, k] x[t, k]),
    silu(a) = a sigmoid(a).  Weights are [out, in]; biases may be None."""
    x = np.asarray(hidden, np.float64)
    a = x @ np.asarray(w1, np.float64).T
    if b1 is not None:
        a = a + np.asarray(b1, np.float64)
    a = a / (1.0 + np.exp(-a))
    f = a @ np.asarray(w2, np.float64).T
    if b2 is not None:
        f = f + np.asarray(b2, np.float64)
    return f


def soft_gated_attention(q, k, v, util_logits, cu_seqlens, window, sm_scale=None):
    """Soft-gated attention forward (training phase 1; Eq. 6 and the soft branch of the
    listing appendix), fp64, over whole packed sequences.

    For the query at position t of a sequence and every key s <= t: pre-softmax score
    scale * q_t . k_s, plus the bias log u_s = log sigmoid(f_s) when the key is outside the
    window (t - s >= window); keys inside the window (0 <= t - s < window) get no bias.
    q: [total, H_q, D]; k, v: [total, H_kv, D]; util_logits: fp32 [total, H_kv]; query head j
    reads KV head j // (H_q / H_kv).  log u is taken exactly from the logit
    (log sigmoid(f) = -log(1 + exp(-f))), not as log(u + 1e-8): that epsilon only keeps a
    gradient finite.  Returns (out [total, H_q, D], lse [total, H_q])."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    f = np.asarray(util_logits)
    if f.dtype != np.float32:
        raise TypeError("utility logits must be float32")
    f = f.astype(np.float64)
    total, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    scale = (1.0 / math.sqrt(D)) if sm_scale is None else float(sm_scale)
    log_u = -np.logaddexp(0.0, -f)                       # log sigmoid(f), stable
    out = np.zeros((total, Hq, D))
    lse = np.zeros((total, Hq))
    for b in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        T = hi - lo
        if T == 0:
            continue
        t = np.arange(T)[:, None]
        s = np.arange(T)[None, :]
        causal = s <= t
        outside = causal & ((t - s) >= window)
        for h in range(Hkv):
            bias = np.where(outside, log_u[lo:hi, h][None, :], 0.0)
            bias = np.where(causal, bias, -np.inf)
            for g in range(G):
                j = h * G + g
                x = scale * (q[lo:hi, j, :] @ k[lo:hi, h, :].T) + bias
                mx = x.max(axis=1, keepdims=True)
                e = np.exp(x - mx)
                den = e.sum(axis=1, keepdims=True)
                out[lo:hi, j, :] = (e @ v[lo:hi, h, :]) / den
                lse[lo:hi, j] = (mx + np.log(den))[:, 0]
    return out, lse


class SPKVOracle:
    """Dense-history SP-KV decode attention, one instance per attention layer.

    Parameters mirror the quantities named in Sec. 2.1: `window` is w, `tau`
    the gate threshold on the sigmoid, `sm_scale` the softmax scale
    (1/sqrt(head_dim) when None, Eq. 5).
    """

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, window=128,
                 tau=0.5, sm_scale=None, store_dtype=np.float32, track_kv=True, n_sink=0):
        if n_q_heads % n_kv_heads != 0:
            raise ValueError("n_q_heads must be a multiple of n_kv_heads")
        if window < 1:
            raise ValueError("window must be >= 1")
        self.B, self.Hq, self.Hkv, self.D = batch, n_q_heads, n_kv_heads, head_dim
        self.G = n_q_heads // n_kv_heads
        self.w = int(window)
        # Optional attention sinks (the "fixed attention sinks" ablation): the first n_sink
        # positions of a sequence count as gated on whatever their logit.  0 = the method.
        self.n_sink = int(n_sink)
        self.theta = threshold_logit(tau)
        self.scale = (1.0 / math.sqrt(head_dim)) if sm_scale is None else float(sm_scale)
        self.store_dtype = store_dtype
        # track_kv=False keeps only the utility logits: gate bookkeeping (kept lists,
        # lengths, density) for every sequence of a large batch without the K/V history;
        # decode is then unavailable.
        self.track_kv = bool(track_kv)
        # Full, never-pruned history per sequence, in buffers that grow by
        # doubling; rows [0, _len[b]) are live.
        self._kbuf = [np.zeros((0, n_kv_heads, head_dim), store_dtype) for _ in range(batch)]
        self._vbuf = [np.zeros((0, n_kv_heads, head_dim), store_dtype) for _ in range(batch)]
        self._fbuf = [np.zeros((0, n_kv_heads), np.float32) for _ in range(batch)]
        self._len = [0] * batch
        # Threshold history per sequence: (tokens stored when it took effect, theta).  With a
        # threshold that never changes this is one entry and every gate below is the plain
        # Eq. 2 comparison.
        self._theta_hist = [[(0, self.theta)] for _ in range(batch)]
        self._prunes = [[] for _ in range(batch)]     # (positions evicted so far, theta) per prune

    # ------------------------------------------------------------------ write
    def append(self, k, v, util_logits, cu_seqlens):
        """Append tokens.  k, v: [total, H_kv, D]; util_logits: fp32
        [total, H_kv] (pre-sigmoid); cu_seqlens: [B+1] row offsets, sequence b
        owns rows cu[b]:cu[b+1] in order of position."""
        f = np.asarray(util_logits)
        if f.dtype != np.float32:
            raise TypeError("utility logits must be float32")
        if self.track_kv:
            k = np.asarray(k)
            v = np.asarray(v)
        cu = [int(x) for x in cu_seqlens]
        if len(cu) != self.B + 1 or cu[0] != 0 or cu[-1] != f.shape[0]:
            raise ValueError("bad cu_seqlens")
        for b in range(self.B):
            lo, hi = cu[b], cu[b + 1]
            if hi < lo:
                raise ValueError("cu_seqlens must be non-decreasing")
            if hi == lo:
                continue
            old, new = self._len[b], self._len[b] + (hi - lo)
            if new > self._fbuf[b].shape[0]:
                cap = max(new, 2 * self._fbuf[b].shape[0])
                grow = (self._kbuf, self._vbuf, self._fbuf) if self.track_kv else (self._fbuf,)
                for bufs in grow:
                    grown = np.zeros((cap,) + bufs[b].shape[1:], bufs[b].dtype)
                    grown[:old] = bufs[b][:old]
                    bufs[b] = grown
            if self.track_kv:
                self._kbuf[b][old:new] = k[lo:hi]
                self._vbuf[b][old:new] = v[lo:hi]
            self._fbuf[b][old:new] = f[lo:hi]
            self._len[b] = new

    def set_tau(self, tau):
        """Change the threshold of a live cache.  A pair's keep-or-drop decision is taken
        when it leaves the window (when position s + w is stored), with the threshold in
        force at that moment; decisions already taken stand.  ("tau can be adjusted a
        posteriori", Sec. 3: here also between steps of one sequence.)"""
        self.theta = threshold_logit(tau)
        for b in range(self.B):
            self._theta_hist[b].append((self._len[b], self.theta))

    def prune(self):
        """Re-threshold what is already kept: every pair that has left the window and whose
        logit fails the threshold now in force is dropped from the long-term cache (pairs
        dropped earlier stay dropped; sink positions stay kept).  With set_tau this is the
        "tau adjusted a posteriori" of Sec. 3 applied to a live cache in the raising
        direction."""
        for b in range(self.B):
            self._prunes[b].append((max(0, self._len[b] - self.w), self.theta))

    def _theta_when_stored(self, b, n_stored):
        """theta in force when the sequence held n_stored[i] tokens and took one more."""
        n_stored = np.asarray(n_stored)
        th = np.empty(n_stored.shape, np.float32)
        for start, theta in self._theta_hist[b]:        # ascending starts: later entries win
            th[n_stored >= start] = theta
        return th

    def release_sequence(self, b):
        """Forget sequence b: slot b holds an empty sequence again."""
        self._theta_hist[b] = [(0, self.theta)]
        self._prunes[b] = []
        self._kbuf[b] = np.zeros((0, self.Hkv, self.D), self.store_dtype)
        self._vbuf[b] = np.zeros((0, self.Hkv, self.D), self.store_dtype)
        self._fbuf[b] = np.zeros((0, self.Hkv), np.float32)
        self._len[b] = 0

    # ------------------------------------------------------------- bookkeeping
    def seq_len(self, b):
        return self._len[b]

    def _k(self, b):
        return self._kbuf[b][:self._len[b]]

    def _v(self, b):
        return self._vbuf[b][:self._len[b]]

    def _f(self, b):
        return self._fbuf[b][:self._len[b]]

    def gate(self, b, h):
        """z_s for every stored position of (b, h): fp32 compare f >= theta (Eq. 2 on the
        logit), theta being the threshold in force when s left the window, i.e. when
        position s + w was stored (for positions still inside the window: the current one;
        their gate is not consulted by Eq. 3-4)."""
        s = np.arange(self.seq_len(b))
        theta = self._theta_when_stored(b, s + self.w)
        theta[s + self.w >= self.seq_len(b)] = self.theta
        z = self._f(b)[:, h] >= theta
        for n_evicted, theta_p in self._prunes[b]:      # a prune re-judges what had left the window
            z[:n_evicted] &= self._f(b)[:n_evicted, h] >= theta_p
        return z | (s < self.n_sink)

    def gate_at_append(self, b, h):
        """The same comparison with the threshold in force when s itself was stored: the
        z_s that Eq. 8 sums over all positions."""
        s = np.arange(self.seq_len(b))
        return (self._f(b)[:, h] >= self._theta_when_stored(b, s)) | (s < self.n_sink)

    def kept_positions(self, b, h):
        """Ascending positions held by the long-term cache of (b, h): gated-on
        positions that have left the window of the newest token t = T-1,
        i.e. s <= t - w."""
        T = self.seq_len(b)
        n_evicted = max(0, T - self.w)
        z = self.gate(b, h)[:n_evicted]
        return np.nonzero(z)[0].astype(np.int32)

    def kept_len(self):
        return np.array([[len(self.kept_positions(b, h)) for h in range(self.Hkv)]
                         for b in range(self.B)], dtype=np.int32)

    def available(self, b, h):
        """Boolean availability of every stored position to the newest query
        t = T-1 (Eq. 3-4): s <= t and (t - s < w or z_s)."""
        T = self.seq_len(b)
        s = np.arange(T)
        t = T - 1
        in_window = (t - s) < self.w          # s <= t holds for every stored s
        return in_window | self.gate(b, h)

    def available_at(self, b, h, t):
        """Availability of positions 0..t to the query at position t (Eq. 3-4), for any
        stored position t: s <= t and (t - s < w or z_s)."""
        s = np.arange(t + 1)
        return ((t - s) < self.w) | self.gate(b, h)[:t + 1]

    def stats(self):
        """Eq. 8 in both readings, plus byte counts at 2 bytes per element."""
        tot_T = sum(self.seq_len(b) for b in range(self.B))
        evicted = sum(max(0, self.seq_len(b) - self.w) for b in range(self.B)) * self.Hkv
        window = sum(min(self.seq_len(b), self.w) for b in range(self.B)) * self.Hkv
        kept = int(self.kept_len().sum())
        gate_on = int(sum(int(self.gate_at_append(b, h).sum())
                          for b in range(self.B) for h in range(self.Hkv)))
        row_bytes = 2 * self.D * 2            # K row + V row, 2 bytes/element
        return dict(
            total_tokens=tot_T, evicted_tokens=evicted, window_tokens=window,
            kept_tokens=kept, gate_on_tokens=gate_on,
            density_evicted=(kept / evicted) if evicted else 0.0,
            density_all=(gate_on / (tot_T * self.Hkv)) if tot_T else 0.0,
            kept_kv_bytes=(kept + window) * row_bytes,
            dense_kv_bytes=tot_T * self.Hkv * row_bytes,
        )

    # ------------------------------------------------------------------- read
    def decode_pair(self, b, h, q_bh):
        """One (sequence, KV head): q_bh [G, D] (the group's query heads) ->
        (out [G, D], lse [G]) for the newest position, in fp64."""
        if not self.track_kv:
            raise RuntimeError("this oracle instance tracks logits only")
        q_bh = np.asarray(q_bh, dtype=np.float64)
        K = self._k(b)[:, h, :].astype(np.float64)       # [T, D]
        V = self._v(b)[:, h, :].astype(np.float64)
        avail = self.available(b, h)
        x = self.scale * (K @ q_bh.T)                    # [T, G], Eq. 5 scores
        x[~avail, :] = -np.inf                           # Eq. 3-4 bias
        m = x.max(axis=0)                                # pass 1
        e = np.exp(x - m)                                # masked -> exactly 0
        denom = e.sum(axis=0)                            # pass 2
        out = (e.T @ V) / denom[:, None]
        lse = m + np.log(denom)
        return out, lse

    def decode_chunk(self, q, counts, rows=None):
        """Outputs for the newest counts[b] positions of every sequence, each attending as if
        it had been decoded right after its own append (causal inside the chunk): the rows
        T - n .. T - 1 of the masked attention of the listing appendix.  q: [sum(counts),
        H_q, D] packed by sequence in position order.  Returns (out, lse) in fp64.  rows: if
        given, only these packed rows are computed (the others stay zero)."""
        q = np.asarray(q).astype(np.float64)
        total = int(sum(counts))
        if q.shape != (total, self.Hq, self.D):
            raise ValueError("q must be [sum(counts), H_q, D]")
        out = np.zeros((total, self.Hq, self.D), np.float64)
        lse = np.zeros((total, self.Hq), np.float64)
        row = 0
        for b in range(self.B):
            T, n = self.seq_len(b), int(counts[b])
            if n > T:
                raise ValueError("chunk longer than the sequence")
            for i in range(n):
                t = T - n + i
                if rows is not None and row not in rows:
                    row += 1
                    continue
                for h in range(self.Hkv):
                    K = self._k(b)[:t + 1, h, :].astype(np.float64)
                    V = self._v(b)[:t + 1, h, :].astype(np.float64)
                    avail = self.available_at(b, h, t)
                    g0 = h * self.G
                    x = self.scale * (K @ q[row, g0:g0 + self.G, :].T)
                    x[~avail, :] = -np.inf
                    m = x.max(axis=0)
                    e = np.exp(x - m)
                    den = e.sum(axis=0)
                    out[row, g0:g0 + self.G, :] = (e.T @ V) / den[:, None]
                    lse[row, g0:g0 + self.G] = m + np.log(den)
                row += 1
        return out, lse

    def decode(self, q, workers=1):
        """One decode step for every sequence: the query is the newest stored
        position (its own key is already appended and sits in the window).
        q: [B, H_q, D].  Returns (out [B, H_q, D], lse [B, H_q]) in fp64, where
        lse = log sum_s exp(score_s) over the available keys."""
        q = np.asarray(q).astype(np.float64)
        if q.shape != (self.B, self.Hq, self.D):
            raise ValueError("q must be [B, H_q, D]")
        for b in range(self.B):
            if self.seq_len(b) == 0:
                raise ValueError("decode on an empty sequence (softmax over nothing)")
        out = np.zeros((self.B, self.Hq, self.D), np.float64)
        lse = np.zeros((self.B, self.Hq), np.float64)

        def job(bh):
            b, h = bh
            g0 = h * self.G
            o, l = self.decode_pair(b, h, q[b, g0:g0 + self.G, :])
            out[b, g0:g0 + self.G, :] = o
            lse[b, g0:g0 + self.G] = l

        pairs = [(b, h) for b in range(self.B) for h in range(self.Hkv)]
        if workers <= 1:
            for bh in pairs:
                job(bh)
        else:
            with ThreadPoolExecutor(max_workers=workers) as ex:
                list(ex.map(job, pairs))
        return out, lse
