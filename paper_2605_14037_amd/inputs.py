"""Seeded synthetic inputs for the SP-KV decode path.

This module only draws random numbers and describes workload shapes.  It holds
none of the method's arithmetic (no gate, no mask, no softmax): the GPU library
and the CPU oracle both consume exactly the tensors produced here.

Recipe (shapes from the paper's Llama-3-8B row of the scaling table: 32 query
heads, 8 KV heads, head_dim 128; batch 16 from the decode-latency figure;
window 128 and tau 0.5 from Sec. 2.1 / the threshold discussion; keep rates
from the densities reported per task and per head):

* q, k, v ~ N(0, 1), rounded to bf16.
* utility logits (pre-sigmoid) for (sequence b, KV head h) ~ N(mu[b, h], 1) in
  fp32, with mu = Phi^-1(keep rate): at tau = 0.5 the gate fires when the logit
  is >= 0, so the expected keep rate is Phi(mu).  keep = 1 / 0 use mu = +40 /
  -40 (deterministic all / none).  Gate positions are i.i.d. along the sequence
  (the paper gives no spatial statistics of the gates).
"""

from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

BASE_SEED = 20260514


@dataclass
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ctx_lens: list            # tokens prefilled per sequence
    keep: np.ndarray          # [batch, n_kv_heads] target keep rate
    window: int = 128
    tau: float = 0.5
    decode_steps: int = 1
    seed: int = BASE_SEED
    n_layers: int = 1
    note: str = ""
    mu: np.ndarray = field(init=False)

    def __post_init__(self):
        self.keep = np.asarray(self.keep, dtype=np.float64).reshape(self.batch, self.n_kv_heads)
        self.mu = mu_from_keep(self.keep)

    @property
    def max_context(self):
        return int(max(self.ctx_lens)) + self.decode_steps

    def expected_kept_tokens(self):
        """Expected sum over (b, h) of long-term entries after prefill."""
        ev = np.maximum(np.asarray(self.ctx_lens) - self.window, 0)[:, None]
        return float((ev * self.keep).sum())


def mu_from_keep(keep):
    """Mean of the unit-variance logit distribution giving P(logit >= 0) = keep."""
    keep = np.asarray(keep, dtype=np.float64)
    inner = np.clip(keep, 1e-12, 1 - 1e-12)
    mu = torch.special.ndtri(torch.from_numpy(inner)).numpy()
    mu = np.where(keep >= 1.0, 40.0, mu)
    mu = np.where(keep <= 0.0, -40.0, mu)
    return mu


def workload(name: str) -> Workload:
    """The five synthetic configurations, by name ("cfg1" .. "cfg5")."""
    idx = int(name[-1])
    seed = BASE_SEED + idx
    rng = np.random.default_rng(seed)
    if idx == 1:
        return Workload(name, 1, 8, 2, 64, [2048], [[0.30, 0.10]],
                        decode_steps=64, seed=seed,
                        note="tiny single-layer decode, 64 steps")
    if idx == 2:
        keep_h = rng.uniform(0.10, 0.33, size=8)
        return Workload(name, 16, 32, 8, 128, [32768] * 16, np.tile(keep_h, (16, 1)),
                        seed=seed, note="Llama-3-8B-shaped layer, batch 16, ctx 32k")
    if idx == 3:
        keep_h = rng.uniform(0.02, 0.15, size=8)
        return Workload(name, 4, 32, 8, 128, [131072] * 4, np.tile(keep_h, (4, 1)),
                        seed=seed, note="long context, batch 4, ctx 128k")
    if idx == 4:
        B, H = 64, 8
        ctx = rng.integers(1024, 65536 + 1, size=B).tolist()
        kind = rng.permutation(B * H) % 4          # 0: dense, 1: local-only, 2-3: sparse
        keep = rng.uniform(0.05, 0.30, size=B * H)
        keep = np.where(kind == 0, 1.0, np.where(kind == 1, 0.0, keep))
        return Workload(name, B, 32, 8, 128, ctx, keep.reshape(B, H), seed=seed,
                        note="heterogeneous batch 64, ctx 1k-64k, mixed heads")
    if idx == 5:
        return Workload(name, 32, 32, 8, 128, [16384] * 32, np.full((32, 8), 0.15),
                        seed=seed, n_layers=32,
                        note="32 layers of batch 32, ctx 16k, ~15% keep")
    raise ValueError(name)


def small_workload(name, batch, n_q_heads, n_kv_heads, head_dim, ctx_lens, keep,
                   window=128, tau=0.5, decode_steps=1, seed=0):
    keep = np.broadcast_to(np.asarray(keep, dtype=np.float64), (batch, n_kv_heads))
    return Workload(name, batch, n_q_heads, n_kv_heads, head_dim, list(ctx_lens),
                    keep.copy(), window=window, tau=tau, decode_steps=decode_steps,
                    seed=BASE_SEED + 1000 + seed)


class TokenStream:
    """Draws packed token batches for a workload from one seeded generator.

    next_tokens(counts) returns (k, v, logits, cu_seqlens) for counts[b] new
    tokens of each sequence b, rows packed by sequence in position order:
    k, v bf16 [total, H_kv, D]; logits fp32 [total, H_kv]; cu_seqlens python
    list [B+1].  next_query() returns q bf16 [B, H_q, D].
    """

    def __init__(self, wl: Workload, device="cpu", q_gain=1.0, layer=0):
        self.wl = wl
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(wl.seed * 1000 + layer)
        self.q_gain = float(q_gain)
        self.mu = torch.tensor(wl.mu, dtype=torch.float32, device=self.device)

    def _randn(self, *shape):
        return torch.randn(*shape, generator=self.gen, device=self.device, dtype=torch.float32)

    def next_tokens(self, counts):
        wl = self.wl
        counts = [int(c) for c in counts]
        total = sum(counts)
        cu = [0]
        for c in counts:
            cu.append(cu[-1] + c)
        k = self._randn(total, wl.n_kv_heads, wl.head_dim).to(torch.bfloat16)
        v = self._randn(total, wl.n_kv_heads, wl.head_dim).to(torch.bfloat16)
        seq_of_row = torch.repeat_interleave(
            torch.arange(wl.batch, device=self.device),
            torch.tensor(counts, device=self.device))
        logits = self._randn(total, wl.n_kv_heads) + self.mu[seq_of_row]
        return k, v, logits.contiguous(), cu

    def next_query(self, rows=None):
        """q bf16 [rows, H_q, D]; rows defaults to one per sequence."""
        wl = self.wl
        rows = wl.batch if rows is None else int(rows)
        q = self._randn(rows, wl.n_q_heads, wl.head_dim) * self.q_gain
        return q.to(torch.bfloat16)


def prefill_chunks(ctx_lens, chunk):
    """Per-call token counts that feed every sequence its context in pieces of
    at most `chunk` tokens (shorter sequences simply finish earlier)."""
    done = [0] * len(ctx_lens)
    while any(d < c for d, c in zip(done, ctx_lens)):
        counts = [min(chunk, c - d) for d, c in zip(done, ctx_lens)]
        yield counts
        done = [d + n for d, n in zip(done, counts)]


def to_numpy_f32(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a bf16/fp32 tensor to a host fp32 array."""
    return t.detach().to(torch.float32).cpu().numpy()
