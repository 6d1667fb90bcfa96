"""Speculative draft-and-verify decoding, step by step, on top of the oracle forward.  TEST INFRASTRUCTURE ONLY.

Follows Sec. II-A (Eq. 1 draft proposal, Eq. 2 acceptance probability, Eq. 3 corrected resample), Alg. 1
Stage B (the decode loop) and Sec. III-C (draft = target with the pruned layers removed, KV reuse), in that
order and notation: q = draft distribution, p = target distribution, k -> K speculation depth.

Readings taken where the paper is silent or inconsistent (each is listed in the design notes):
  * The draft proposes its K tokens one after another, each conditioned on the previous ones (Eq. 1 and the
    conditioning written under Eq. 1), not simultaneously.
  * Eq. 3's residual is taken per candidate token, r(y) = max(0, p(y) - q(y)) / sum(...): the only form that
    is a distribution and keeps the output law equal to p (the "lossless" statement after Eq. 3).
  * Every step commits the accepted prefix plus one token drawn from the target: the resample of Eq. 3 at
    the first rejection, or a draw from p_K when all K are accepted.
  * Greedy decoding (Table 1 caption) is the one-hot limit: accept iff the draft token equals the target's
    arg-max; the extra token is the target's arg-max.  Arg-max compares float32 logits, lowest index wins.
  * Acceptance test without a division: accept iff u * q(d) < p(d), u uniform on [0, 1).
  * Sampling from weights w: smallest j with cumsum(w)[j] > u * sum(w).
  * Uniforms per step, in order: K for the draft's draws, K for the acceptance tests (all K slots are
    consumed even after a rejection), 1 for the resample / bonus token.  The prefill consumes 1.
  * One KV cache: the draft's active layers read the target-written prefix and write their own entries at
    the speculative positions; verification overwrites those positions in every layer; rollback only
    shortens the valid length.

Parity pins (tests/test_oracle_sd.py): greedy SD == plain greedy decode for any mask and K; empty mask
accepts everything; chi-squared law of sampled tokens == soft-max of the target logits; acceptance
frequency == sum_y min(p, q); K = 0 step == plain decode step; rollback == fresh prefill.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np


def argmax_f32(z: np.ndarray) -> int:
    """Arg-max of logits compared in float32; the lowest index wins ties."""
    return int(np.argmax(np.asarray(z, np.float64).astype(np.float32)))


def softmax64(z: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    z = np.asarray(z, np.float64) / float(temperature)
    e = np.exp(z - z.max())
    return e / e.sum()


def inv_cdf(w: np.ndarray, u: float) -> int:
    """Smallest j with (w_0 + ... + w_j) > u * sum(w); sums in index order, float64."""
    c = np.cumsum(np.asarray(w, np.float64))
    j = int(np.searchsorted(c, float(u) * c[-1], side="right"))
    return min(j, len(c) - 1)


def accept_greedy(d: np.ndarray, zp: np.ndarray):
    """d: K draft tokens; zp: [K+1, V] target logits.  Returns (n accepted, extra token x)."""
    K = len(d)
    n = K
    for i in range(K):
        if int(d[i]) != argmax_f32(zp[i]):
            n = i
            break
    return n, argmax_f32(zp[n])


def accept_sample(d: np.ndarray, zq: np.ndarray, zp: np.ndarray, u_acc: np.ndarray, u_res: float,
                  temperature: float = 1.0):
    """Eq. 2 acceptance then Eq. 3 resample.  zq: [K, V] draft logits, zp: [K+1, V] target logits."""
    K = len(d)
    n = K
    for i in range(K):
        p = softmax64(zp[i], temperature)
        q = softmax64(zq[i], temperature)
        t = int(d[i])
        if not (float(u_acc[i]) * q[t] < p[t]):      # accept with probability min(1, p/q)
            n = i
            break
    p = softmax64(zp[n], temperature)
    if n < K:
        q = softmax64(zq[n], temperature)
        r = np.maximum(0.0, p - q)
        x = inv_cdf(r if r.sum() > 0.0 else p, u_res)
    else:
        x = inv_cdf(p, u_res)
    return n, x


@dataclasses.dataclass
class StepRecord:
    P: int                    # cache length when the step started
    t_in: int                 # pending token fed first to draft and verify
    d: np.ndarray             # K draft tokens
    n: int                    # accepted draft tokens
    x: int                    # extra target-derived token
    zq: Optional[np.ndarray]  # [K, V] draft logits (float64) if kept
    zp: Optional[np.ndarray]  # [K+1, V] target logits (float64) if kept


class SpecDecoder:
    """State machine prefill -> (draft -> verify -> accept -> rollback)*, mirroring the paper's loop."""

    def __init__(self, model, skip_mask, K: int, mode: str = "greedy", temperature: float = 1.0,
                 keep_logits: bool = False):
        assert mode in ("greedy", "sample")
        self.m = model
        self.skip = np.ascontiguousarray(skip_mask, np.uint8)
        self.K = int(K)
        self.mode = mode
        self.T = float(temperature)
        self.keep_logits = keep_logits
        self.P = 0
        self.t_last = -1
        self.out: List[int] = []
        self.records: List[StepRecord] = []
        self.stats = dict(steps=0, drafted=0, accepted=0, examined=0)

    def _pick(self, z, u):
        return argmax_f32(z) if self.mode == "greedy" else inv_cdf(softmax64(z, self.T), u)

    def prefill(self, prompt, u: Optional[float] = None):
        """Target forward over the prompt; the first generated token comes from its last row."""
        prompt = np.asarray(prompt, np.int32)
        z = self.m.forward(prompt, 0, None, logits_from=len(prompt) - 1)[0]
        self.P = len(prompt)
        self.t_last = self._pick(z, u)
        self.out = [self.t_last]
        self.z_prefill = z
        return self.t_last

    def draft(self, u_draft=None):
        """Eq. 1: K tokens from the layer-skipped model, one at a time, sharing the cache."""
        K = self.K
        self.d = np.zeros(K, np.int32)
        self.zq = np.zeros((K, self.m.shape.vocab), np.float64)
        tok = self.t_last
        for i in range(K):
            self.zq[i] = self.m.forward([tok], self.P + i, self.skip)[0]
            tok = self._pick(self.zq[i], None if u_draft is None else u_draft[i])
            self.d[i] = tok
        return self.d

    def verify(self):
        """One causal (K+1)-row forward of the full model over [t_last, d_1..d_K] at positions P..P+K."""
        rows = np.concatenate([[self.t_last], self.d]).astype(np.int32)
        self.zp = self.m.forward(rows, self.P, None)
        return self.zp

    def accept(self, u_acc=None, u_res=None):
        if self.mode == "greedy":
            self.n, self.x = accept_greedy(self.d, self.zp)
        else:
            self.n, self.x = accept_sample(self.d, self.zq, self.zp, u_acc, u_res, self.T)
        return self.n, self.x

    def rollback(self):
        """Keep cache entries of t_last and the n accepted drafts; everything after is dead."""
        self.P = self.P + self.n + 1
        self.t_last = self.x

    def step(self, u=None):
        """One full step. In sample mode `u` holds 2K+1 uniforms: K draft, K accept, 1 resample."""
        K = self.K
        P0, t0 = self.P, self.t_last
        if self.mode == "sample":
            u = np.asarray(u, np.float32)
            assert len(u) == 2 * K + 1
            ud, ua, ur = u[:K], u[K:2 * K], float(u[2 * K])
        else:
            ud = ua = ur = None
        self.draft(ud)
        self.verify()
        n, x = self.accept(ua, ur)
        committed = [int(t) for t in self.d[:n]] + [int(x)]
        self.rollback()
        self.out.extend(committed)
        st = self.stats
        st["steps"] += 1; st["drafted"] += K; st["accepted"] += n; st["examined"] += n + (1 if n < K else 0)
        self.records.append(StepRecord(P0, t0, self.d.copy(), n, x,
                                       self.zq.copy() if self.keep_logits else None,
                                       self.zp.copy() if self.keep_logits else None))
        return committed

    def generate(self, prompt, G: int, uniforms=None):
        """Exactly G tokens after the prompt (the first is the prefill's); the last step is truncated."""
        cur = 0
        u0 = None
        if self.mode == "sample":
            u0 = float(uniforms[0]); cur = 1
        self.prefill(prompt, u0)
        per = 2 * self.K + 1
        while len(self.out) < G:
            if self.P + self.K + 1 > self.m.max_seq:
                raise ValueError("KV capacity exceeded")
            u = None
            if self.mode == "sample":
                u = uniforms[cur:cur + per]; cur += per
            self.step(u)
        return np.asarray(self.out[:G], np.int32)


def plain_decode(model, prompt, G: int, mode: str = "greedy", uniforms=None, temperature: float = 1.0,
                 keep_logits: bool = False):
    """Vanilla autoregressive decoding with the full model: one token per forward."""
    prompt = np.asarray(prompt, np.int32)
    out, rows = [], []
    z = model.forward(prompt, 0, None, logits_from=len(prompt) - 1)[0]
    P = len(prompt)
    for g in range(G):
        if keep_logits:
            rows.append(z.copy())
        tok = argmax_f32(z) if mode == "greedy" else inv_cdf(softmax64(z, temperature), float(uniforms[g]))
        out.append(tok)
        if g + 1 < G:
            z = model.forward([tok], P, None)[0]
            P += 1
    out = np.asarray(out, np.int32)
    return (out, np.asarray(rows)) if keep_logits else out


def expected_tokens_per_step(alpha: float, K: int) -> float:
    """Mean committed tokens per step when each draft token is accepted independently with probability alpha."""
    if alpha >= 1.0:
        return float(K + 1)
    return (1.0 - alpha ** (K + 1)) / (1.0 - alpha)


def projected_speedup(alpha: float, K: int, c: float, verify_ratio: float = 1.0) -> float:
    """Tokens/s of SD over plain decode: c = t_draft_forward / t_plain_forward,
    verify_ratio = t_verify / t_plain_forward."""
    return expected_tokens_per_step(alpha, K) / (K * c + verify_ratio)
