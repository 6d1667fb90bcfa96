"""Pins for the oracle's speculative loop (CPU only): what the paper and the mathematics fix.

 * lossless under greedy decoding (statement after Eq. 3; Table 1 caption): SD == plain greedy decode
 * Eq. 2 with p == q: everything accepted, K+1 tokens per step
 * Eq. 2 + Eq. 3: the emitted tokens follow the target distribution (chi-squared), acceptance
   probability sum_y min(p, q)
 * K = 0 step == plain decode step; rollback == fresh prefill; expected tokens per step closed form
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import synth
from oracle import (OracleModel, SpecDecoder, plain_decode, accept_greedy, accept_sample, softmax64, inv_cdf,
                    argmax_f32, expected_tokens_per_step, projected_speedup)


def _model(shape, **kw):
    w = synth.gen_host_weights(shape, **kw)
    return OracleModel(shape, w), w


# ---- lossless greedy (P1) ------------------------------------------------------------------------------
def test_tiny_config_greedy_sd_equals_plain_decode():
    s = synth.CONFIGS["tiny"]
    prompt = synth.gen_prompt(synth.SEED_PROMPT, s.n_prompt, s.vocab)
    m, w = _model(s)
    ref = plain_decode(m, prompt, s.n_gen)
    sd = SpecDecoder(OracleModel(s, w), synth.gen_skip_mask(s), s.K)
    out = sd.generate(prompt, s.n_gen)
    assert np.array_equal(out, ref)
    assert sd.stats["drafted"] == s.K * sd.stats["steps"]


@pytest.mark.parametrize("name", ["mha_f32", "gqa_bf16"])
def test_greedy_sd_equals_plain_for_any_mask_and_K(small_shapes, name):
    s = small_shapes[name]
    L = s.n_layers
    masks = [np.zeros(L, np.uint8), np.full(L, 3, np.uint8), synth.gen_skip_mask(s)]
    only0 = np.full(L, 3, np.uint8); only0[0] = 0
    sub = np.array([(1, 2, 0, 3)[i % 4] for i in range(L)], np.uint8)        # attention-only / FFN-only skips
    masks += [only0, sub]
    for std in (0.08, 0.3):                      # a flat and a peaky regime: different token dynamics
        sh = s.with_(init_std=std)
        w = synth.gen_host_weights(sh)
        prompt = synth.gen_prompt(11, sh.n_prompt, sh.vocab)
        G = sh.n_gen
        ref = plain_decode(OracleModel(sh, w, max_seq=64), prompt, G)
        for mi, mask in enumerate(masks):
            for K in ((1, 2, 3, 4, 5, 6, 7, 8) if mi == 2 else (1, 4)):
                sd = SpecDecoder(OracleModel(sh, w, max_seq=64), mask, K)
                assert np.array_equal(sd.generate(prompt, G), ref), (std, mi, K)
                assert 0 <= sd.stats["accepted"] <= sd.stats["drafted"]


def test_partial_acceptance_actually_occurs(small_shapes):
    """The lossless checks above must cover accepted, partly accepted and rejected blocks."""
    s = small_shapes["mha_f32"].with_(init_std=0.3)
    mask = synth.gen_skip_mask(s)
    w = synth.gen_host_weights(s, damp_skipped=0.2, skip_mask=mask)
    prompt = synth.gen_prompt(12, s.n_prompt, s.vocab)
    ref = plain_decode(OracleModel(s, w, max_seq=80), prompt, 40)
    sd = SpecDecoder(OracleModel(s, w, max_seq=80), mask, 4)
    assert np.array_equal(sd.generate(prompt, 40), ref)
    ns = {r.n for r in sd.records}
    assert len(ns) >= 3 and 0 in ns and 4 in ns, ns


# ---- p == q (P2) ---------------------------------------------------------------------------------------
def test_empty_mask_accepts_everything(small_shapes):
    s = small_shapes["gqa_bf16"]
    w = synth.gen_host_weights(s)
    prompt = synth.gen_prompt(13, s.n_prompt, s.vocab)
    for K in (1, 3, 4):
        G = 22
        sd = SpecDecoder(OracleModel(s, w, max_seq=64), np.zeros(s.n_layers, np.uint8), K)
        sd.generate(prompt, G)
        assert all(r.n == K for r in sd.records)
        assert sd.stats["steps"] == math.ceil((G - 1) / (K + 1))
    # sampling: with p == q every acceptance test passes whatever the uniforms are
    K = 3
    sd = SpecDecoder(OracleModel(s, w, max_seq=64), np.zeros(s.n_layers, np.uint8), K, mode="sample")
    u = synth.gen_uniforms(5, 1 + (2 * K + 1) * 10)
    sd.generate(prompt, 20, u)
    assert all(r.n == K for r in sd.records)


# ---- accept rule on explicit distributions (P3, P4) ----------------------------------------------------
def test_accept_greedy_cases():
    V = 6
    zp = np.full((4, V), -1.0)
    zp[0, 2] = 1; zp[1, 5] = 1; zp[2, 0] = 1; zp[3, 4] = 1
    assert accept_greedy(np.array([2, 5, 0]), zp) == (3, 4)          # all accepted -> bonus from row K
    assert accept_greedy(np.array([2, 1, 0]), zp) == (1, 5)          # first mismatch at i=1 -> correction
    assert accept_greedy(np.array([3, 5, 0]), zp) == (0, 2)
    assert accept_greedy(np.array([], np.int32), zp[:1]) == (0, 2)   # K = 0
    zt = np.zeros((1, V)); zt[0, 3] = zt[0, 1] = 2.0
    assert argmax_f32(zt[0]) == 1                                     # lowest index wins ties
    # differences below float32 resolution are ties
    zt[0, 3] = 2.0 + 1e-9
    assert argmax_f32(zt[0]) == 1


def test_inv_cdf_conventions():
    w = np.array([0.0, 0.25, 0.0, 0.5, 0.25])
    assert inv_cdf(w, 0.0) == 1           # zero-weight entries are never chosen
    assert inv_cdf(w, 0.2499) == 1
    assert inv_cdf(w, 0.25) == 3          # boundary belongs to the next token (strict >)
    assert inv_cdf(w, 0.7499) == 3
    assert inv_cdf(w, 0.75) == 4
    assert inv_cdf(w, 1.0 - 2.0 ** -24) == 4
    assert inv_cdf(w * 7.0, 0.5) == 3     # unnormalised weights
    u = synth.gen_uniforms(1, 200000)
    cnt = np.bincount([inv_cdf(w, x) for x in u[:40000]], minlength=5)
    assert stats.chisquare(cnt[[1, 3, 4]], 40000 * w[[1, 3, 4]]).pvalue > 1e-3 and cnt[0] == cnt[2] == 0


def test_one_draft_token_law_and_acceptance_rate():
    """K = 1 on explicit p, q: emitted token ~ p exactly; P(accept) = sum min(p, q); residual mass = 1 - that."""
    rng = np.random.default_rng(4)
    V, N = 12, 60000
    zp = rng.standard_normal((2, V)) * 1.5
    zq = rng.standard_normal((1, V)) * 1.5
    p, q = softmax64(zp[0]), softmax64(zq[0])
    u = synth.gen_uniforms(6, 3 * N).reshape(N, 3)
    first = np.zeros(V, np.int64)
    acc = 0
    for ud, ua, ur in u:
        d = inv_cdf(q, ud)
        n, x = accept_sample(np.array([d]), zq, zp, np.array([ua]), ur)
        first[d if n == 1 else x] += 1
        acc += n
    assert stats.chisquare(first, N * p).pvalue > 1e-3
    a = np.minimum(p, q).sum()
    assert abs(acc / N - a) < 4 * math.sqrt(a * (1 - a) / N)
    assert abs(np.maximum(0, p - q).sum() - (1 - a)) < 1e-12
    # the naive scalar reading of Eq. 3 (alpha of the rejected token) is not a distribution for these p, q
    d = int(np.argmax(q - p))
    assert (p - min(1.0, p[d] / q[d]) * q).min() < 0


def test_planted_mistakes_in_the_accept_rule_are_detected():
    """The chi-squared pin has power: plausible wrong rules (no residual clamp target, swapped p/q) fail it."""
    rng = np.random.default_rng(4)
    V, N = 12, 60000
    zp = rng.standard_normal((2, V)) * 1.5
    zq = rng.standard_normal((1, V)) * 1.5
    p, q = softmax64(zp[0]), softmax64(zq[0])
    u = synth.gen_uniforms(6, 3 * N).reshape(N, 3)
    resample_from_p = np.zeros(V, np.int64)
    swapped = np.zeros(V, np.int64)
    for ud, ua, ur in u:
        d = inv_cdf(q, ud)
        ok = ua * q[d] < p[d]
        resample_from_p[d if ok else inv_cdf(p, ur)] += 1
        ok2 = ua * p[d] < q[d]
        swapped[d if ok2 else inv_cdf(np.maximum(0, p - q), ur)] += 1
    assert stats.chisquare(resample_from_p, N * p).pvalue < 1e-6
    assert stats.chisquare(swapped, N * p).pvalue < 1e-6


# ---- whole loop in sampling mode on a tiny vocabulary (P3) ---------------------------------------------
def test_sampled_sd_tokens_follow_target_distribution(small_shapes):
    s = small_shapes["v16"]
    mask = synth.gen_skip_mask(s)
    w = synth.gen_host_weights(s, damp_skipped=0.6, skip_mask=mask)
    prompt = synth.gen_prompt(21, s.n_prompt, s.vocab)
    V, K = s.vocab, s.K
    base = OracleModel(s, w, max_seq=32)
    # exact law of the two tokens after the first generated one, from the target alone
    z0 = base.forward(prompt, 0, None, logits_from=len(prompt) - 1)[0]
    t0 = argmax_f32(z0)
    p1 = softmax64(base.forward([t0], len(prompt))[0])
    joint = np.zeros((V, V))
    for y1 in range(V):
        joint[y1] = p1[y1] * softmax64(base.forward([y1], len(prompt) + 1)[0])
    N = 12000
    per = 2 * K + 1
    u = synth.gen_uniforms(31, N * 2 * per).reshape(N, 2 * per)
    counts = np.zeros((V, V), np.int64)
    n_hist = np.zeros(K + 1, np.int64)
    m = OracleModel(s, w, max_seq=32)
    sd = SpecDecoder(m, mask, K, mode="sample")
    sd.prefill(prompt, 0.0)
    sd.t_last = t0                      # condition every trial on the same first token
    P0 = sd.P
    for i in range(N):
        sd.P, sd.t_last, sd.out = P0, t0, [t0]
        sd.step(u[i, :per])
        n_hist[sd.records[-1].n] += 1
        if len(sd.out) < 3:
            sd.step(u[i, per:])
        counts[sd.out[1], sd.out[2]] += 1
    assert n_hist[0] > 0 and n_hist[1:].sum() > 0          # both rejections and acceptances are exercised
    exp = (joint * N).ravel()
    obs = counts.ravel().astype(np.float64)
    order = np.argsort(exp)                                 # pool cells with small expectation
    small = order[np.cumsum(exp[order]) < 20]
    big = np.setdiff1d(np.arange(V * V), small)
    obs2 = np.append(obs[big], obs[small].sum()); exp2 = np.append(exp[big], exp[small].sum())
    keep = exp2 > 0
    assert stats.chisquare(obs2[keep], exp2[keep] * obs2[keep].sum() / exp2[keep].sum()).pvalue > 1e-3
    assert stats.chisquare(counts.sum(1), N * p1).pvalue > 1e-3
    # acceptance frequency of the first draft token = sum_y min(p, q)  (closed form)
    q1 = softmax64(base.forward([t0], len(prompt), mask)[0])
    a = np.minimum(p1, q1).sum()
    assert abs(n_hist[1:].sum() / N - a) < 4.5 * math.sqrt(a * (1 - a) / N)


# ---- degenerate and structural cases (P7, P8) ----------------------------------------------------------
def test_K0_step_is_a_plain_decode_step(small_shapes):
    s = small_shapes["mha_f32"].with_(init_std=0.3)
    w = synth.gen_host_weights(s)
    prompt = synth.gen_prompt(14, s.n_prompt, s.vocab)
    ref = plain_decode(OracleModel(s, w, max_seq=64), prompt, 15)
    sd = SpecDecoder(OracleModel(s, w, max_seq=64), synth.gen_skip_mask(s), 0)
    assert np.array_equal(sd.generate(prompt, 15), ref)
    assert sd.stats["steps"] == 14 and sd.stats["drafted"] == 0
    # sampling: same uniforms, one per token
    u = synth.gen_uniforms(9, 15)
    ref = plain_decode(OracleModel(s, w, max_seq=64), prompt, 15, mode="sample", uniforms=u)
    sd = SpecDecoder(OracleModel(s, w, max_seq=64), synth.gen_skip_mask(s), 0, mode="sample")
    assert np.array_equal(sd.generate(prompt, 15, u), ref)


def test_rollback_state_equals_fresh_prefill(small_shapes):
    s = small_shapes["gqa_bf16"].with_(init_std=0.3)
    mask = synth.gen_skip_mask(s)
    w = synth.gen_host_weights(s, damp_skipped=0.4, skip_mask=mask)
    prompt = synth.gen_prompt(15, s.n_prompt, s.vocab)
    m = OracleModel(s, w, max_seq=64)
    sd = SpecDecoder(m, mask, 4)
    sd.generate(prompt, 18)
    assert sd.P == len(prompt) + len(sd.out) - 1            # cache holds every committed token but the pending one
    fresh = OracleModel(s, w, max_seq=64)
    seq = np.concatenate([prompt, np.asarray(sd.out[:-1], np.int32)])
    fresh.forward(seq, 0)
    (k1, v1), (k2, v2) = m.kv_arrays(), fresh.kv_arrays()
    assert np.array_equal(k1[:, :sd.P], k2[:, :sd.P]) and np.array_equal(v1[:, :sd.P], v2[:, :sd.P])
    # continuing from either state gives the same next logits
    a = m.forward([sd.t_last], sd.P)[0]
    b = fresh.forward([sd.t_last], sd.P)[0]
    assert np.abs(a - b).max() < 1e-12


def test_truncation_and_capacity(small_shapes):
    s = small_shapes["mha_f32"]
    w = synth.gen_host_weights(s)
    prompt = synth.gen_prompt(16, 6, s.vocab)
    sd = SpecDecoder(OracleModel(s, w, max_seq=40), np.zeros(s.n_layers, np.uint8), 4)
    assert len(sd.generate(prompt, 13)) == 13               # 1 + 5 + 5 + 5 truncated to 13
    sd = SpecDecoder(OracleModel(s, w, max_seq=12), np.zeros(s.n_layers, np.uint8), 4)
    with pytest.raises(ValueError):
        sd.generate(prompt, 30)


# ---- report formulas (P11) and the paper's printed figures ---------------------------------------------
def test_expected_tokens_per_step_closed_form_vs_simulation():
    rng = np.random.default_rng(0)
    for alpha, K in ((0.0, 4), (0.5, 4), (0.8, 6), (0.95, 5), (1.0, 3)):
        acc = rng.random((200000, K)) < alpha
        n = np.where(acc.all(1), K, np.argmin(acc, 1))
        assert abs((n + 1).mean() - expected_tokens_per_step(alpha, K)) < 0.02
    assert expected_tokens_per_step(0.0, 4) == 1.0 and expected_tokens_per_step(1.0, 4) == 5.0
    assert abs(projected_speedup(0.0, 4, 0.5) - 1 / 3) < 1e-12


def test_paper_table1_speedups_are_reachable_by_the_projection():
    """Table 1 rows (acceptance rate, speed-up) stored under tests/golden: each is consistent with the
    projection for some draft/target cost ratio c in (0, 1) and depth K in 2..8; the 13B row with half the
    layers skipped is not reachable at c >= 1 (a draft as slow as the target cannot speed anything up)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_table1.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 9
    for model, dataset, alpha, speedup in rows:
        alpha, speedup = float(alpha), float(speedup)
        ok = any(projected_speedup(alpha, K, c / 100) >= speedup and projected_speedup(alpha, K, 0.999) < speedup
                 for K in range(2, 9) for c in range(1, 100))
        assert ok, (model, dataset)
