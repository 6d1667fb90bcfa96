"""Pins for the oracle's transformer forward (CPU only).

None of these re-type the oracle's formula: the main pin is an independent LLaMA forward built here from
PyTorch library routines (scaled_dot_product_attention, complex-number rotary, F.silu, matmul) without any
cache; the others are brute-force recomputation, closed forms and invariants.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import OracleModel
from oracle import model as om


def _to_t(a, dtype):
    if dtype == "bf16":
        return torch.from_numpy(synth.bf16_bits_to_f32(a).reshape(a.shape)).double()
    return torch.from_numpy(a).double()


def torch_llama_logits(shape, w, tokens, skip=None):
    """Independent full-sequence forward (no cache), float64, library ops.  Returns [T, V] logits."""
    s = shape
    T = len(tokens)
    H, Hk, hd = s.n_heads, s.n_kv_heads, s.head_dim
    dt = s.dtype

    def store(x):  # values as they would read back from a cache of the storage type
        return x.float().to(torch.bfloat16).double() if dt == "bf16" else x.float().double()

    def rms(x, g):
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + s.rms_eps) * torch.from_numpy(g).double()

    def rot(x):  # x [T, heads, hd] ; complex rotation of the pair (i, i + hd/2)
        half = hd // 2
        freqs = 1.0 / (s.rope_theta ** (torch.arange(0, half, dtype=torch.float64) * 2.0 / hd))
        ang = torch.outer(torch.arange(T, dtype=torch.float64), freqs)          # [T, half]
        z = torch.complex(x[..., :half], x[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    h = _to_t(w.tok_emb, dt)[torch.as_tensor(np.asarray(tokens), dtype=torch.long)]
    for l, lw in enumerate(w.layers):
        sk = 0 if skip is None else int(skip[l])
        if not sk & 1:
            x = rms(h, lw["attn_norm"])
            q = (x @ _to_t(lw["wq"], dt).T).view(T, H, hd)
            k = (x @ _to_t(lw["wk"], dt).T).view(T, Hk, hd)
            v = (x @ _to_t(lw["wv"], dt).T).view(T, Hk, hd)
            q, k = rot(q), store(rot(k))
            v = store(v)
            k = k.repeat_interleave(H // Hk, dim=1)
            v = v.repeat_interleave(H // Hk, dim=1)
            o = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                               is_causal=True)
            h = h + o.transpose(0, 1).reshape(T, H * hd) @ _to_t(lw["wo"], dt).T
        if not sk & 2:
            x = rms(h, lw["ffn_norm"])
            a = F.silu(x @ _to_t(lw["w_gate"], dt).T) * (x @ _to_t(lw["w_up"], dt).T)
            h = h + a @ _to_t(lw["w_down"], dt).T
    return (rms(h, w.final_norm) @ _to_t(w.lm_head, dt).T).numpy()


@pytest.mark.parametrize("name", ["tiny", "mha_f32", "gqa_bf16"])
def test_forward_matches_independent_torch_llama(small_shapes, name):
    s = small_shapes[name]
    w = synth.gen_host_weights(s)
    toks = synth.gen_prompt(7, 19, s.vocab)
    ref = torch_llama_logits(s, w, toks)
    got = OracleModel(s, w).forward(toks, 0)
    assert np.abs(got - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())
    # with a skip mask (draft model) as well, including half-skipped layers
    skip = np.zeros(s.n_layers, np.uint8)
    skip[0] = 1; skip[1] = 3; skip[-1] = 2
    ref = torch_llama_logits(s, w, toks, skip)
    got = OracleModel(s, w).forward(toks, 0, skip)
    assert np.abs(got - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())


def test_norm_gains_are_used(small_shapes):
    s = small_shapes["mha_f32"]
    w = synth.gen_host_weights(s)
    rng = np.random.default_rng(1)
    for lw in w.layers:
        lw["attn_norm"] = (1 + 0.3 * rng.standard_normal(s.d_model)).astype(np.float32)
        lw["ffn_norm"] = (1 + 0.3 * rng.standard_normal(s.d_model)).astype(np.float32)
    w.final_norm = (1 + 0.3 * rng.standard_normal(s.d_model)).astype(np.float32)
    toks = synth.gen_prompt(8, 11, s.vocab)
    assert np.abs(OracleModel(s, w).forward(toks, 0) - torch_llama_logits(s, w, toks)).max() < 1e-10


def test_cached_forward_equals_full_recompute(small_shapes):
    """Definition of KV caching: any split of the sequence into successive calls gives the same logits."""
    for name in ("mha_f32", "gqa_bf16"):
        s = small_shapes[name]
        w = synth.gen_host_weights(s)
        toks = synth.gen_prompt(3, 17, s.vocab)
        full = OracleModel(s, w).forward(toks, 0)
        m = OracleModel(s, w)
        parts = [m.forward(toks[:6], 0)]
        parts += [m.forward(toks[i:i + 1], i) for i in range(6, 10)]
        parts.append(m.forward(toks[10:17], 10))
        assert np.abs(np.concatenate(parts) - full).max() < 1e-12


def test_multi_row_row_equals_single_row_decode(small_shapes):
    """Row i of a causal (K+1)-row forward is the one-row decode of the same prefix."""
    s = small_shapes["gqa_bf16"]
    w = synth.gen_host_weights(s)
    toks = synth.gen_prompt(4, 13, s.vocab)
    m = OracleModel(s, w)
    m.forward(toks[:8], 0)
    rows = m.forward(toks[8:13], 8)
    m2 = OracleModel(s, w)
    m2.forward(toks[:8], 0)
    for i in range(5):
        one = m2.forward(toks[8 + i:9 + i], 8 + i)[0]
        assert np.abs(one - rows[i]).max() < 1e-12


def test_skipped_layers_pass_through_and_write_no_kv(small_shapes):
    s = small_shapes["mha_f32"]
    w = synth.gen_host_weights(s)
    toks = synth.gen_prompt(5, 6, s.vocab)
    m = OracleModel(s, w)
    allskip = np.full(s.n_layers, 3, np.uint8)
    got = m.forward(toks, 0, allskip)
    # closed form: logits = lm_head . (rmsnorm(embedding) * final gain)
    e = w.tok_emb[toks].astype(np.float64)
    x = e / np.sqrt((e * e).mean(-1, keepdims=True) + s.rms_eps) * w.final_norm.astype(np.float64)
    assert np.abs(got - x @ w.lm_head.astype(np.float64).T).max() < 1e-12
    k, v = m.kv_arrays()
    assert not k.any() and not v.any()
    # skipping only layer 1: its cache rows stay zero, the others are written at exactly the fed positions
    m = OracleModel(s, w)
    sk = np.zeros(s.n_layers, np.uint8); sk[1] = 3
    m.forward(toks, 2, sk)
    k, v = m.kv_arrays()
    assert not k[1].any() and not v[1].any()
    for l in (0, 2):
        assert k[l, 2:8].any() and v[l, 2:8].any()
        assert not k[l, :2].any() and not k[l, 8:].any()


def test_gqa_equals_mha_with_replicated_kv_heads(small_shapes):
    """Grouped-query attention is MHA whose K/V projections are repeated per group (head h uses KV head h//g)."""
    s = small_shapes["gqa_bf16"]
    w = synth.gen_host_weights(s)
    g = s.n_heads // s.n_kv_heads
    s_mha = s.with_(n_kv_heads=s.n_heads)
    w2 = synth.gen_host_weights(s)
    for lw in w2.layers:
        for nm in ("wk", "wv"):
            a = lw[nm].reshape(s.n_kv_heads, s.head_dim, s.d_model)
            lw[nm] = np.ascontiguousarray(np.repeat(a, g, axis=0).reshape(s.n_heads * s.head_dim, s.d_model))
    toks = synth.gen_prompt(6, 12, s.vocab)
    a = OracleModel(s, w).forward(toks, 0)
    b = OracleModel(s_mha, w2).forward(toks, 0)
    assert np.abs(a - b).max() < 1e-12


def test_kv_cache_holds_storage_rounded_values(small_shapes):
    s = small_shapes["gqa_bf16"]
    w = synth.gen_host_weights(s)
    m = OracleModel(s, w)
    m.forward(synth.gen_prompt(9, 5, s.vocab), 0)
    k, v = m.kv_arrays()
    for a in (k[0, :5], v[3, :5]):
        assert a.any()
        assert np.array_equal(a.view(np.uint32) & 0xFFFF, np.zeros_like(a, np.uint32))   # exactly bf16-representable
    assert om.round_storage(1.00390625, "bf16") == 1.0            # tie rounds to even
    assert om.round_storage(1.01171875, "bf16") == 1.015625       # tie rounds to even (up)
    assert om.round_storage(1.0 + 2.0 ** -30, "f32") == 1.0


# ---- primitives ------------------------------------------------------------------------------------------
def test_rope_invariants():
    rng = np.random.default_rng(0)
    hd, theta = 64, 10000.0
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    assert np.allclose(om.rope(q, 0, theta), q, atol=0, rtol=0)
    for pos in (1, 17, 4095):
        assert abs(np.linalg.norm(om.rope(q, pos, theta)) - np.linalg.norm(q)) < 1e-12
    # inner product depends on the position difference only
    a = om.rope(q, 100, theta) @ om.rope(k, 93, theta)
    b = om.rope(q, 1007, theta) @ om.rope(k, 1000, theta)
    assert abs(a - b) < 1e-10
    # explicit 2-d case: hd = 2, frequency 1 -> plain rotation by pos radians
    r = om.rope(np.array([1.0, 0.0]), 1, theta)
    assert np.allclose(r, [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    # pairing is (i, i + hd/2) and the second pair turns slower: theta^(-2/4)
    r = om.rope(np.array([0.0, 1.0, 0.0, 0.0]), 3, 100.0)
    assert np.allclose(r, [0.0, math.cos(0.3), 0.0, math.sin(0.3)], atol=1e-15)


def test_rmsnorm_unit_rms_and_gain():
    rng = np.random.default_rng(1)
    h = rng.standard_normal(300) * 7.0
    out = om.rmsnorm(h, np.ones(300, np.float32), 0.0)
    assert abs(np.sqrt((out ** 2).mean()) - 1.0) < 1e-12
    g = rng.standard_normal(300).astype(np.float32)
    assert np.allclose(om.rmsnorm(h, g, 1e-5), h / np.sqrt((h * h).mean() + 1e-5) * g, rtol=1e-14)
    assert np.allclose(om.rmsnorm(np.zeros(4), np.ones(4, np.float32), 1e-5), 0.0)


def test_matmul_against_numpy_both_storage_types():
    rng = np.random.default_rng(2)
    W = (rng.standard_normal((37, 53)) * 0.02).astype(np.float32)
    X = rng.standard_normal((5, 53))
    assert np.allclose(om.matmul(W, "f32", X), X @ W.astype(np.float64).T, rtol=1e-13, atol=1e-15)
    Wb = synth.f32_to_bf16_bits(W).reshape(W.shape)
    Wd = synth.bf16_bits_to_f32(Wb).reshape(W.shape).astype(np.float64)
    got = om.matmul(Wb, "bf16", X)
    assert np.allclose(got, X @ Wd.T, rtol=1e-13, atol=1e-15)
    assert got.shape == (5, 37)                       # [M, N]: not transposed
    one = om.matmul(Wb, "bf16", X[2:3])
    assert np.allclose(one[0], got[2], rtol=1e-15)


def test_attend_against_closed_forms():
    rng = np.random.default_rng(3)
    hd, n = 16, 9
    q = rng.standard_normal(hd)
    kc = rng.standard_normal((n, hd)).astype(np.float32)
    vc = rng.standard_normal((n, hd)).astype(np.float32)
    s = kc.astype(np.float64) @ q / math.sqrt(hd)
    p = np.exp(s - s.max()); p /= p.sum()
    assert np.allclose(om.attend(q, kc, vc), p @ vc.astype(np.float64), rtol=1e-13)
    # one position: output is that value vector; zero query: plain mean of the values
    assert np.allclose(om.attend(q, kc[:1], vc[:1]), vc[0], rtol=1e-15)
    assert np.allclose(om.attend(np.zeros(hd), kc, vc), vc.astype(np.float64).mean(0), rtol=1e-13)
    # a huge score on one key must not overflow and selects that value
    kc2 = kc.copy(); kc2[4] = (q * 1e4).astype(np.float32)
    assert np.allclose(om.attend(q, kc2, vc), vc[4], rtol=1e-12)


def test_silu_closed_forms():
    assert om.silu(0.0) == 0.0
    for z in (0.3, 2.0, 11.0):
        assert abs(om.silu(z) - om.silu(-z) - z) < 4e-15          # silu(z) - silu(-z) = z
        assert abs(om.silu(z) - z / (1 + math.exp(-z))) < 4e-15
    assert abs(om.silu(40.0) - 40.0) < 1e-12 and abs(om.silu(-40.0)) < 1e-12


def test_bad_arguments_are_rejected(small_shapes):
    s = small_shapes["mha_f32"]
    w = synth.gen_host_weights(s)
    m = OracleModel(s, w, max_seq=8)
    with pytest.raises(ValueError):
        m.forward(np.zeros(9, np.int32), 0)
    with pytest.raises(ValueError):
        m.forward([s.vocab], 0)
    with pytest.raises(ValueError):
        m.forward([0], 8)
