"""Pins of the oracle's FIT scores (Eq. 11; Alg. 1 Stage A) against things other than itself: PyTorch's automatic
differentiation of an independent float64 LLaMA forward written here from library routines, central finite
differences of the oracle's own loss, a case whose gradients are known to vanish, and the ranking rule on ties."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle.fit import LAYER_ATTN, LAYER_FFN, fit_scores, prune_set, sample_gradients


def _t(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return torch.tensor(a.astype(np.float64))


def torch_loss_and_grads(s, w, tokens):
    """Mean next-token cross-entropy of a float64 LLaMA forward (SDPA, complex rotary, F.silu, F.cross_entropy) and
    autograd's gradients of every layer tensor."""
    T, H, Hk, hd = len(tokens), s.n_heads, s.n_kv_heads, s.head_dim
    half = hd // 2
    params = [{k: _t(lw[k]).requires_grad_(True) for k in LAYER_ATTN + LAYER_FFN} for lw in w.layers]

    def rms(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + s.rms_eps) * g

    freqs = 1.0 / (s.rope_theta ** (torch.arange(0, half, dtype=torch.float64) * 2.0 / hd))
    rot = torch.polar(torch.ones(T, half, dtype=torch.float64), torch.outer(torch.arange(T, dtype=torch.float64), freqs))

    def rope(x):
        z = torch.complex(x[..., :half], x[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    h = _t(w.tok_emb)[torch.as_tensor(np.asarray(tokens), dtype=torch.long)]
    for p in params:
        x = rms(h, p["attn_norm"])
        q = rope((x @ p["wq"].T).view(T, H, hd))
        k = rope((x @ p["wk"].T).view(T, Hk, hd)).repeat_interleave(H // Hk, dim=1)
        v = (x @ p["wv"].T).view(T, Hk, hd).repeat_interleave(H // Hk, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        h = h + o.transpose(0, 1).reshape(T, H * hd) @ p["wo"].T
        x = rms(h, p["ffn_norm"])
        h = h + (F.silu(x @ p["w_gate"].T) * (x @ p["w_up"].T)) @ p["w_down"].T
    logits = rms(h, _t(w.final_norm)) @ _t(w.lm_head).T
    loss = F.cross_entropy(logits[:-1], torch.as_tensor(np.asarray(tokens[1:]), dtype=torch.long))
    loss.backward()
    return float(loss.detach()), [{k: p[k].grad.numpy() for k in p} for p in params]


@pytest.mark.parametrize("name", ["mha_f32", "gqa_bf16"])
def test_gradients_match_autograd_of_an_independent_forward(small_shapes, name):
    s = small_shapes[name]                      # seeded non-unit norm gains; grouped KV heads in the second shape
    w = synth.gen_host_weights(s)
    toks = synth.gen_prompt(11, 13, s.vocab)
    loss, grads = sample_gradients(s, w, toks)
    ref_loss, ref = torch_loss_and_grads(s, w, toks)
    assert abs(loss - ref_loss) < 1e-12 * max(1.0, abs(ref_loss))
    for l in range(s.n_layers):
        for k in LAYER_ATTN + LAYER_FFN:
            a, b = grads[l][k], ref[l][k].reshape(grads[l][k].shape)
            assert np.abs(a - b).max() <= 1e-10 * max(1e-30, np.abs(b).max()), (l, k)
    # and the scores are the sums of squares of exactly these gradients
    ta, tf, losses = fit_scores(s, w, [toks])
    for l in range(s.n_layers):
        assert np.isclose(ta[l], sum(float((ref[l][k] ** 2).sum()) for k in LAYER_ATTN), rtol=1e-9)
        assert np.isclose(tf[l], sum(float((ref[l][k] ** 2).sum()) for k in LAYER_FFN), rtol=1e-9)
    assert np.isclose(losses[0], ref_loss)


def test_directional_derivative_by_central_differences(small_shapes):
    """d/dt loss(W + t D) at t = 0 equals <grad W, D>, for a matrix of each sub-layer and a norm gain."""
    s = small_shapes["mha_f32"]
    w = synth.gen_host_weights(s)
    toks = synth.gen_prompt(5, 9, s.vocab)
    _, grads = sample_gradients(s, w, toks)
    rng = np.random.default_rng(0)
    for l, k in ((0, "wk"), (1, "w_gate"), (s.n_layers - 1, "wo"), (0, "ffn_norm")):
        base = w.layers[l][k].copy()
        D = rng.standard_normal(base.shape)
        t = 1e-5

        def loss_at(step):
            w.layers[l][k] = (base.astype(np.float64) + step * D).astype(np.float64)
            return sample_gradients(s, w, toks)[0]
        num = (loss_at(t) - loss_at(-t)) / (2 * t)
        w.layers[l][k] = base
        ana = float(np.sum(grads[l][k] * D))
        assert abs(num - ana) <= 1e-7 * max(1.0, abs(ana)), (l, k, num, ana)


def test_layers_that_output_nothing_have_gradient_only_in_their_output_projections(small_shapes):
    """With W_o = 0 and W_down = 0 in a layer, the loss does not depend on that layer's other tensors at all."""
    s = small_shapes["mha_f32"]
    w = synth.gen_host_weights(s)
    w.layers[1]["wo"] = np.zeros_like(w.layers[1]["wo"])
    w.layers[1]["w_down"] = np.zeros_like(w.layers[1]["w_down"])
    _, grads = sample_gradients(s, w, synth.gen_prompt(6, 10, s.vocab))
    for k in ("attn_norm", "wq", "wk", "wv", "ffn_norm", "w_gate", "w_up"):
        assert np.abs(grads[1][k]).max() == 0.0, k
    assert np.abs(grads[1]["wo"]).max() > 0 and np.abs(grads[1]["w_down"]).max() > 0
    assert np.abs(grads[0]["wq"]).max() > 0


def test_scores_are_means_over_the_calibration_set(small_shapes):
    s = small_shapes["gqa_bf16"]
    w = synth.gen_host_weights(s)
    a, b = synth.gen_prompt(1, 12, s.vocab), synth.gen_prompt(2, 7, s.vocab)
    ta, tf, _ = fit_scores(s, w, [a, b])
    ta1, tf1, _ = fit_scores(s, w, [a])
    ta2, tf2, _ = fit_scores(s, w, [b])
    assert np.allclose(ta, (ta1 + ta2) / 2, rtol=1e-12) and np.allclose(tf, (tf1 + tf2) / 2, rtol=1e-12)
    assert (ta > 0).all() and (tf > 0).all()


def test_prune_set_rule():
    assert prune_set([5.0, 1.0, 3.0, 2.0], 0.5) == [1, 3]
    assert prune_set([5.0, 1.0, 3.0, 2.0], 0.49) == [1]          # floor(r L)
    assert prune_set([2.0, 1.0, 1.0, 1.0], 0.5) == [1, 2]        # equal scores: the lower index goes first
    assert prune_set([1.0, 2.0], 0.0) == []
    assert prune_set([3.0, 2.0, 1.0], 1.0) == [0, 1, 2]
