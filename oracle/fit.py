"""FIT layer scores and the prune set (paper Sec. III-A / III-B, Eq. 9 and Eq. 11; Alg. 1 Stage A), on the CPU in float64.
TEST INFRASTRUCTURE ONLY: nothing in the product path may import this module.

What is computed.  For every sample z_i = (tokens x_0 .. x_{T-1}) of the calibration set, the loss f(z_i, theta) is the
mean next-token cross-entropy of the model's logits at positions 0 .. T-2 against x_1 .. x_{T-1}.  The score of
layer l is the empirical Fisher trace of its parameters, Eq. 11:

    T_l = 1/N * sum_i || grad_{theta_l} f(z_i, theta) ||_2^2 ,

with theta_l = {attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down} of layer l.  The two halves of the sum --
the attention sub-layer's five tensors and the feed-forward sub-layer's four -- are returned separately as well
(Sec. IV-A prunes attention and feed-forward sub-layers at separate ratios).  Alg. 1 then sorts the layers by
ascending T_l and removes the first floor(r * L).

The forward is the model of `sdfp_oracle.c` run over a whole sequence without a cache: pre-norm residual blocks,
RMSNorm, rotary embedding in the (i, i + hd/2) pairing, causal soft-max attention with grouped KV heads, SwiGLU.
Weights are the stored values (bfloat16 bit patterns or float32) taken exactly; nothing else is rounded -- in
particular keys and values are not rounded to the storage type here, there is no cache in this pass.  The backward
is the chain rule written out operation by operation; the gradient of every weight matrix is formed in full
(grad W = dY^T X) and its squares summed, the plain definition of the norm in Eq. 11.
"""
from __future__ import annotations

import numpy as np

LAYER_ATTN = ("attn_norm", "wq", "wk", "wv", "wo")
LAYER_FFN = ("ffn_norm", "w_gate", "w_up", "w_down")


def _f64(a):
    """A stored tensor as float64: float32 values, or bfloat16 bit patterns (uint16)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _rope_tables(shape, T):
    half = shape.head_dim // 2
    inv = 1.0 / (float(shape.rope_theta) ** (np.arange(half, dtype=np.float64) * 2.0 / shape.head_dim))
    ang = np.outer(np.arange(T, dtype=np.float64), inv)          # [T, half]
    return np.cos(ang), np.sin(ang)


def _rotate(x, cos, sin, inverse=False):
    """x: [T, heads, hd]; pairs (i, i + hd/2) rotated by the position's angle (by minus the angle if inverse)."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], (-sin if inverse else sin)[:, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def _rms_forward(x, gain, eps):
    rs = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)   # [T, 1]
    return x * rs * gain, rs


def _rms_backward(x, gain, rs, dy):
    """y = x * rs * gain with rs = (mean(x^2) + eps)^(-1/2).  Returns (dx, dgain)."""
    d = x.shape[-1]
    dgain = np.sum(dy * x * rs, axis=0)
    gdy = dy * gain
    dx = gdy * rs - x * (rs ** 3) * np.sum(gdy * x, axis=-1, keepdims=True) / d
    return dx, dgain


def sample_gradients(shape, weights, tokens):
    """Loss of one sample and the gradient of every layer tensor.

    Returns (loss, grads) with grads[l][slot] an array of the tensor's shape (float64)."""
    s = shape
    T = len(tokens)
    assert T >= 2
    H, Hk, hd, d = s.n_heads, s.n_kv_heads, s.head_dim, s.d_model
    grp = H // Hk
    eps = float(s.rms_eps)
    cos, sin = _rope_tables(s, T)
    tok = np.asarray(tokens, dtype=np.int64)
    causal = np.tril(np.ones((T, T), dtype=bool))
    scale = 1.0 / np.sqrt(hd)

    # ---- forward, keeping what the backward needs
    h = _f64(weights.tok_emb)[tok]                               # [T, d]
    saved = []
    for lw in weights.layers:
        W = {k: _f64(lw[k]) for k in LAYER_ATTN + LAYER_FFN}
        n1, rs1 = _rms_forward(h, W["attn_norm"], eps)
        q = _rotate((n1 @ W["wq"].T).reshape(T, H, hd), cos, sin)
        k = _rotate((n1 @ W["wk"].T).reshape(T, Hk, hd), cos, sin)
        v = (n1 @ W["wv"].T).reshape(T, Hk, hd)
        P = np.zeros((H, T, T))
        att = np.zeros((T, H, hd))
        for hq in range(H):
            g = hq // grp
            sc = (q[:, hq, :] @ k[:, g, :].T) * scale            # [T, T]
            sc = np.where(causal, sc, -np.inf)
            sc = sc - sc.max(axis=-1, keepdims=True)
            e = np.exp(sc)
            P[hq] = e / e.sum(axis=-1, keepdims=True)
            att[:, hq, :] = P[hq] @ v[:, g, :]
        att2 = att.reshape(T, H * hd)
        h_mid = h + att2 @ W["wo"].T
        n2, rs2 = _rms_forward(h_mid, W["ffn_norm"], eps)
        gt = n2 @ W["w_gate"].T
        up = n2 @ W["w_up"].T
        sig = 1.0 / (1.0 + np.exp(-gt))
        act = gt * sig * up
        h_out = h_mid + act @ W["w_down"].T
        saved.append(dict(W=W, x1=h, n1=n1, rs1=rs1, q=q, k=k, v=v, P=P, att2=att2, x2=h_mid, n2=n2, rs2=rs2,
                          gt=gt, up=up, sig=sig, act=act))
        h = h_out
    gf = _f64(weights.final_norm)
    nf, rsf = _rms_forward(h, gf, eps)
    Wh = _f64(weights.lm_head)
    logits = nf @ Wh.T                                           # [T, V]

    # ---- loss: mean over positions 0 .. T-2 of -log softmax(logits_t)[x_{t+1}]
    z = logits[:-1]
    z = z - z.max(axis=-1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=-1, keepdims=True))
    tgt = tok[1:]
    loss = -np.mean(logp[np.arange(T - 1), tgt])

    # ---- backward
    dlogits = np.zeros_like(logits)
    p = np.exp(logp)
    p[np.arange(T - 1), tgt] -= 1.0
    dlogits[:-1] = p / (T - 1)
    dnf = dlogits @ Wh
    dh, _ = _rms_backward(h, gf, rsf, dnf)
    grads = [None] * len(saved)
    for l in range(len(saved) - 1, -1, -1):
        S = saved[l]
        W = S["W"]
        g = {}
        # feed-forward sub-layer: h_out = h_mid + act W_down^T
        g["w_down"] = dh.T @ S["act"]
        dact = dh @ W["w_down"]
        dup = dact * S["gt"] * S["sig"]
        dgt = dact * S["up"] * (S["sig"] * (1.0 + S["gt"] * (1.0 - S["sig"])))
        g["w_up"] = dup.T @ S["n2"]
        g["w_gate"] = dgt.T @ S["n2"]
        dn2 = dup @ W["w_up"] + dgt @ W["w_gate"]
        dx2, g["ffn_norm"] = _rms_backward(S["x2"], W["ffn_norm"], S["rs2"], dn2)
        dh_mid = dh + dx2
        # attention sub-layer: h_mid = h + att W_o^T
        g["wo"] = dh_mid.T @ S["att2"]
        datt = (dh_mid @ W["wo"]).reshape(T, H, hd)
        dq = np.zeros_like(S["q"])
        dk = np.zeros_like(S["k"])
        dv = np.zeros_like(S["v"])
        for hq in range(H):
            kv = hq // grp
            P = S["P"][hq]
            dP = datt[:, hq, :] @ S["v"][:, kv, :].T             # [T, T]
            dv[:, kv, :] += P.T @ datt[:, hq, :]
            dS = P * (dP - np.sum(P * dP, axis=-1, keepdims=True))
            dq[:, hq, :] = (dS @ S["k"][:, kv, :]) * scale
            dk[:, kv, :] += (dS.T @ S["q"][:, hq, :]) * scale
        dq_pre = _rotate(dq, cos, sin, inverse=True).reshape(T, H * hd)
        dk_pre = _rotate(dk, cos, sin, inverse=True).reshape(T, Hk * hd)
        dv2 = dv.reshape(T, Hk * hd)
        g["wq"] = dq_pre.T @ S["n1"]
        g["wk"] = dk_pre.T @ S["n1"]
        g["wv"] = dv2.T @ S["n1"]
        dn1 = dq_pre @ W["wq"] + dk_pre @ W["wk"] + dv2 @ W["wv"]
        dx1, g["attn_norm"] = _rms_backward(S["x1"], W["attn_norm"], S["rs1"], dn1)
        dh = dh_mid + dx1
        grads[l] = g
    return float(loss), grads


def fit_scores(shape, weights, samples):
    """Eq. 11 over the calibration set `samples` (a sequence of token sequences).

    Returns (T_attn, T_ffn, losses): float64 arrays [L], [L] and [N]; the layer score T_l is T_attn[l] + T_ffn[l]."""
    L = shape.n_layers
    t_attn, t_ffn = np.zeros(L), np.zeros(L)
    losses = []
    for toks in samples:
        loss, grads = sample_gradients(shape, weights, toks)
        losses.append(loss)
        for l, g in enumerate(grads):
            t_attn[l] += sum(float(np.sum(g[k] ** 2)) for k in LAYER_ATTN)
            t_ffn[l] += sum(float(np.sum(g[k] ** 2)) for k in LAYER_FFN)
    n = len(losses)
    return t_attn / n, t_ffn / n, np.asarray(losses)


def prune_set(scores, ratio):
    """Alg. 1 Stage A, last step: the floor(ratio * L) layers of smallest score (equal scores: lower index first),
    as a sorted list of layer indices."""
    scores = np.asarray(scores, dtype=np.float64)
    n = int(np.floor(ratio * len(scores) + 1e-12))
    order = sorted(range(len(scores)), key=lambda l: (scores[l], l))
    return sorted(order[:n])
