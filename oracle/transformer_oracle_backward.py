"""fp64 CPU oracle for the backward pass of the two MoE Transformer encoder layers (GShard).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the test-suite and the smoke check
may call it.  It shares no code with the HIP library and imports nothing from it.

The paper trains the model by automatic differentiation and prints no backward formulas
(Section 2.1 names the components of an encoder layer, Section 3.1 / Algorithm 2 the MoE
layer).  This file writes the derivative of

    L = sum dy * y  +  sum_g daux[g] * l_aux[g]

for the pair of layers of ``transformer_oracle.encoder_pair_forward`` out by the chain rule,
one function per forward function, every piece in float64 by its textbook form:

* ``layer_norm_backward``      n = gamma * xhat + beta, xhat = (x - mean) / sqrt(var + eps):
                               dx = rstd * (g - mean(g) - xhat * mean(g * xhat)), g = gamma * dn
* ``softmax_rows_backward``    p = softmax(s): ds = p * (dp - sum_k p dp)
* ``self_attention_backward``  the four projections and the scaled dot-product core
* ``dense_ffn_backward``       relu(u w1) w2 with relu'(0) = 0
* ``encoder_pair_backward``    the two layers, the MoE layer's part from
                               ``moe_oracle_backward.moe_backward`` (its readings B1-B5 apply)

Readings T1-T5 of the forward oracle apply unchanged (pre-LN, eps 1e-6, no bias, mask or
dropout).  The residual branches add their gradients.

Parity pins (tests/test_oracle_transformer_backward.py): torch.autograd in float64 on an
independent restatement with the library's layer_norm / scaled_dot_product_attention, central
finite differences of the forward oracle, closed forms (uniform attention, single position).
Nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from . import moe_oracle_backward as moe_bwd
from . import transformer_oracle as fwd


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def layer_norm_backward(x, gamma, dn, eps=fwd.LN_EPS):
    """Returns (dx, dgamma, dbeta) for n = LN(x) over the last axis."""
    x, gamma, dn = _f64(x), _f64(gamma), _f64(dn)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    g = dn * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    M = x.shape[-1]
    dgamma = (dn * xhat).reshape(-1, M).sum(axis=0)
    dbeta = dn.reshape(-1, M).sum(axis=0)
    return dx, dgamma, dbeta


def softmax_rows_backward(p, dp):
    p, dp = _f64(p), _f64(dp)
    return p * (dp - np.sum(p * dp, axis=-1, keepdims=True))


def self_attention_backward(u, wq, wk, wv, wo, heads, dout):
    """Gradients of out = Attention(u) (reading T3).  Returns (du, dwq, dwk, dwv, dwo)."""
    u, wq, wk, wv, wo, dout = (_f64(a) for a in (u, wq, wk, wv, wo, dout))
    B, L, M = u.shape
    A = wq.shape[1]
    d = A // heads
    u2 = u.reshape(B * L, M)
    q = (u @ wq).reshape(B, L, heads, d)
    k = (u @ wk).reshape(B, L, heads, d)
    v = (u @ wv).reshape(B, L, heads, d)
    ctx = np.zeros((B, L, heads, d))
    probs = np.zeros((B, heads, L, L))
    for b in range(B):
        for h in range(heads):
            s = q[b, :, h] @ k[b, :, h].T / np.sqrt(d)
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=-1, keepdims=True)
            probs[b, h] = p
            ctx[b, :, h] = p @ v[b, :, h]
    # out = ctx . wo
    dwo = ctx.reshape(B * L, A).T @ dout.reshape(B * L, M)
    dctx = (dout @ wo.T).reshape(B, L, heads, d)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b in range(B):
        for h in range(heads):
            p = probs[b, h]
            dv[b, :, h] = p.T @ dctx[b, :, h]
            dp = dctx[b, :, h] @ v[b, :, h].T
            ds = softmax_rows_backward(p, dp) / np.sqrt(d)
            dq[b, :, h] = ds @ k[b, :, h]
            dk[b, :, h] = ds.T @ q[b, :, h]
    dq2, dk2, dv2 = (a.reshape(B * L, A) for a in (dq, dk, dv))
    dwq, dwk, dwv = u2.T @ dq2, u2.T @ dk2, u2.T @ dv2
    du = (dq2 @ wq.T + dk2 @ wk.T + dv2 @ wv.T).reshape(B, L, M)
    return du, dwq, dwk, dwv, dwo


def dense_ffn_backward(u, w1, w2, dout):
    """out = relu(u w1) w2 (reading T4), relu'(0) = 0.  Returns (du, dw1, dw2)."""
    u, w1, w2, dout = _f64(u), _f64(w1), _f64(w2), _f64(dout)
    M = u.shape[-1]
    u2, d2 = u.reshape(-1, M), dout.reshape(-1, dout.shape[-1])
    pre = u2 @ w1
    hden = np.maximum(pre, 0.0)
    dw2 = hden.T @ d2
    dpre = np.where(pre > 0.0, d2 @ w2.T, 0.0)
    dw1 = u2.T @ dpre
    du = (dpre @ w1.T).reshape(u.shape)
    return du, dw1, dw2


def encoder_pair_backward(x, p, heads, G, C, u_rand, dy, daux):
    """Gradients of L for the two encoder layers; ``p`` as in ``encoder_pair_forward``.

    Returns a dict: dx [B,L,M]; ln1..ln4 -> (dgamma, dbeta); wq1, wk1, wv1, wo1, wq2, wk2, wv2,
    wo2, w1, w2; the MoE layer's wg [M,E], wi {e: [M,H]}, wo {e: [H,M]}; and ``moe`` = the MoE
    oracle's full result.
    """
    x, dy = _f64(x), _f64(dy)
    B, L, M = x.shape
    _, _, mid = fwd.encoder_pair_forward(x, p, heads, G, C, u_rand)
    a, b, c = mid["a"], mid["b"], mid["c"]
    out = {}
    # y = c + MoE(LN4(c))
    m = moe_bwd.moe_backward(mid["moe_in"], p["wg"], u_rand, p["wi"], p["wo"], C,
                             dy.reshape(G, -1, M), daux)
    out["moe"] = m
    out["wg"], out["wi"], out["wo"] = m["dwg"], m["dwi"], m["dwo"]
    dln, dg, db_ = layer_norm_backward(c, p["ln4"][0], m["dx"].reshape(B, L, M))
    out["ln4"] = (dg, db_)
    dc = dy + dln
    # c = b + Attention_2(LN3(b))
    n3 = fwd.layer_norm(b, *p["ln3"])
    dn3, out["wq2"], out["wk2"], out["wv2"], out["wo2"] = self_attention_backward(
        n3, p["wq2"], p["wk2"], p["wv2"], p["wo2"], heads, dc)
    dln, dg, db_ = layer_norm_backward(b, p["ln3"][0], dn3)
    out["ln3"] = (dg, db_)
    dbb = dc + dln
    # b = a + FFN(LN2(a))
    n2 = fwd.layer_norm(a, *p["ln2"])
    dn2, out["w1"], out["w2"] = dense_ffn_backward(n2, p["w1"], p["w2"], dbb)
    dln, dg, db_ = layer_norm_backward(a, p["ln2"][0], dn2)
    out["ln2"] = (dg, db_)
    da = dbb + dln
    # a = x + Attention_1(LN1(x))
    n1 = fwd.layer_norm(x, *p["ln1"])
    dn1, out["wq1"], out["wk1"], out["wv1"], out["wo1"] = self_attention_backward(
        n1, p["wq1"], p["wk1"], p["wv1"], p["wo1"], heads, da)
    dln, dg, db_ = layer_norm_backward(x, p["ln1"][0], dn1)
    out["ln1"] = (dg, db_)
    out["dx"] = da + dln
    return out
