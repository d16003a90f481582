"""fp64 CPU oracle for the MoE Transformer encoder layers around the MoE layer (GShard).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the test-suite and the smoke check
may call it.  It shares no code with the HIP library and imports nothing from it.

Section 2.1 of the paper: a Transformer encoder layer is a self-attention layer followed by a
position-wise feed-forward layer, "interleaved with residual connections and layer
normalization"; the MoE Transformer replaces every other feed-forward layer with the MoE
layer.  This file evaluates one such pair of encoder layers,

    layer 1:  a  = x  + Attention_1(LN(x))        b  = a + FFN(LN(a))          (dense)
    layer 2:  c  = b  + Attention_2(LN(b))        y  = c + MoE(LN(c))          (Eq. 1-3)

in float64, every piece by its textbook definition.

Readings (the paper only names the components; Appendix "Machine Translation Experiments
Details" gives M = 1024, H = 8192, 16 heads, key/value dimension 128):

T1  Layer normalisation comes first in each sub-layer and the residual is added to the
    un-normalised input (pre-LN).  The paper does not say; this is the arrangement that the
    deep (36-60 layer) models of the paper need to train stably.
T2  LN(x) = gamma * (x - mean) / sqrt(var + eps) + beta over the model dimension, population
    variance, eps = 1e-6.
T3  Multi-head attention: per head h, softmax(Q_h K_h^T / sqrt(d)) V_h with Q = u Wq,
    K = u Wk, V = u Wv (each [M, heads*d]), heads concatenated, then Wo [heads*d, M].
    No biases (the experts have none either), no attention mask (every sequence of the
    synthetic batch has the full length L), no dropout (evaluation mode; the paper trains
    with rate 0.1).
T4  The dense feed-forward layer has the expert's form, relu(u W1) W2, without biases.
T5  Tokens are the rows of a [B, L, M] batch; the MoE layer sees them as G groups of S
    (B*L = G*S, row-major order unchanged), Section 2.2 "Local group dispatching".

Parity pins (tests/test_oracle_transformer.py): torch.nn.functional.layer_norm and
scaled_dot_product_attention in float64, a single-head / single-key closed form, the MoE
oracle itself for the last sub-layer.  Nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from . import moe_oracle as moe

LN_EPS = 1e-6


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def layer_norm(x, gamma, beta, eps=LN_EPS):
    """Reading T2, over the last axis."""
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return _f64(gamma) * (x - mu) / np.sqrt(var + eps) + _f64(beta)


def self_attention(u, wq, wk, wv, wo, heads):
    """Reading T3.  u [B,L,M]; wq, wk, wv [M, heads*d]; wo [heads*d, M]  ->  [B,L,M]."""
    u, wq, wk, wv, wo = _f64(u), _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    B, L, M = u.shape
    A = wq.shape[1]
    d = A // heads
    q = (u @ wq).reshape(B, L, heads, d)
    k = (u @ wk).reshape(B, L, heads, d)
    v = (u @ wv).reshape(B, L, heads, d)
    ctx = np.zeros((B, L, heads, d))
    for b in range(B):
        for h in range(heads):
            s = q[b, :, h] @ k[b, :, h].T / np.sqrt(d)            # [L queries, L keys]
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=-1, keepdims=True)
            ctx[b, :, h] = p @ v[b, :, h]
    return ctx.reshape(B, L, A) @ wo


def dense_ffn(u, w1, w2):
    """Reading T4."""
    return np.maximum(_f64(u) @ _f64(w1), 0.0) @ _f64(w2)


def encoder_pair_forward(x, p, heads, G, C, u_rand):
    """The two encoder layers of the module header.

    x [B,L,M]; p: dict with ln1..ln4 = (gamma, beta), attention weights wq1, wk1, wv1, wo1,
    wq2, wk2, wv2, wo2, dense FFN w1, w2, and the MoE layer's wg [M,E], wi [E,M,H], wo [E,H,M];
    u_rand [G,S] uniforms of the MoE layer's random routing; C expert capacity.
    Returns (y [B,L,M], aux [G], intermediates dict).
    """
    x = _f64(x)
    B, L, M = x.shape
    a = x + self_attention(layer_norm(x, *p["ln1"]), p["wq1"], p["wk1"], p["wv1"], p["wo1"], heads)
    b = a + dense_ffn(layer_norm(a, *p["ln2"]), p["w1"], p["w2"])
    c = b + self_attention(layer_norm(b, *p["ln3"]), p["wq2"], p["wk2"], p["wv2"], p["wo2"], heads)
    moe_in = layer_norm(c, *p["ln4"]).reshape(G, (B * L) // G, M)
    m, routing, _, _ = moe.moe_forward(moe_in, p["wg"], u_rand, p["wi"], p["wo"], C)
    y = c + m.reshape(B, L, M)
    return y, routing["aux"], {"a": a, "b": b, "c": c, "moe_in": moe_in, "routing": routing}
