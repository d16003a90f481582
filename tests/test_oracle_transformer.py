"""Pins for the encoder-layer oracle (Section 2.1: self-attention, feed-forward, residuals,
layer normalisation around the MoE layer).  CPU only; torch's float64 library routines and
closed forms are the independent evidence."""
import numpy as np
import torch

from oracle import moe_oracle as orc
from oracle import transformer_oracle as tro


def test_layer_norm_against_the_library_routine():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(3, 7, 24)) * 3 + 1
    g, b = rng.normal(size=24), rng.normal(size=24)
    want = torch.nn.functional.layer_norm(torch.tensor(x), (24,), torch.tensor(g), torch.tensor(b), eps=1e-6)
    np.testing.assert_allclose(tro.layer_norm(x, g, b), want.numpy(), rtol=1e-12, atol=1e-12)
    # rows come out with zero mean and unit variance before the affine part
    n = tro.layer_norm(x, np.ones(24), np.zeros(24))
    np.testing.assert_allclose(n.mean(-1), 0, atol=1e-12)
    np.testing.assert_allclose(n.var(-1), 1, rtol=1e-5)


def test_attention_against_the_library_routine():
    rng = np.random.default_rng(1)
    B, L, M, heads, d = 2, 11, 12, 3, 8
    A = heads * d
    u = rng.normal(size=(B, L, M))
    wq, wk, wv = (rng.normal(size=(M, A)) / np.sqrt(M) for _ in range(3))
    wo = rng.normal(size=(A, M)) / np.sqrt(A)
    got = tro.self_attention(u, wq, wk, wv, wo, heads)
    tu = torch.tensor(u)
    q, k, v = ((tu @ torch.tensor(w)).reshape(B, L, heads, d).transpose(1, 2) for w in (wq, wk, wv))
    ctx = torch.nn.functional.scaled_dot_product_attention(q, k, v)           # scale 1/sqrt(d)
    want = ctx.transpose(1, 2).reshape(B, L, A) @ torch.tensor(wo)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    B, L, M, heads, d = 1, 6, 8, 2, 4
    A = heads * d
    u = rng.normal(size=(B, L, M))
    wv = rng.normal(size=(M, A))
    wo = rng.normal(size=(A, M))
    # zero query/key projections: uniform attention, every position gets the mean value row
    got = tro.self_attention(u, np.zeros((M, A)), np.zeros((M, A)), wv, wo, heads)
    want = np.broadcast_to((u @ wv).mean(axis=1, keepdims=True) @ wo, (B, L, M))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # a single position attends to itself
    one = tro.self_attention(u[:, :1], rng.normal(size=(M, A)), rng.normal(size=(M, A)), wv, wo, heads)
    np.testing.assert_allclose(one, u[:, :1] @ wv @ wo, rtol=1e-12, atol=1e-12)
    # sequences are independent
    two = np.concatenate([u, rng.normal(size=(B, L, M))])
    wq, wk = rng.normal(size=(M, A)), rng.normal(size=(M, A))
    np.testing.assert_allclose(tro.self_attention(two, wq, wk, wv, wo, heads)[:1],
                               tro.self_attention(u, wq, wk, wv, wo, heads), rtol=1e-12, atol=1e-12)


def test_encoder_pair_is_the_composition_of_its_parts():
    rng = np.random.default_rng(3)
    B, L, M, H, heads, d, E, G, C = 2, 8, 8, 12, 2, 4, 4, 2, 5
    A = heads * d
    x = rng.normal(size=(B, L, M))
    p = {f"ln{i}": (1 + 0.1 * rng.normal(size=M), 0.1 * rng.normal(size=M)) for i in range(1, 5)}
    for i in (1, 2):
        for n in ("wq", "wk", "wv"):
            p[f"{n}{i}"] = rng.normal(size=(M, A)) / np.sqrt(M)
        p[f"wo{i}"] = rng.normal(size=(A, M)) / np.sqrt(A)
    p["w1"], p["w2"] = rng.normal(size=(M, H)) / np.sqrt(M), rng.normal(size=(H, M)) / np.sqrt(H)
    p["wg"] = rng.normal(size=(M, E)) / np.sqrt(M)
    p["wi"], p["wo"] = rng.normal(size=(E, M, H)) / np.sqrt(M), rng.normal(size=(E, H, M)) / np.sqrt(H)
    u = rng.random((G, B * L // G))
    y, aux, mid = tro.encoder_pair_forward(x, p, heads, G, C, u)
    # torch float64 restatement of the dense part
    tx = torch.tensor(x)
    ln = lambda v, i: torch.nn.functional.layer_norm(v, (M,), torch.tensor(p[f"ln{i}"][0]), torch.tensor(p[f"ln{i}"][1]), eps=1e-6)
    def att(v, i):
        q, k, vv = ((v @ torch.tensor(p[f"{n}{i}"])).reshape(B, L, heads, d).transpose(1, 2) for n in ("wq", "wk", "wv"))
        c = torch.nn.functional.scaled_dot_product_attention(q, k, vv).transpose(1, 2).reshape(B, L, A)
        return c @ torch.tensor(p[f"wo{i}"])
    a = tx + att(ln(tx, 1), 1)
    b = a + torch.relu(ln(a, 2) @ torch.tensor(p["w1"])) @ torch.tensor(p["w2"])
    c = b + att(ln(b, 3), 2)
    np.testing.assert_allclose(mid["c"], c.numpy(), rtol=1e-10, atol=1e-12)
    moe_in = ln(c, 4).numpy().reshape(G, -1, M)
    m, routing, _, _ = orc.moe_forward(moe_in, p["wg"], u, p["wi"], p["wo"], C)
    np.testing.assert_allclose(y, c.numpy() + m.reshape(B, L, M), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(aux, routing["aux"], rtol=1e-12)
