"""Pins for the backward oracle of the encoder layers.  CPU only.  Independent evidence:
torch.autograd in float64 on the library's layer_norm / scaled_dot_product_attention, central
finite differences of the FORWARD oracle, closed forms."""
import numpy as np
import pytest
import torch

from oracle import transformer_oracle as tro
from oracle import transformer_oracle_backward as trb
from test_oracle_backward import _same_routing, _torch_dense_layer


def _t(a, grad=True):
    return torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=grad)


def test_layer_norm_backward_against_autograd():
    rng = np.random.default_rng(10)
    x = rng.normal(size=(3, 5, 24)) * 2 + 0.5
    g, b = 1 + 0.3 * rng.normal(size=24), rng.normal(size=24)
    dn = rng.normal(size=x.shape)
    tx, tg, tb = _t(x), _t(g), _t(b)
    n = torch.nn.functional.layer_norm(tx, (24,), tg, tb, eps=1e-6)
    (n * torch.tensor(dn)).sum().backward()
    dx, dg, db = trb.layer_norm_backward(x, g, dn)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-10, atol=1e-12)
    # the normalisation removes the mean and the scale of a row: dx is orthogonal to 1 and to xhat
    np.testing.assert_allclose(dx.sum(-1), 0, atol=1e-12)
    xhat = tro.layer_norm(x, np.ones(24), np.zeros(24))
    np.testing.assert_allclose((dx * xhat).sum(-1), 0, atol=1e-5)          # exact only for eps = 0


def _attention_inputs(rng, B, L, M, heads, d):
    A = heads * d
    u = rng.normal(size=(B, L, M))
    wq, wk, wv = (rng.normal(size=(M, A)) / np.sqrt(M) for _ in range(3))
    wo = rng.normal(size=(A, M)) / np.sqrt(A)
    return u, wq, wk, wv, wo


def _torch_attention(tu, twq, twk, twv, two, heads):
    B, L, _ = tu.shape
    A = twq.shape[1]
    d = A // heads
    q, k, v = ((tu @ w).reshape(B, L, heads, d).transpose(1, 2) for w in (twq, twk, twv))
    ctx = torch.nn.functional.scaled_dot_product_attention(q, k, v)
    return ctx.transpose(1, 2).reshape(B, L, A) @ two


@pytest.mark.parametrize("B,L,M,heads,d,seed", [(2, 9, 12, 3, 4, 0), (1, 17, 8, 2, 8, 1), (3, 4, 6, 1, 6, 2)])
def test_attention_backward_against_autograd(B, L, M, heads, d, seed):
    rng = np.random.default_rng(20 + seed)
    u, wq, wk, wv, wo = _attention_inputs(rng, B, L, M, heads, d)
    dout = rng.normal(size=(B, L, M))
    ts = [_t(a) for a in (u, wq, wk, wv, wo)]
    (_torch_attention(*ts, heads) * torch.tensor(dout)).sum().backward()
    got = trb.self_attention_backward(u, wq, wk, wv, wo, heads, dout)
    for g, t in zip(got, ts):
        np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_attention_backward_closed_forms():
    rng = np.random.default_rng(30)
    B, L, M, heads, d = 1, 6, 8, 2, 4
    A = heads * d
    u, _, _, wv, wo = _attention_inputs(rng, B, L, M, heads, d)
    dout = rng.normal(size=(B, L, M))
    zero = np.zeros((M, A))
    # zero query/key projections: out[l] = mean_l'(u[l'] wv) wo for every l, so
    # d/du[l'] = (1/L) sum_l dout[l] wo^T wv^T and no gradient reaches wq, wk through the scores
    # except via q = k = 0 (ds k = 0, ds^T q = 0)
    du, dwq, dwk, dwv, dwo = trb.self_attention_backward(u, zero, zero, wv, wo, heads, dout)
    want = np.broadcast_to(dout.sum(axis=1, keepdims=True) @ wo.T @ wv.T / L, u.shape)
    np.testing.assert_allclose(du, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dwq, 0, atol=1e-14)
    np.testing.assert_allclose(dwk, 0, atol=1e-14)
    np.testing.assert_allclose(dwv, u[0].mean(0)[:, None] * (dout[0].sum(0) @ wo.T)[None, :], rtol=1e-12)
    # a single position: out = u wv wo, the scores have no influence
    wq, wk = rng.normal(size=(M, A)), rng.normal(size=(M, A))
    du1, dwq1, dwk1, dwv1, dwo1 = trb.self_attention_backward(u[:, :1], wq, wk, wv, wo, heads, dout[:, :1])
    np.testing.assert_allclose(du1, dout[:, :1] @ wo.T @ wv.T, rtol=1e-12)
    np.testing.assert_allclose(dwq1, 0, atol=1e-14)
    np.testing.assert_allclose(dwo1, (u[0, :1] @ wv).T @ dout[0, :1], rtol=1e-12)


def test_dense_ffn_backward_against_autograd():
    rng = np.random.default_rng(40)
    u = rng.normal(size=(2, 7, 6))
    w1, w2 = rng.normal(size=(6, 10)), rng.normal(size=(10, 6))
    dout = rng.normal(size=u.shape)
    tu, t1, t2 = _t(u), _t(w1), _t(w2)
    ((torch.relu(tu @ t1) @ t2) * torch.tensor(dout)).sum().backward()
    du, dw1, dw2 = trb.dense_ffn_backward(u, w1, w2, dout)
    np.testing.assert_allclose(du, tu.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dw1, t1.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dw2, t2.grad.numpy(), rtol=1e-11, atol=1e-12)


def _pair_params(rng, M, H, heads, d, E):
    A = heads * d
    p = {f"ln{i}": (1 + 0.1 * rng.normal(size=M), 0.1 * rng.normal(size=M)) for i in range(1, 5)}
    for i in (1, 2):
        for n in ("wq", "wk", "wv"):
            p[f"{n}{i}"] = rng.normal(size=(M, A)) / np.sqrt(M)
        p[f"wo{i}"] = rng.normal(size=(A, M)) / np.sqrt(A)
    p["w1"], p["w2"] = rng.normal(size=(M, H)) / np.sqrt(M), rng.normal(size=(H, M)) / np.sqrt(H)
    p["wg"] = rng.normal(size=(M, E)) / np.sqrt(M)
    p["wi"], p["wo"] = rng.normal(size=(E, M, H)) / np.sqrt(M), rng.normal(size=(E, H, M)) / np.sqrt(H)
    return p


@pytest.mark.parametrize("seed", [0, 1])
def test_encoder_pair_backward_against_autograd(seed):
    rng = np.random.default_rng(50 + seed)
    B, L, M, H, heads, d, E, G, C = 2, 8, 8, 12, 2, 4, 4, 2, 5
    x = rng.normal(size=(B, L, M))
    p = _pair_params(rng, M, H, heads, d, E)
    u = rng.random((G, B * L // G))
    dy, daux = rng.normal(size=(B, L, M)), rng.normal(size=G)
    got = trb.encoder_pair_backward(x, p, heads, G, C, u, dy, daux)

    tp = {k: (tuple(_t(a) for a in v) if isinstance(v, tuple) else _t(v)) for k, v in p.items()}
    tx = _t(x)
    ln = lambda v, i: torch.nn.functional.layer_norm(v, (M,), tp[f"ln{i}"][0], tp[f"ln{i}"][1], eps=1e-6)
    att = lambda v, i: _torch_attention(v, tp[f"wq{i}"], tp[f"wk{i}"], tp[f"wv{i}"], tp[f"wo{i}"], heads)
    a = tx + att(ln(tx, 1), 1)
    b = a + torch.relu(ln(a, 2) @ tp["w1"]) @ tp["w2"]
    c = b + att(ln(b, 3), 2)
    m, aux = _torch_dense_layer(ln(c, 4).reshape(G, -1, M), tp["wg"], tp["wi"], tp["wo"],
                                got["moe"]["routing"], C)
    y = c + m.reshape(B, L, M)
    ((y * torch.tensor(dy)).sum() + (aux * torch.tensor(daux)).sum()).backward()

    np.testing.assert_allclose(got["dx"], tx.grad.numpy(), rtol=1e-8, atol=1e-11)
    for i in range(1, 5):
        np.testing.assert_allclose(got[f"ln{i}"][0], tp[f"ln{i}"][0].grad.numpy(), rtol=1e-8, atol=1e-11)
        np.testing.assert_allclose(got[f"ln{i}"][1], tp[f"ln{i}"][1].grad.numpy(), rtol=1e-8, atol=1e-11)
    for k in ("wq1", "wk1", "wv1", "wo1", "wq2", "wk2", "wv2", "wo2", "w1", "w2", "wg"):
        np.testing.assert_allclose(got[k], tp[k].grad.numpy(), rtol=1e-8, atol=1e-11, err_msg=k)
    for e in range(E):
        np.testing.assert_allclose(got["wi"][e], tp["wi"].grad[e].numpy(), rtol=1e-8, atol=1e-11)
        np.testing.assert_allclose(got["wo"][e], tp["wo"].grad[e].numpy(), rtol=1e-8, atol=1e-11)


def test_encoder_pair_backward_against_finite_differences():
    rng = np.random.default_rng(60)
    B, L, M, H, heads, d, E, G, C = 1, 8, 6, 8, 2, 3, 3, 1, 6
    x = rng.normal(size=(B, L, M))
    p = _pair_params(rng, M, H, heads, d, E)
    u = rng.random((G, B * L // G))
    dy, daux = rng.normal(size=(B, L, M)), rng.normal(size=G)
    got = trb.encoder_pair_backward(x, p, heads, G, C, u, dy, daux)

    def loss(xx, pp):
        y, aux, mid = tro.encoder_pair_forward(xx, pp, heads, G, C, u)
        return (dy * y).sum() + (daux * aux).sum(), mid["routing"]

    _, r0 = loss(x, p)
    h = 1e-6
    checked = 0
    # a few coordinates of x and of one weight of every kind
    targets = [("x", None, got["dx"])] + [(k, None, got[k]) for k in ("wq1", "wo2", "w1", "w2", "wg")] + \
              [("ln2", 0, got["ln2"][0]), ("ln3", 1, got["ln3"][1])]
    for name, part, grad in targets:
        base = x if name == "x" else (p[name][part] if part is not None else p[name])
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in base.shape)
            vals = []
            same = True
            for sgn in (+1, -1):
                pert = base.copy()
                pert[idx] += sgn * h
                if name == "x":
                    v, r = loss(pert, p)
                else:
                    pp = dict(p)
                    if part is None:
                        pp[name] = pert
                    else:
                        t = list(p[name]); t[part] = pert; pp[name] = tuple(t)
                    v, r = loss(x, pp)
                same = same and _same_routing(r0, r)
                vals.append(v)
            if not same:
                continue                                   # the step changed a routing decision
            fd = (vals[0] - vals[1]) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])
            checked += 1
    assert checked >= 36
