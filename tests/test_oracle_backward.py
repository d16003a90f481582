"""Pins for the backward oracle (chain rule through Eq. 1-3 and Algorithms 1-2).  CPU only.

Independent evidence, none of it the oracle's own formulas retyped:
* central finite differences of the FORWARD oracle (routing checked unchanged),
* torch.autograd on a dense float64 restatement of Algorithm 2's einsums,
* closed forms / special cases.
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from oracle import moe_oracle_backward as bwd


def _rand_layer(rng, G, S, M, H, E):
    x = rng.normal(size=(G, S, M))
    wg = rng.normal(size=(M, E)) / np.sqrt(M)
    wi = rng.normal(size=(E, M, H)) / np.sqrt(M)
    wo = rng.normal(size=(E, H, M)) / np.sqrt(H)
    u = rng.random((G, S))
    dy = rng.normal(size=(G, S, M))
    daux = rng.normal(size=(G,))
    return x, wg, u, wi, wo, dy, daux


def _loss(x, wg, u, wi, wo, C, dy, daux):
    y, routing, _, _ = orc.moe_forward(x, wg, u, wi, wo, C)
    return float((dy * y).sum() + (daux * routing["aux"]).sum()), routing


def _same_routing(a, b):
    return (a["expert_idx"] == b["expert_idx"]).all() and (a["slot"] == b["slot"]).all()


# G, S, M, H, E, C chosen so that the cases contain overflowing first choices, second choices
# that are not sampled, second choices that overflow and tokens that keep only their second.
FD_CASES = [(2, 14, 5, 6, 4, 4, 0), (1, 20, 4, 7, 3, 5, 1), (3, 9, 6, 5, 5, 2, 2), (1, 12, 3, 4, 2, 12, 3)]


@pytest.mark.parametrize("G,S,M,H,E,C,seed", FD_CASES)
def test_against_finite_differences_of_the_forward_oracle(G, S, M, H, E, C, seed):
    rng = np.random.default_rng(100 + seed)
    x, wg, u, wi, wo, dy, daux = _rand_layer(rng, G, S, M, H, E)
    got = bwd.moe_backward(x, wg, u, wi, wo, C, dy, daux)
    base, routing0 = _loss(x, wg, u, wi, wo, C, dy, daux)
    slot = routing0["slot"]
    if seed == 0:                                   # the mix of cases the derivative must handle
        assert (slot[..., 0] == -1).any() and (slot[..., 1] == -2).any() and (slot[..., 1] == -1).any()
        assert ((slot[..., 0] < 0) & (slot[..., 1] >= 0)).any()
    dwi = np.stack([got["dwi"][e] for e in range(E)])
    dwo = np.stack([got["dwo"][e] for e in range(E)])
    eps = 1e-6
    checked = tried = 0
    for name, arr, grad in (("x", x, got["dx"]), ("wg", wg, got["dwg"]), ("wi", wi, dwi), ("wo", wo, dwo)):
        flat = arr.reshape(-1)
        picks = rng.choice(flat.size, size=min(flat.size, 40), replace=False)
        for i in picks:
            tried += 1
            keep = flat[i]
            flat[i] = keep + eps
            lp, rp = _loss(x, wg, u, wi, wo, C, dy, daux)
            flat[i] = keep - eps
            lm, rm = _loss(x, wg, u, wi, wo, C, dy, daux)
            flat[i] = keep
            if not (_same_routing(rp, routing0) and _same_routing(rm, routing0)):
                continue                            # a discrete decision flipped: no derivative there
            num = (lp - lm) / (2 * eps)
            assert abs(num - grad.reshape(-1)[i]) <= 1e-6 * (1.0 + abs(num)), (name, i, num, grad.reshape(-1)[i])
            checked += 1
    assert checked > 0.8 * tried and checked >= 60


def _torch_dense_layer(x, wg, wi, wo, routing, C):
    """Algorithm 2 with dense [G,S,E,C] tensors in torch float64; the discrete routing
    (indices, slots) enters as constants, the weights are recomputed from the gates."""
    G, S, M = x.shape
    E = wg.shape[1]
    gates = torch.softmax(torch.einsum("gsm,me->gse", x, wg), dim=-1)
    idx = torch.as_tensor(routing["expert_idx"])
    top = torch.gather(gates, 2, idx)                               # [G,S,2] raw top-2 gates
    norm = top / top.sum(dim=-1, keepdim=True)
    kept = torch.as_tensor(routing["slot"] >= 0)
    onehot_e = torch.nn.functional.one_hot(idx, E).to(torch.float64)                  # [G,S,2,E]
    pos = torch.as_tensor(np.maximum(routing["slot"], 0))
    onehot_c = torch.nn.functional.one_hot(pos, C).to(torch.float64)                  # [G,S,2,C]
    mask = torch.einsum("gske,gskc->gskec", onehot_e, onehot_c) * kept[..., None, None]
    combine_weights = (mask * norm[..., None, None]).sum(dim=2)                       # [G,S,E,C]
    dispatch_mask = mask.sum(dim=2)
    dispatched = torch.einsum("gsec,gsm->egcm", dispatch_mask, x)
    h = torch.relu(torch.einsum("egcm,emh->egch", dispatched, wi))
    expert_outputs = torch.einsum("egch,ehm->egcm", h, wo)
    y = torch.einsum("gsec,egcm->gsm", combine_weights, expert_outputs)
    c1 = torch.as_tensor(routing["c1"]).to(torch.float64)
    aux = ((c1 / S) * gates.mean(dim=1)).sum(dim=-1) / E
    return y, aux


@pytest.mark.parametrize("G,S,M,H,E,C,seed", [(2, 24, 8, 12, 6, 5, 0), (1, 40, 6, 9, 4, 16, 1), (3, 10, 7, 5, 2, 10, 2),
                                               (2, 30, 5, 8, 9, 3, 3)])
def test_against_autograd_on_the_dense_einsums(G, S, M, H, E, C, seed):
    rng = np.random.default_rng(200 + seed)
    x, wg, u, wi, wo, dy, daux = _rand_layer(rng, G, S, M, H, E)
    got = bwd.moe_backward(x, wg, u, wi, wo, C, dy, daux)
    tx, twg, twi, two = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, wg, wi, wo))
    y, aux = _torch_dense_layer(tx, twg, twi, two, got["routing"], C)
    np.testing.assert_allclose(y.detach().numpy(), got["y"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(aux.detach().numpy(), got["routing"]["aux"], rtol=1e-12)
    loss = (torch.as_tensor(dy) * y).sum() + (torch.as_tensor(daux) * aux).sum()
    loss.backward()
    np.testing.assert_allclose(got["dx"], tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(got["dwg"], twg.grad.numpy(), rtol=1e-10, atol=1e-12)
    for e in range(E):
        np.testing.assert_allclose(got["dwi"][e], twi.grad[e].numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(got["dwo"][e], two.grad[e].numpy(), rtol=1e-10, atol=1e-12)


def test_two_experts_all_kept_is_the_dense_mixture_gradient():
    """E=2, C>=S, u=0: y_s = sum_e softmax(x_s wg)_e FFN_e(x_s), a plain differentiable
    function with no routing at all; its autograd gradient is the layer's."""
    rng = np.random.default_rng(7)
    G, S, M, H, E = 2, 9, 6, 10, 2
    x, wg, u, wi, wo, dy, _ = _rand_layer(rng, G, S, M, H, E)
    u[:] = 0.0
    got = bwd.moe_backward(x, wg, u, wi, wo, S, dy, np.zeros(G))
    assert (got["routing"]["slot"] >= 0).all()
    tx, twg, twi, two = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, wg, wi, wo))
    p = torch.softmax(tx @ twg, dim=-1)
    ffn = torch.stack([torch.relu(tx @ twi[e]) @ two[e] for e in range(E)], dim=-1)   # [G,S,M,E]
    ((ffn * p[:, :, None, :]).sum(-1) * torch.as_tensor(dy)).sum().backward()
    np.testing.assert_allclose(got["dx"], tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(got["dwg"], twg.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(np.stack([got["dwi"][e] for e in range(E)]), twi.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(np.stack([got["dwo"][e] for e in range(E)]), two.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_auxiliary_loss_gradient_alone():
    """dy = 0: only l_aux = (1/E) sum_e (c_e/S) m_e is differentiated, the counts being
    constants (Section 2.2).  d l_aux/d logits has the closed form of a softmax-weighted
    mean: dz[s,e] = g[s,e] (a_e - sum_e' g[s,e'] a_e') with a_e = c_e/(E S^2)."""
    rng = np.random.default_rng(8)
    G, S, M, H, E, C = 2, 16, 5, 6, 4, 6
    x, wg, u, wi, wo, _, daux = _rand_layer(rng, G, S, M, H, E)
    got = bwd.moe_backward(x, wg, u, wi, wo, C, np.zeros((G, S, M)), daux)
    r = got["routing"]
    for e in range(E):
        assert not got["dwi"][e].any() and not got["dwo"][e].any()
    assert not got["dout"].any() and not got["dweight"].any()
    want_dwg = np.zeros((M, E))
    want_dx = np.zeros((G, S, M))
    for g in range(G):
        a = daux[g] * r["c1"][g] / (E * S * S)
        for s in range(S):
            p = r["gates"][g, s]
            dz = p * (a - (p * a).sum())
            want_dwg += np.outer(x[g, s], dz)
            want_dx[g, s] = wg @ dz
    np.testing.assert_allclose(got["dwg"], want_dwg, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(got["dx"], want_dx, rtol=1e-12, atol=1e-15)
    # the gradient of a softmax output sums to zero over the logits of a token
    np.testing.assert_allclose(got["dlogits"].sum(-1), 0.0, atol=1e-15)


def test_structure_of_the_gradients():
    rng = np.random.default_rng(9)
    G, S, M, H, E, C = 2, 30, 6, 8, 5, 4
    x, wg, u, wi, wo, dy, daux = _rand_layer(rng, G, S, M, H, E)
    got = bwd.moe_backward(x, wg, u, wi, wo, C, dy, daux)
    r = got["routing"]
    # empty slots carry no gradient; occupied ones carry weight * dy of their token
    occupied = r["src_token"] >= 0
    assert not got["dout"][~occupied].any() and not got["dbuf"][~occupied].any()
    e, g, c = [a[0] for a in np.nonzero(occupied)]
    s = r["src_token"][e, g, c]
    k = 0 if r["expert_idx"][g, s, 0] == e else 1
    np.testing.assert_allclose(got["dout"][e, g, c], r["weight"][g, s, k] * dy[g, s], rtol=1e-15)
    # a fully dropped token receives gradient only through the gate (its experts never saw it)
    dropped = (r["slot"] < 0).all(-1)
    assert dropped.any()
    np.testing.assert_allclose(got["dx"][dropped], np.einsum("ne,me->nm", got["dlogits"][dropped], wg), rtol=1e-13)
    # the layer is linear in (dy, daux): gradients scale with them
    twice = bwd.moe_backward(x, wg, u, wi, wo, C, 2 * dy, 2 * daux)
    np.testing.assert_allclose(twice["dx"], 2 * got["dx"], rtol=1e-13)
    np.testing.assert_allclose(twice["dwg"], 2 * got["dwg"], rtol=1e-13)
    # weight gradients on request only
    some = bwd.moe_backward(x, wg, u, wi, wo, C, dy, daux, experts=[3])
    assert list(some["dwi"]) == [3]
    np.testing.assert_array_equal(some["dwi"][3], got["dwi"][3])
    np.testing.assert_array_equal(some["dx"], got["dx"])
