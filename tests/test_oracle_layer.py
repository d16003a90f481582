"""Pins for the oracle's layer output (Eq. 1-3, Algorithm 2).  CPU only."""
import itertools

import numpy as np
import pytest
import scipy.special

from oracle import moe_oracle as orc


def _rand_layer(rng, G, S, M, H, E):
    x = rng.normal(size=(G, S, M))
    wg = rng.normal(size=(M, E)) / np.sqrt(M)
    wi = rng.normal(size=(E, M, H)) / np.sqrt(M)
    wo = rng.normal(size=(E, H, M)) / np.sqrt(H)
    u = rng.random((G, S))
    return x, wg, u, wi, wo


def test_expert_ffn_against_explicit_loops():
    """Eq. 2 with every index written out: catches a transposed operand."""
    rng = np.random.default_rng(0)
    R, M, H = 3, 4, 5
    rows = rng.normal(size=(R, M))
    wi = rng.normal(size=(M, H))
    wo = rng.normal(size=(H, M))
    want = np.zeros((R, M))
    for r in range(R):
        hid = [max(0.0, sum(rows[r, m] * wi[m, h] for m in range(M))) for h in range(H)]
        for m in range(M):
            want[r, m] = sum(hid[h] * wo[h, m] for h in range(H))
    np.testing.assert_allclose(orc.expert_ffn(rows, wi, wo), want, rtol=1e-13, atol=1e-14)
    assert (orc.expert_ffn(np.zeros((2, M)), wi, wo) == 0).all()      # FFN_e(0) = 0
    # the inner half on its own: index loops again, negative pre-activations clipped to 0
    hid = np.array([[max(0.0, sum(rows[r, m] * wi[m, h] for m in range(M))) for h in range(H)]
                    for r in range(R)])
    np.testing.assert_allclose(orc.expert_hidden(rows, wi), hid, rtol=1e-13, atol=1e-14)
    assert (hid == 0).any() and (hid > 0).any()


def test_two_experts_is_the_dense_mixture():
    """E=2, C>=S, u=0: both experts always kept and g1+g2=1, so
    y_s = sum_e softmax(x_s wg)_e FFN_e(x_s): Eq. 3 with the raw gates."""
    rng = np.random.default_rng(1)
    G, S, M, H, E = 2, 9, 6, 10, 2
    x, wg, _, wi, wo = _rand_layer(rng, G, S, M, H, E)
    y, r, _, _ = orc.moe_forward(x, wg, np.zeros((G, S)), wi, wo, C=S)
    gates = scipy.special.softmax(x @ wg, axis=-1)
    want = sum(gates[..., e:e + 1] * (np.maximum(x @ wi[e], 0) @ wo[e]) for e in range(E))
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-13)


def test_identical_experts_make_routing_irrelevant():
    """All experts equal, nothing dropped: weights sum to 1 so y_s = FFN(x_s)."""
    rng = np.random.default_rng(2)
    G, S, M, H, E = 2, 20, 5, 7, 6
    x, wg, _, wi, wo = _rand_layer(rng, G, S, M, H, E)
    wi[:] = wi[0]
    wo[:] = wo[0]
    y, r, _, _ = orc.moe_forward(x, wg, np.zeros((G, S)), wi, wo, C=S)
    np.testing.assert_allclose(y, np.maximum(x @ wi[0], 0) @ wo[0], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("seed", range(6))
def test_definition_equals_dense_formulation(seed):
    """Eq. 1-3 evaluated per expert == Algorithm 2's sums over the dense
    [G,S,E,C] tensors == a per-token sum over the group combine weights G_{S,E}."""
    rng = np.random.default_rng(20 + seed)
    G, S, M, H, E = int(rng.integers(1, 4)), int(rng.integers(2, 20)), 5, 6, int(rng.integers(2, 6))
    C = int(rng.integers(1, 2 * S // E + 3))
    x, wg, u, wi, wo = _rand_layer(rng, G, S, M, H, E)
    y, r, buf, out = orc.moe_forward(x, wg, u, wi, wo, C)
    y2, r2, buf2, out2 = orc.moe_forward_dense(x, wg, u, wi, wo, C)
    np.testing.assert_allclose(y, y2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(buf, buf2, rtol=0, atol=0)
    np.testing.assert_allclose(out, out2, rtol=1e-12, atol=1e-13)
    # Eq. 3 straight from G_{S,E}: no slots, no buffers
    y3 = np.zeros_like(y)
    for g, s, e in itertools.product(range(G), range(S), range(E)):
        if r["combine"][g, s, e] != 0:
            y3[g, s] += r["combine"][g, s, e] * (np.maximum(x[g, s] @ wi[e], 0) @ wo[e])
    np.testing.assert_allclose(y, y3, rtol=1e-12, atol=1e-13)
    # the dense tensors have the support Section 3.1 describes
    cw, dm = orc.dense_combine_weights(r, E, C)
    assert ((cw != 0).sum(axis=(2, 3)) <= 2).all()
    assert (dm.sum(axis=1) <= 1).all()                    # one token per (g,e,c)
    assert (dm.sum(axis=(1, 3)) <= C).all()
    np.testing.assert_allclose(cw.sum(axis=3), r["combine"], rtol=1e-15)
    # selected-token evaluation agrees with the full one
    toks = [(g, s) for g in range(G) for s in range(0, S, 3)]
    yt = orc.moe_forward_tokens(x, r, wi, wo, toks)
    np.testing.assert_allclose(yt, np.stack([y[g, s] for g, s in toks]), rtol=1e-12, atol=1e-13)


def test_fully_dropped_token_outputs_zero():
    """Section 2.2: a token whose two experts are both full gets a zero vector."""
    rng = np.random.default_rng(5)
    G, S, M, H, E = 1, 12, 4, 6, 3
    x, _, _, wi, wo = _rand_layer(rng, G, S, M, H, E)
    y, r, _, _ = orc.moe_forward(x, np.zeros((M, E)), np.zeros((G, S)), wi, wo, C=2)
    assert (r["slot"][0, 2:] == -1).all()
    assert (y[0, 2:] == 0).all()
    assert (y[0, :2] != 0).any()
