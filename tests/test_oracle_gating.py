"""Pins for the oracle's gating (Algorithm 1).  CPU only.

Each test checks the oracle against something that is not the oracle: a
hand-worked example, a closed form, brute-force counting or a library routine.
"""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

from oracle import moe_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


def _frac(p):
    return float(Fraction(p[0]) / Fraction(p[1])) if not isinstance(p[0], float) \
        else p[0] / p[1]


# ---------------------------------------------------------------- hand example
def test_hand_example_default_reading():
    ex = json.load(open(GOLDEN))
    gates = np.array(ex["gates"])[None]
    u = np.array(ex["u"])[None]
    r = orc.top2_gating(gates, u, ex["C"])
    assert r["expert_idx"][0].tolist() == ex["expert_idx"]
    assert r["slot"][0].tolist() == ex["slot"]
    want_w = np.array([[_frac(a), _frac(b)] for a, b in ex["weight_fractions"]])
    np.testing.assert_allclose(r["weight"][0], want_w, rtol=1e-15, atol=0)
    assert r["c1"][0].tolist() == ex["c1"]
    np.testing.assert_allclose(r["mean_gate"][0], ex["mean_gate"], rtol=1e-15)
    np.testing.assert_allclose(r["aux"][0], _frac(ex["aux_fraction"]), rtol=1e-14)
    assert r["fill"][0].tolist() == ex["fill"]
    assert r["src_token"][:, 0, :].tolist() == ex["src_token"]
    sums = r["weight"][0].sum(axis=1)
    np.testing.assert_allclose(sums, [_frac(p) for p in ex["weight_sums_fractions"]],
                               rtol=1e-15)
    # group combine weights G_{S,E}: the same weights placed at the expert index
    comb = np.zeros((ex["S"], ex["E"]))
    for s in range(ex["S"]):
        for k in range(2):
            comb[s, ex["expert_idx"][s][k]] += want_w[s, k]
    np.testing.assert_allclose(r["combine"][0], comb, rtol=1e-15)


def test_hand_example_typeset_reading_differs_only_where_expected():
    ex = json.load(open(GOLDEN))
    gates = np.array(ex["gates"])[None]
    u = np.array(ex["u"])[None]
    r = orc.top2_gating(gates, u, ex["C"], literal_pass2=True)
    assert r["slot"][0].tolist() == ex["slot_literal_pass2"]
    assert r["c1"][0].tolist() == ex["c1"]


# ---------------------------------------------------------------- softmax / logits
def test_softmax_against_scipy_and_loops():
    rng = np.random.default_rng(1)
    G, S, M, E = 2, 5, 7, 6
    x = rng.normal(size=(G, S, M))
    wg = rng.normal(size=(M, E))
    z = np.zeros((G, S, E))
    for g, s, e, m in itertools.product(range(G), range(S), range(E), range(M)):
        z[g, s, e] += x[g, s, m] * wg[m, e]
    np.testing.assert_allclose(orc.gate_logits(x, wg), z, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(orc.softmax_gates(x, wg), scipy.special.softmax(z, axis=-1),
                               rtol=1e-13)
    # shift invariance with huge logits: no overflow
    big = orc.softmax_gates(x * 1e3, wg)
    assert np.isfinite(big).all()
    np.testing.assert_allclose(big.sum(-1), 1.0, rtol=1e-13)


def test_top_2_first_index_wins_ties():
    assert orc.top_2([0.25, 0.25, 0.25, 0.25]) == (0.25, 0, 0.25, 1)
    assert orc.top_2([0.1, 0.4, 0.4, 0.1]) == (0.4, 1, 0.4, 2)
    assert orc.top_2([0.1, 0.2, 0.7])[1::2] == (2, 1)


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("E,S,C", [(4, 16, 8), (8, 64, 16), (3, 5, 2)])
def test_zero_gate_weights_closed_form(E, S, C):
    """wg = 0: all gates 1/E, every token picks experts (0,1); expert 0 keeps the
    first C tokens in order; m_e = 1/E, c = [S,0,...] so l_aux = 1/E^2."""
    M = 6
    rng = np.random.default_rng(0)
    x = rng.normal(size=(1, S, M))
    gates = orc.softmax_gates(x, np.zeros((M, E)))
    np.testing.assert_allclose(gates, 1.0 / E, rtol=1e-15)
    r = orc.top2_gating(gates, np.zeros((1, S)), C)        # u=0: always sampled
    assert (r["expert_idx"][0] == [0, 1]).all()
    assert r["slot"][0, :, 0].tolist() == [s if s < C else -1 for s in range(S)]
    assert r["slot"][0, :, 1].tolist() == [s if s < C else -1 for s in range(S)]
    np.testing.assert_allclose(r["weight"][0, :C], 0.5, rtol=1e-15)
    assert (r["weight"][0, C:] == 0).all()
    assert r["c1"][0].tolist() == [S] + [0] * (E - 1)
    np.testing.assert_allclose(r["aux"][0], 1.0 / E ** 2, rtol=1e-14)


def test_balanced_top1_closed_form():
    """Perfectly balanced first choices and uniform mean gates: l_aux = 1/E^2."""
    E, S = 4, 16
    gates = np.full((S, E), 0.2)
    for s in range(S):                 # winner rotates, runner-up is the next expert
        gates[s, s % E] = 0.3
        gates[s, (s + 1) % E] = 0.3 - 1e-9
    gates /= gates.sum(axis=1, keepdims=True)
    r = orc.top2_gating(gates[None], np.zeros((1, S)), C=S)
    assert r["c1"][0].tolist() == [S // E] * E
    np.testing.assert_allclose(r["aux"][0], 1.0 / E ** 2, rtol=1e-9)


def test_u_near_one_is_top1_routing():
    rng = np.random.default_rng(3)
    gates = scipy.special.softmax(rng.normal(size=(2, 32, 5)), axis=-1)
    r = orc.top2_gating(gates, np.full((2, 32), 0.999999), C=32)
    assert (r["slot"][:, :, 1] == orc.SLOT_NOT_SAMPLED).all()
    assert (r["weight"][:, :, 1] == 0).all()
    assert (r["slot"][:, :, 0] >= 0).all()
    srt = np.sort(gates, axis=-1)
    np.testing.assert_allclose(r["weight"][:, :, 0], srt[..., -1] / (srt[..., -1] + srt[..., -2]),
                               rtol=1e-14)


def test_aux_sums():
    """sum_e c1_e = S and sum_e m_e = 1; E * aux = sum_e (c1_e/S) m_e."""
    rng = np.random.default_rng(4)
    G, S, E = 3, 40, 7
    gates = scipy.special.softmax(rng.normal(size=(G, S, E)) * 2, axis=-1)
    r = orc.top2_gating(gates, rng.random((G, S)), C=9)
    assert (r["c1"].sum(axis=1) == S).all()
    np.testing.assert_allclose(r["mean_gate"].sum(axis=1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(r["aux"] * E, ((r["c1"] / S) * gates.mean(axis=1)).sum(axis=1),
                               rtol=1e-13)


# ---------------------------------------------------------------- brute force
def _brute_force_group(gates, u, C):
    """Positions by direct counting over all earlier tokens (no running state)."""
    S, E = gates.shape
    e1 = np.zeros(S, int)
    e2 = np.zeros(S, int)
    for s in range(S):
        best = sorted(range(E), key=lambda e: (-gates[s, e], e))
        e1[s], e2[s] = best[0], best[1]
    g1 = gates[np.arange(S), e1]
    g2 = gates[np.arange(S), e2]
    sampled = [2 * g2[s] / (g1[s] + g2[s]) > u[s] for s in range(S)]
    slot = np.zeros((S, 2), int)
    weight = np.zeros((S, 2))
    for s in range(S):
        p1 = sum(1 for t in range(s) if e1[t] == e1[s])
        slot[s, 0] = p1 if p1 < C else -1
        n_first = sum(1 for t in range(S) if e1[t] == e2[s])
        p2 = n_first + sum(1 for t in range(s) if sampled[t] and e2[t] == e2[s])
        slot[s, 1] = -2 if not sampled[s] else (p2 if p2 < C else -1)
        if slot[s, 0] >= 0:
            weight[s, 0] = g1[s] / (g1[s] + g2[s])
        if slot[s, 1] >= 0:
            weight[s, 1] = g2[s] / (g1[s] + g2[s])
    return np.stack([e1, e2], 1), slot, weight


def test_exhaustive_rank_patterns_tiny():
    """Every assignment of (first, second) expert to S<=4 tokens, E=3, C in {1,2},
    with every sampled/not-sampled pattern: sequential == counting == cumsum form."""
    E = 3
    pairs = [(a, b) for a in range(E) for b in range(E) if a != b]
    n = 0
    for S in (1, 2, 3, 4):
        for C in (1, 2):
            for choice in itertools.product(pairs, repeat=S):
                gates = np.full((S, E), 0.1)
                for s, (a, b) in enumerate(choice):
                    gates[s, a], gates[s, b] = 0.6, 0.3
                for keep in itertools.product((0.0, 0.9), repeat=S):   # 2*g2n = 2/3
                    u = np.array(keep)
                    r = orc.top2_gating(gates[None], u[None], C)
                    bi, bs, bw = _brute_force_group(gates, u, C)
                    assert (r["expert_idx"][0] == bi).all()
                    assert (r["slot"][0] == bs).all(), (choice, keep, C)
                    np.testing.assert_allclose(r["weight"][0], bw, rtol=1e-15)
                    ci, cs, cw, cc1, caux = orc.top2_gating_cumsum(gates, u, C)
                    assert (ci == bi).all() and (cs == bs).all()
                    np.testing.assert_allclose(cw, bw, rtol=1e-15)
                    assert (cc1 == r["c1"][0]).all()
                    np.testing.assert_allclose(caux, r["aux"][0], rtol=1e-14)
                    n += 1
    assert n > 20000


@pytest.mark.parametrize("seed", range(8))
def test_random_cases_three_forms_and_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    G = int(rng.integers(1, 4))
    S = int(rng.integers(1, 70))
    E = int(rng.integers(2, 9))
    C = int(rng.integers(1, max(2, 2 * S // E + 2)))
    gates = scipy.special.softmax(rng.normal(size=(G, S, E)) * 1.5, axis=-1)
    u = rng.random((G, S))
    r = orc.top2_gating(gates, u, C)
    for g in range(G):
        bi, bs, bw = _brute_force_group(gates[g], u[g], C)
        assert (r["expert_idx"][g] == bi).all()
        assert (r["slot"][g] == bs).all()
        np.testing.assert_allclose(r["weight"][g], bw, rtol=1e-14)
        ci, cs, cw, cc1, caux = orc.top2_gating_cumsum(gates[g], u[g], C)
        assert (ci == bi).all() and (cs == bs).all() and (cc1 == r["c1"][g]).all()
        np.testing.assert_allclose(caux, r["aux"][g], rtol=1e-13)
    check_routing_invariants(r, S, E, C)


def check_routing_invariants(r, S, E, C):
    """Structural facts Section 2.2 / 3.1 state about any routing."""
    G = r["slot"].shape[0]
    idx, slot, w, fill, src = (r[k] for k in ("expert_idx", "slot", "weight", "fill", "src_token"))
    assert (idx[..., 0] != idx[..., 1]).all()
    assert (fill <= C).all() and (fill >= 0).all()
    assert (w >= 0).all()
    assert (w[slot < 0] == 0).all()
    assert (w.sum(-1) <= 1 + 1e-12).all()
    for g in range(G):
        for e in range(E):
            first = [(s, slot[g, s, 0]) for s in range(S) if idx[g, s, 0] == e and slot[g, s, 0] >= 0]
            second = [(s, slot[g, s, 1]) for s in range(S) if idx[g, s, 1] == e and slot[g, s, 1] >= 0]
            pos = [p for _, p in first] + [p for _, p in second]
            assert sorted(pos) == list(range(fill[g, e]))          # 0..fill-1, no holes
            assert [p for _, p in first] == sorted(p for _, p in first)   # token order
            assert [p for _, p in second] == sorted(p for _, p in second)
            if first and second:
                assert min(p for _, p in second) > max(p for _, p in first)
            for s, p in first + second:
                assert src[e, g, p] == s
            assert (src[e, g, fill[g, e]:] == -1).all()


def test_groups_are_independent_and_prefix_stable():
    rng = np.random.default_rng(7)
    G, S, E, C = 3, 24, 5, 6
    gates = scipy.special.softmax(rng.normal(size=(G, S, E)), axis=-1)
    u = rng.random((G, S))
    r = orc.top2_gating(gates, u, C)
    perm = [2, 0, 1]
    rp = orc.top2_gating(gates[perm], u[perm], C)
    for k in ("expert_idx", "slot", "weight", "c1", "aux", "fill"):
        np.testing.assert_array_equal(rp[k], r[k][perm])
    # appending tokens never changes the first-choice slots of earlier tokens
    rs = orc.top2_gating(gates[:, :15], u[:, :15], C)
    np.testing.assert_array_equal(rs["slot"][:, :, 0], r["slot"][:, :15, 0])


def test_capacity_one_and_huge_capacity():
    rng = np.random.default_rng(9)
    gates = scipy.special.softmax(rng.normal(size=(1, 30, 4)), axis=-1)
    u = np.zeros((1, 30))
    r1 = orc.top2_gating(gates, u, 1)
    assert (r1["fill"] <= 1).all() and r1["fill"].sum() <= 4
    rb = orc.top2_gating(gates, u, 1000)
    assert (rb["slot"] >= 0).all()
    np.testing.assert_allclose(rb["weight"].sum(-1), 1.0, rtol=1e-14)
