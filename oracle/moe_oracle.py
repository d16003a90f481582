"""fp64 CPU oracle for the position-wise top-2 Mixture-of-Experts layer (GShard).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the test-suite, the
smoke check and the CPU-baseline leg of the benchmark may call it.  It shares no
code with the HIP library and imports nothing from it.

Everything is plain numpy in float64, written to be checked against the paper
by eye:

* ``softmax_gates``            -- Algorithm 1, the line  g_{S,E} = softmax(wg . x_S)
                                   (= line 1 of Algorithm 2)
* ``top_2``                    -- Algorithm 1, the ``top_2`` call
* ``top2_gating_group``        -- Algorithm 1, literally: two sequential passes over
                                   the tokens of one group with the running
                                   counters c_E
* ``top2_gating``              -- Section 2.2 "Local group dispatching": the same for
                                   G independent groups
* ``top2_gating_cumsum``       -- the same function restated with one-hot masks and
                                   cumulative sums (Section 3.1 / Section 5.2 name
                                   Cumsum and ArgMax as the building blocks); used
                                   only to cross-check the sequential form
* ``dense_combine_weights``    -- Section 3.1: the [G,S,E,C] combine_weights tensor
                                   and the binary dispatch_mask
* ``moe_forward_dense``        -- Algorithm 2 / Section 3.1: the layer as sums over the dense
                                   [G,S,E,C] tensors (tiny inputs)
* ``expert_hidden``            -- Eq. 2, inner half:  ReLU(wi_e . x)
* ``expert_ffn``               -- Eq. 2:  FFN_e(x) = wo_e . ReLU(wi_e . x)
* ``moe_forward``              -- Eq. 1-3:  y_s = sum_e G_{s,e} FFN_e(x_s)
* ``moe_forward_tokens``       -- Eq. 1-3 for a chosen subset of tokens

Readings of the paper taken where it is silent or ambiguous:

R1  Pass 2 of Algorithm 1 typesets the counter increment outside the ``if``; the
    text of Section 2.2 ("Random routing") says the second expert is skipped to
    conserve capacity.  Default reading: a second choice rejected by the random
    draw does NOT advance c_{e2}.  ``literal_pass2=True`` gives the typeset reading.
R2  l_aux = (1/E) sum_e (c_e/S) m_e  with c_e the first-choice counters as they
    stand after pass 1 (incremented for every token, also overflowing ones).
R3  top_2 ties: the lowest expert index wins.
R4  Both renormalisations divide by the sum of the two RAW top-2 gates.
R5  A token is "dispatched" to a slot by slot validity, not by its weight being
    non-zero (a gate that underflows to 0 still occupies its slot).
R6  Weights are not renormalised again when one of the two choices is dropped.
R7  Expert outputs stay in [E,G,C,M] order on one device (Algorithm 2 prints
    GECM, which is the layout after the reverse exchange between devices).

Slot codes (shared vocabulary with the C ABI): ``slot >= 0`` position in the
expert buffer, ``-1`` dropped because the expert was full, ``-2`` second choice
not sampled by random routing (takes precedence over ``-1``).

Parity pins: every function here is pinned by tests/test_oracle_*.py (hand-worked
example, closed forms, dense-mixture special cases, brute-force counting on tiny
inputs, library softmax / matmul); nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

SLOT_OVERFLOW = -1
SLOT_NOT_SAMPLED = -2


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------
# Algorithm 1, line "g_{S,E} <- softmax(wg . x_S)"
# --------------------------------------------------------------------------
def gate_logits(x, wg):
    """z[g,s,e] = sum_m x[g,s,m] * wg[m,e]   (Algorithm 2, line 1: GSM,ME->GSE)."""
    x = _f64(x)
    wg = _f64(wg)
    G, S, M = x.shape
    return (x.reshape(G * S, M) @ wg).reshape(G, S, wg.shape[1])


def softmax_gates(x, wg):
    """g[g,s,:] = softmax over experts of the gate logits (Algorithm 1)."""
    z = gate_logits(x, wg)
    z = z - z.max(axis=-1, keepdims=True)
    p = np.exp(z)
    return p / p.sum(axis=-1, keepdims=True)


# --------------------------------------------------------------------------
# Algorithm 1: top_2 and the two sequential passes
# --------------------------------------------------------------------------
def top_2(gates_row):
    """(g1, e1, g2, e2): largest and second largest gate of one token (R3)."""
    row = _f64(gates_row)
    e1 = int(np.argmax(row))                 # first maximum
    rest = row.copy()
    rest[e1] = -np.inf
    e2 = int(np.argmax(rest))                # first maximum among the others
    return float(row[e1]), e1, float(row[e2]), e2


def top2_gating_group(gates, u, C, literal_pass2=False):
    """Algorithm 1 for ONE group.

    gates [S,E] softmax gates, u [S] the uniforms ``rnd`` of pass 2 (inputs, so
    that results are reproducible), C the group's expert capacity.

    Returns a dict with
      combine [S,E]  the group combine weights  G_{S,E}
      expert_idx [S,2], slot [S,2], weight [S,2]  the same information per choice
      c1 [E]         counters after pass 1,   mean_gate [E]  m_E,   aux  l_aux
      counters [E]   counters after pass 2
    """
    gates = _f64(gates)
    u = _f64(u)
    S, E = gates.shape
    # every token's two largest gates and their normalised values (the same in both passes: R4)
    picks = [top_2(gates[s]) for s in range(S)]
    first = [(e1, g1 / (g1 + g2)) for (g1, e1, g2, e2) in picks]
    second = [(e2, g2 / (g1 + g2)) for (g1, e1, g2, e2) in picks]

    c = np.zeros(E, dtype=np.int64)                       # running count of tokens sent to each expert
    m = gates.sum(axis=0) / S                             # mean gate per expert
    combine = np.zeros((S, E))
    expert_idx = np.zeros((S, 2), dtype=np.int64)
    slot = np.full((S, 2), SLOT_OVERFLOW, dtype=np.int64)
    weight = np.zeros((S, 2))

    # pass 1: first choices in token order; an expert that is full turns the token away but
    # still counts it
    for s, (e1, g1n) in enumerate(first):
        pos = c[e1]
        expert_idx[s, 0] = e1
        if pos < C:
            combine[s, e1] = g1n
            slot[s, 0] = pos
            weight[s, 0] = g1n
        c[e1] = pos + 1

    c1 = c.copy()
    aux = float(np.sum((c / S) * m) / E)                  # l_aux from the counts as they stand now (R2)

    # pass 2: second choices queue behind all first choices; a token takes part with
    # probability proportional to its second gate (2 g2n > uniform)
    for s, (e2, g2n) in enumerate(second):
        pos = c[e2]
        sampled = (2.0 * g2n > u[s])
        expert_idx[s, 1] = e2
        if pos < C and sampled:
            combine[s, e2] = g2n
            slot[s, 1] = pos
            weight[s, 1] = g2n
        elif not sampled:
            slot[s, 1] = SLOT_NOT_SAMPLED
        if sampled or literal_pass2:                      # R1: a token that is not sampled takes no place
            c[e2] = pos + 1

    return dict(combine=combine, expert_idx=expert_idx, slot=slot, weight=weight,
                c1=c1, mean_gate=m, aux=aux, counters=c)


def top2_gating(gates, u, C, literal_pass2=False):
    """Algorithm 1 for G independent groups (Section 2.2, local group dispatching).

    gates [G,S,E], u [G,S].  Returns arrays stacked over groups plus
      fill [G,E]        number of occupied slots of expert e in group g
      src_token [E,G,C] inverse map slot -> token index s in the group (-1 empty);
                        the index form of the gather-based dispatch of Section 3.2
    """
    gates = _f64(gates)
    u = _f64(u)
    G, S, E = gates.shape
    per = [top2_gating_group(gates[g], u[g], C, literal_pass2) for g in range(G)]
    out = {k: np.stack([p[k] for p in per]) for k in
           ("combine", "expert_idx", "slot", "weight", "c1", "mean_gate", "counters")}
    out["aux"] = np.array([p["aux"] for p in per])
    fill = np.zeros((G, E), dtype=np.int64)
    src = np.full((E, G, C), -1, dtype=np.int64)
    for g in range(G):
        for s in range(S):
            for k in range(2):
                pos = out["slot"][g, s, k]
                if pos >= 0:
                    e = out["expert_idx"][g, s, k]
                    assert src[e, g, pos] == -1, "two tokens in one slot"
                    src[e, g, pos] = s
                    fill[g, e] += 1
    out["fill"] = fill
    out["src_token"] = src
    return out


# --------------------------------------------------------------------------
# The same gating restated with one-hot masks and cumulative sums
# --------------------------------------------------------------------------
def top2_gating_cumsum(gates, u, C):
    """One group, default reading R1, no loop over tokens.

    position of a token in its expert = exclusive cumulative sum over S of the
    one-hot choice mask; second choices start after all first choices.
    Returns (expert_idx [S,2], slot [S,2], weight [S,2], c1 [E], aux).
    """
    gates = _f64(gates)
    u = _f64(u)
    S, E = gates.shape
    order = np.argsort(-gates, axis=1, kind="stable")     # stable: low index first
    e1, e2 = order[:, 0], order[:, 1]
    rows = np.arange(S)
    g1, g2 = gates[rows, e1], gates[rows, e2]
    g1n, g2n = g1 / (g1 + g2), g2 / (g1 + g2)

    mask1 = np.zeros((S, E), dtype=np.int64)
    mask1[rows, e1] = 1
    pos1 = (np.cumsum(mask1, axis=0) - mask1)[rows, e1]
    c1 = mask1.sum(axis=0)
    aux = float(np.mean((c1 / S) * gates.mean(axis=0)))

    sampled = 2.0 * g2n > u
    mask2 = np.zeros((S, E), dtype=np.int64)
    mask2[rows, e2] = sampled.astype(np.int64)
    pos2 = (np.cumsum(mask2, axis=0) - mask2 + c1[None, :])[rows, e2]

    slot = np.empty((S, 2), dtype=np.int64)
    slot[:, 0] = np.where(pos1 < C, pos1, SLOT_OVERFLOW)
    slot[:, 1] = np.where(~sampled, SLOT_NOT_SAMPLED,
                          np.where(pos2 < C, pos2, SLOT_OVERFLOW))
    weight = np.stack([np.where(slot[:, 0] >= 0, g1n, 0.0),
                       np.where(slot[:, 1] >= 0, g2n, 0.0)], axis=1)
    return np.stack([e1, e2], axis=1), slot, weight, c1, aux


# --------------------------------------------------------------------------
# Section 3.1: dense combine_weights / dispatch_mask and Algorithm 2
# --------------------------------------------------------------------------
def dense_combine_weights(routing, E, C):
    """combine_weights[G,S,E,C] and dispatch_mask[G,S,E,C] from a routing dict."""
    G, S, _ = routing["slot"].shape
    cw = np.zeros((G, S, E, C))
    dm = np.zeros((G, S, E, C))
    for g in range(G):
        for s in range(S):
            for k in range(2):
                pos = routing["slot"][g, s, k]
                if pos >= 0:
                    e = routing["expert_idx"][g, s, k]
                    cw[g, s, e, pos] = routing["weight"][g, s, k]
                    dm[g, s, e, pos] = 1.0                 # reading R5
    return cw, dm


def moe_forward_dense(x, wg, u, wi, wo, C, literal_pass2=False):
    """The layer through the dense tensors of Section 3.1 (Algorithm 2's formulation).

    Instead of following the routing record, every step is a sum over ALL tokens or ALL
    buffer positions, weighted by dispatch_mask / combine_weights [G,S,E,C]:
      slot input   buf[e,g,c,:] = sum_s dispatch_mask[g,s,e,c] x[g,s,:]
      expert       out[e,g,c,:] = FFN_e(buf[e,g,c,:])                        (Eq. 2)
      token output y[g,s,:]     = sum_{e,c} combine_weights[g,s,e,c] out[e,g,c,:]
    written as one small matrix product per (group, expert).  O(G S M E C): tiny inputs
    only.  The expert outputs stay in [E,G,C,M] order (reading R7).
    """
    x, wg = _f64(x), _f64(wg)
    G, S, M = x.shape
    E = wg.shape[1]
    routing = top2_gating(softmax_gates(x, wg), u, C, literal_pass2)
    weights_dense, mask_dense = dense_combine_weights(routing, E, C)
    buf = np.zeros((E, G, C, M))
    out = np.zeros((E, G, C, M))
    y = np.zeros((G, S, M))
    for g in range(G):
        for e in range(E):
            buf[e, g] = mask_dense[g, :, e, :].T @ x[g]                  # [C,S] . [S,M]
            out[e, g] = expert_ffn(buf[e, g], wi[e], wo[e])
            y[g] += weights_dense[g, :, e, :] @ out[e, g]                # [S,C] . [C,M]
    return y, routing, buf, out


# --------------------------------------------------------------------------
# Eq. 1-3: the layer by its definition
# --------------------------------------------------------------------------
def expert_hidden(rows, wi_e):
    """The inner half of Eq. 2 for a batch of rows: ReLU(rows . wi_e)   (no bias)."""
    return np.maximum(_f64(rows) @ _f64(wi_e), 0.0)


def expert_ffn(rows, wi_e, wo_e):
    """Eq. 2 for a batch of rows: relu(rows . wi_e) . wo_e   (no bias)."""
    return expert_hidden(rows, wi_e) @ _f64(wo_e)


def moe_forward(x, wg, u, wi, wo, C, literal_pass2=False):
    """y[g,s,:] = sum_e G_{s,e} FFN_e(x[g,s,:])  (Eq. 1-3), plus the routing.

    ``wi`` / ``wo`` may be any indexable whose item e converts to a float64
    [M,H] / [H,M] array (so that huge weight tensors can be widened per expert).
    Also returns buf[E,G,C,M] (dispatched inputs, zeros in empty slots) and
    out[E,G,C,M] (expert outputs), the intermediate tensors of Algorithm 2.
    """
    x = _f64(x)
    G, S, M = x.shape
    gates = softmax_gates(x, wg)
    E = gates.shape[-1]
    routing = top2_gating(gates, u, C, literal_pass2)
    src = routing["src_token"]
    buf = np.zeros((E, G, C, M))
    out = np.zeros((E, G, C, M))
    y = np.zeros((G, S, M))
    for e in range(E):
        gi, ci = np.nonzero(src[e] >= 0)
        if gi.size == 0:
            continue
        si = src[e, gi, ci]
        buf[e, gi, ci] = x[gi, si]
        out[e, gi, ci] = expert_ffn(buf[e, gi, ci], wi[e], wo[e])
    for k in range(2):
        gi, si = np.nonzero(routing["slot"][:, :, k] >= 0)
        ei = routing["expert_idx"][gi, si, k]
        ci = routing["slot"][gi, si, k]
        y[gi, si] += routing["weight"][gi, si, k][:, None] * out[ei, gi, ci]
    routing["gates"] = gates
    return y, routing, buf, out


def moe_forward_tokens(x, routing, wi, wo, tokens):
    """Eq. 1-3 for selected tokens only: ``tokens`` is a list of (g, s).

    ``routing`` comes from ``top2_gating`` on ALL tokens (slots depend on every
    earlier token of the group); the expert networks are evaluated just for the
    requested tokens.  Returns y [len(tokens), M].
    """
    x = _f64(x)
    M = x.shape[-1]
    y = np.zeros((len(tokens), M))
    by_expert = {}
    for i, (g, s) in enumerate(tokens):
        for k in range(2):
            if routing["slot"][g, s, k] >= 0:
                by_expert.setdefault(int(routing["expert_idx"][g, s, k]), []).append((i, g, s, k))
    for e, items in sorted(by_expert.items()):
        rows = np.stack([x[g, s] for (_, g, s, _) in items])
        res = expert_ffn(rows, wi[e], wo[e])
        for r, (i, g, s, k) in enumerate(items):
            y[i] += routing["weight"][g, s, k] * res[r]
    return y
