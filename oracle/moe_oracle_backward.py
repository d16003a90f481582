"""fp64 CPU oracle for the backward pass of the top-2 Mixture-of-Experts layer (GShard).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the test-suite, the smoke
check and the CPU-baseline leg of the benchmark may call it.  It shares no code
with the HIP library and imports nothing from it.

The paper trains the layer by automatic differentiation of Algorithm 2 and only
says which part of the auxiliary loss carries a gradient (Section 2.2, "Auxiliary
loss": the counts c_e are not differentiable, the mean gates m_e are).  This file
writes that derivative out by the chain rule, one function per line of the forward
definition, in float64.  With

    L = sum_{g,s,m} dy[g,s,m] * y[g,s,m]  +  sum_g daux[g] * l_aux[g]

as the scalar that is differentiated (dy, daux = upstream gradients), it returns
dL/dx, dL/dwg, dL/dwi, dL/dwo.

Readings (the paper gives no backward listing):

B1  Every discrete decision of Algorithm 1 is a constant of the derivative: the
    top-2 indices, the capacity tests, the random-routing comparison and the
    counters c_e (Section 2.2 states the last one).
B2  The normalised weights g1/(g1+g2) and g2/(g1+g2) are differentiated with
    respect to BOTH raw gates (Algorithm 1 normalises inside the function that is
    differentiated).
B3  A choice that is not kept contributes the constant 0 to Eq. 3, so nothing flows
    through its weight; when only one choice is kept the surviving weight is still
    g_k/(g1+g2) and still depends on both gates.
B4  relu'(0) = 0.
B5  l_aux = (1/E) sum_e (c_e/S) m_e with m_e = (1/S) sum_s g_{s,e}: d l_aux / d g_{s,e}
    = c_e / (E S^2), for every expert e of every token (not only the top-2).

* ``combine_backward``     -- Eq. 3 / Algorithm 2's last einsum, transposed
* ``expert_ffn_backward``  -- Eq. 2 differentiated
* ``dispatch_backward``    -- Algorithm 2's dispatch einsum, transposed
* ``gating_backward``      -- Algorithm 1's normalisation lines and the l_aux line
* ``softmax_backward``     -- the softmax line of Algorithm 1
* ``moe_backward``         -- all of it

Parity pins (tests/test_oracle_backward.py): central finite differences of the
FORWARD oracle on inputs whose routing does not change under the perturbation,
torch.autograd (float64, CPU) on an independent dense restatement of the layer,
closed forms (two experts with everything kept is a dense mixture; the l_aux-only
gradient; structure of the gradients).  Nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from . import moe_oracle as fwd


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def combine_backward(routing, out, dy):
    """y[g,s] = sum_k weight[g,s,k] out[e_k,g,c_k]  (Eq. 3)  =>

    dout[e_k,g,c_k,:] = weight[g,s,k] dy[g,s,:]   (empty slots get 0)
    dweight[g,s,k]    = <dy[g,s,:], out[e_k,g,c_k,:]>   for kept choices, else 0.
    """
    out, dy = _f64(out), _f64(dy)
    G, S, _ = routing["slot"].shape
    dout = np.zeros_like(out)
    dweight = np.zeros((G, S, 2))
    for g in range(G):
        for s in range(S):
            for k in range(2):
                c = routing["slot"][g, s, k]
                if c >= 0:
                    e = routing["expert_idx"][g, s, k]
                    dout[e, g, c] = routing["weight"][g, s, k] * dy[g, s]
                    dweight[g, s, k] = dy[g, s] @ out[e, g, c]
    return dout, dweight


def expert_ffn_backward(rows, wi_e, wo_e, dout_rows):
    """Eq. 2, out = relu(rows . wi) . wo, differentiated (reading B4).

    Returns (drows, dwi_e, dwo_e).
    """
    rows, wi_e, wo_e, dout_rows = _f64(rows), _f64(wi_e), _f64(wo_e), _f64(dout_rows)
    pre = rows @ wi_e
    h = np.maximum(pre, 0.0)
    dh = dout_rows @ wo_e.T
    dpre = np.where(pre > 0.0, dh, 0.0)
    dwo_e = h.T @ dout_rows
    dwi_e = rows.T @ dpre
    drows = dpre @ wi_e.T
    return drows, dwi_e, dwo_e


def dispatch_backward(routing, dbuf, shape_x):
    """buf[e,g,c] = x[g,s] for every kept choice  =>  dx[g,s] = sum_k dbuf[e_k,g,c_k]."""
    dx = np.zeros(shape_x)
    G, S, _ = routing["slot"].shape
    for g in range(G):
        for s in range(S):
            for k in range(2):
                c = routing["slot"][g, s, k]
                if c >= 0:
                    dx[g, s] += dbuf[routing["expert_idx"][g, s, k], g, c]
    return dx


def gating_backward(gates, routing, dweight, daux):
    """d L / d gates [G,S,E] from the gradients of the combine weights and of l_aux.

    weight_1 = g1/(g1+g2), weight_2 = g2/(g1+g2) when kept (readings B2, B3), so with
    D = g1+g2:   d weight_1 = ( g2 dg1 - g1 dg2) / D^2,
                 d weight_2 = (-g2 dg1 + g1 dg2) / D^2.
    l_aux adds daux[g] c_e/(E S^2) to every gate of group g (reading B5).
    """
    gates = _f64(gates)
    G, S, E = gates.shape
    dgates = np.zeros((G, S, E))
    for g in range(G):
        dgates[g] += daux[g] * _f64(routing["c1"][g])[None, :] / (E * S * S)
        for s in range(S):
            e1, e2 = routing["expert_idx"][g, s]
            g1, g2 = gates[g, s, e1], gates[g, s, e2]
            D = g1 + g2
            d1 = dweight[g, s, 0] if routing["slot"][g, s, 0] >= 0 else 0.0
            d2 = dweight[g, s, 1] if routing["slot"][g, s, 1] >= 0 else 0.0
            dgates[g, s, e1] += (d1 - d2) * g2 / (D * D)
            dgates[g, s, e2] += (d2 - d1) * g1 / (D * D)
    return dgates


def softmax_backward(gates, dgates):
    """g = softmax(z) over the last axis  =>  dz = g * (dg - sum_e g dg)."""
    gates, dgates = _f64(gates), _f64(dgates)
    return gates * (dgates - np.sum(gates * dgates, axis=-1, keepdims=True))


def moe_backward(x, wg, u, wi, wo, C, dy, daux, experts=None):
    """Gradients of L (see the module header) for the whole layer.

    ``wi`` / ``wo`` may be any indexable whose item e converts to float64 [M,H] / [H,M].
    ``experts``: iterable of expert indices whose weight gradients are wanted (default
    all); dx, dwg always cover every expert.  Returns a dict with dx [G,S,M], dwg [M,E],
    dwi {e: [M,H]}, dwo {e: [H,M]} and the intermediates dout, dbuf [E,G,C,M],
    dweight [G,S,2], dgates, dlogits [G,S,E].
    """
    x, wg, dy, daux = _f64(x), _f64(wg), _f64(dy), _f64(daux)
    G, S, M = x.shape
    y, routing, buf, out = fwd.moe_forward(x, wg, u, wi, wo, C)
    E = routing["gates"].shape[-1]
    want = set(range(E)) if experts is None else set(int(e) for e in experts)

    dout, dweight = combine_backward(routing, out, dy)
    dbuf = np.zeros_like(buf)
    dwi, dwo = {}, {}
    src = routing["src_token"]
    for e in range(E):
        # occupied slots only: an empty slot holds a zero row and a zero gradient, which
        # contribute nothing to either weight gradient
        gi, ci = np.nonzero(src[e] >= 0)
        if gi.size == 0:
            if e in want:
                dwi[e] = np.zeros(np.shape(wi[e]))
                dwo[e] = np.zeros(np.shape(wo[e]))
            continue
        drows, dwi_e, dwo_e = expert_ffn_backward(buf[e, gi, ci], wi[e], wo[e], dout[e, gi, ci])
        dbuf[e, gi, ci] = drows
        if e in want:
            dwi[e], dwo[e] = dwi_e, dwo_e
    dx = dispatch_backward(routing, dbuf, x.shape)

    dgates = gating_backward(routing["gates"], routing, dweight, daux)
    dlogits = softmax_backward(routing["gates"], dgates)
    # logits[g,s,e] = sum_m x[g,s,m] wg[m,e]
    E_ = dlogits.shape[-1]
    dwg = x.reshape(-1, M).T @ dlogits.reshape(-1, E_)
    dx = dx + (dlogits.reshape(-1, E_) @ wg.T).reshape(G, S, M)
    return {"dx": dx, "dwg": dwg, "dwi": dwi, "dwo": dwo, "dout": dout, "dbuf": dbuf,
            "dweight": dweight, "dgates": dgates, "dlogits": dlogits, "routing": routing,
            "y": y, "buf": buf, "out": out}
