"""GPU parity of the backward pass of the two encoder layers against the fp64 oracle, through
the C ABI.

The MoE sub-layer routes discretely on its input and the GPU's activations carry the rounding
of everything before them, so the oracle's chain rule is evaluated at the GPU's own forward
activations (taken from the staged forward calls, which the fused entry point reproduces bit
for bit): every oracle stage gets the GPU's input of that stage and the ORACLE's upstream
gradient.  The fp32 case is also compared with the oracle run end to end from x."""
import numpy as np
import pytest
import torch

import paper_2006_16668_amd as moe
from harness import f64, rel_fro, shape_of
from oracle import moe_oracle_backward as orb
from oracle import transformer_oracle_backward as trb
from test_gpu_encoder import CASES, _split_qkv, _staged
from workloads import ExpertWeightsF64, MoEConfig, make_encoder_weights, make_inputs, make_upstream

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 2e-5, "bf16": 1.5e-2}


def _gpu_backward(cfg, dims, inp, w, dy, daux):
    sh = shape_of(cfg)
    dt = sh.torch_dtype
    weights = dict(w, wg=inp.wg, wi=inp.wi, wo=inp.wo)
    y = torch.full((cfg.G, cfg.S, cfg.M), float("nan"), dtype=dt, device=DEV)
    aux = torch.full((cfg.G,), float("nan"), dtype=torch.float32, device=DEV)
    fws = torch.empty(moe.moe_encoder_train_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)
    moe.moe_encoder_pair_forward_train(sh, dims, inp.x, weights, inp.u, y, aux, fws)
    nan_like = lambda t: torch.full_like(t, float("nan"))
    grads = {"ln_gamma": [nan_like(t) for t in w["ln_gamma"]], "ln_beta": [nan_like(t) for t in w["ln_beta"]],
             "wqkv": [nan_like(t) for t in w["wqkv"]], "wo_att": [nan_like(t) for t in w["wo_att"]],
             "w1": nan_like(w["w1"]), "w2": nan_like(w["w2"]), "wg": nan_like(inp.wg),
             "wi": nan_like(inp.wi), "wo": nan_like(inp.wo)}
    dx = nan_like(inp.x)
    bws = torch.empty(moe.moe_encoder_backward_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)
    moe.moe_encoder_pair_backward(sh, dims, inp.x, weights, dy, daux, fws, dx, grads, bws)
    torch.cuda.synchronize()
    return y, aux, dx, grads


@pytest.mark.parametrize("cfg,B,L,heads,d", CASES, ids=lambda v: v.name if isinstance(v, MoEConfig) else None)
def test_encoder_pair_backward(cfg, B, L, heads, d):
    print(f"case {cfg} B={B} L={L} heads={heads} d={d}", flush=True)
    dims = moe.EncoderDims(B, L, heads, d)
    A = heads * d
    tol = TOL[cfg.act_dtype]
    inp = make_inputs(cfg, device=DEV)
    w = make_encoder_weights(cfg, heads, d, device=DEV)
    dy, daux = make_upstream(cfg, device=DEV)
    y, aux, dx, g = _gpu_backward(cfg, dims, inp, w, dy, daux)

    # the training forward is the inference forward
    sh = shape_of(cfg)
    y2, aux2 = torch.empty_like(y), torch.empty_like(aux)
    ws = torch.empty(moe.moe_encoder_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)
    moe.moe_encoder_pair_forward(sh, dims, inp.x, dict(w, wg=inp.wg, wi=inp.wi, wo=inp.wo), inp.u, y2, aux2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(aux, aux2)

    # oracle chain at the GPU's forward activations
    r = _staged(cfg, dims, inp, w)
    seq = lambda t: f64(t).reshape(B, L, cfg.M)
    gam = [f64(t) for t in w["ln_gamma"]]
    dyf = f64(dy)
    m = orb.moe_backward(f64(r["n4"]), f64(inp.wg), f64(inp.u), ExpertWeightsF64(inp.wi),
                         ExpertWeightsF64(inp.wo), cfg.C, dyf, f64(daux))
    want = {"wg": m["dwg"], "wi": np.stack([m["dwi"][e] for e in range(cfg.E)]),
            "wo": np.stack([m["dwo"][e] for e in range(cfg.E)])}
    dln, want["g3"], want["b3"] = trb.layer_norm_backward(f64(r["c"]), gam[3], m["dx"])
    gc = dyf + dln
    wq, wk, wv = _split_qkv(w["wqkv"][1], A)
    dn3, dwq, dwk, dwv, want["wo_att1"] = trb.self_attention_backward(
        seq(r["n3"]), wq, wk, wv, f64(w["wo_att"][1]), heads, gc.reshape(B, L, cfg.M))
    want["wqkv1"] = np.concatenate([dwq, dwk, dwv], axis=1)
    dln, want["g2"], want["b2"] = trb.layer_norm_backward(f64(r["b"]), gam[2], dn3.reshape(dyf.shape))
    gb = gc + dln
    dn2, want["w1"], want["w2"] = trb.dense_ffn_backward(f64(r["n2"]), f64(w["w1"]), f64(w["w2"]), gb)
    dln, want["g1"], want["b1"] = trb.layer_norm_backward(f64(r["a"]), gam[1], dn2)
    ga = gb + dln
    wq, wk, wv = _split_qkv(w["wqkv"][0], A)
    dn1, dwq, dwk, dwv, want["wo_att0"] = trb.self_attention_backward(
        seq(r["n1"]), wq, wk, wv, f64(w["wo_att"][0]), heads, ga.reshape(B, L, cfg.M))
    want["wqkv0"] = np.concatenate([dwq, dwk, dwv], axis=1)
    dln, want["g0"], want["b0"] = trb.layer_norm_backward(f64(inp.x), gam[0], dn1.reshape(dyf.shape))
    want["dx"] = ga + dln

    got = {"dx": dx, "wg": g["wg"], "wi": g["wi"], "wo": g["wo"], "w1": g["w1"], "w2": g["w2"]}
    for i in range(2):
        got[f"wqkv{i}"], got[f"wo_att{i}"] = g["wqkv"][i], g["wo_att"][i]
    for i in range(4):
        got[f"g{i}"], got[f"b{i}"] = g["ln_gamma"][i], g["ln_beta"][i]
    errs = {k: rel_fro(f64(got[k]), want[k]) for k in want}
    print("  rel errors:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert np.isfinite(f64(got[k])).all(), k
        assert v < tol, (k, v)
    # per token row of dx
    rows = np.linalg.norm(f64(dx) - want["dx"], axis=-1) / np.maximum(np.linalg.norm(want["dx"], axis=-1), 1e-30)
    assert rows.max() < 8 * tol, rows.max()

    if cfg.act_dtype == "f32":
        # end to end from x: same routing as long as no gate is within rounding of a tie
        p = {f"ln{i + 1}": (gam[i], f64(w["ln_beta"][i])) for i in range(4)}
        for i in (0, 1):
            p[f"wq{i + 1}"], p[f"wk{i + 1}"], p[f"wv{i + 1}"] = _split_qkv(w["wqkv"][i], A)
            p[f"wo{i + 1}"] = f64(w["wo_att"][i])
        p["w1"], p["w2"] = f64(w["w1"]), f64(w["w2"])
        p["wg"], p["wi"], p["wo"] = f64(inp.wg), f64(inp.wi), f64(inp.wo)
        full = trb.encoder_pair_backward(seq(inp.x), p, heads, cfg.G, cfg.C, f64(inp.u), seq(dy), f64(daux))
        assert rel_fro(seq(dx), full["dx"]) < tol
        assert rel_fro(f64(g["w1"]), full["w1"]) < tol
        assert rel_fro(f64(g["wqkv"][0]), np.concatenate([full["wq1"], full["wk1"], full["wv1"]], axis=1)) < tol
        assert rel_fro(f64(g["ln_gamma"][0]), full["ln1"][0]) < tol


def test_encoder_backward_is_reproducible_and_checks_arguments():
    cfg, B, L, heads, d = CASES[-1]
    dims = moe.EncoderDims(B, L, heads, d)
    inp = make_inputs(cfg, device=DEV)
    w = make_encoder_weights(cfg, heads, d, device=DEV)
    dy, daux = make_upstream(cfg, device=DEV)
    _, _, dx1, g1 = _gpu_backward(cfg, dims, inp, w, dy, daux)
    _, _, dx2, g2 = _gpu_backward(cfg, dims, inp, w, dy, daux)
    assert torch.equal(dx1, dx2)
    assert torch.equal(g1["w1"], g2["w1"]) and torch.equal(g1["ln_gamma"][2], g2["ln_gamma"][2])
    sh = shape_of(cfg)
    with pytest.raises(moe.MoEError) as ei:               # workspace too small
        weights = dict(w, wg=inp.wg, wi=inp.wi, wo=inp.wo)
        small = torch.empty(1024, dtype=torch.uint8, device=DEV)
        y = torch.empty_like(inp.x)
        aux = torch.empty(cfg.G, dtype=torch.float32, device=DEV)
        moe.moe_encoder_pair_forward_train(sh, dims, inp.x, weights, inp.u, y, aux, small)
    assert ei.value.status == -3


def test_encoder_training_step_replays_from_a_hip_graph():
    """Forward-train + backward of the pair only enqueue kernels on the caller's stream, so the
    step can be captured once and replayed on fresh inputs in the captured buffers; every
    replay must equal the eager calls bit for bit."""
    cfg, B, L, heads, d = CASES[0]
    dims = moe.EncoderDims(B, L, heads, d)
    sh = shape_of(cfg)
    sets = []
    for k in range(2):
        c = cfg.with_(seed=cfg.seed + 7 * k)
        sets.append((make_inputs(c, device=DEV), make_encoder_weights(c, heads, d, device=DEV),
                     make_upstream(c, device=DEV)))
    inp0, w0, (dy0, daux0) = sets[0]
    x, u = inp0.x.clone(), inp0.u.clone()
    weights = {k: ([t.clone() for t in v] if isinstance(v, list) else v.clone()) for k, v in w0.items()}
    weights.update(wg=inp0.wg.clone(), wi=inp0.wi.clone(), wo=inp0.wo.clone())
    dy, daux = dy0.clone(), daux0.clone()
    y = torch.empty_like(x)
    aux = torch.empty(cfg.G, dtype=torch.float32, device=DEV)
    grads = {k: ([torch.empty_like(t) for t in v] if isinstance(v, list) else torch.empty_like(v))
             for k, v in weights.items()}
    dx = torch.empty_like(x)
    fws = torch.empty(moe.moe_encoder_train_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)
    bws = torch.empty(moe.moe_encoder_backward_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)

    def step():
        moe.moe_encoder_pair_forward_train(sh, dims, x, weights, u, y, aux, fws)
        moe.moe_encoder_pair_backward(sh, dims, x, weights, dy, daux, fws, dx, grads, bws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                        # first call outside capture: one-time kernel attributes
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in (1, 0, 1):
        inp, w, (dyk, dauxk) = sets[k]
        x.copy_(inp.x); u.copy_(inp.u); dy.copy_(dyk); daux.copy_(dauxk)
        for name, v in w.items():
            if isinstance(v, list):
                for dst, src in zip(weights[name], v):
                    dst.copy_(src)
            else:
                weights[name].copy_(v)
        weights["wg"].copy_(inp.wg); weights["wi"].copy_(inp.wi); weights["wo"].copy_(inp.wo)
        graph.replay()
        torch.cuda.synchronize()
        y_e, aux_e, dx_e, g_e = _gpu_backward(cfg, dims, inp, w, dyk, dauxk)      # eager, own buffers
        assert torch.equal(y, y_e) and torch.equal(aux, aux_e) and torch.equal(dx, dx_e), k
        for name in ("w1", "w2", "wg", "wi", "wo"):
            assert torch.equal(grads[name], g_e[name]), (k, name)
        for i in range(2):
            assert torch.equal(grads["wqkv"][i], g_e["wqkv"][i]) and torch.equal(grads["wo_att"][i], g_e["wo_att"][i])
        for i in range(4):
            assert torch.equal(grads["ln_gamma"][i], g_e["ln_gamma"][i]) and torch.equal(grads["ln_beta"][i], g_e["ln_beta"][i])


def test_encoder_backward_is_linear_in_the_upstream_gradient():
    """Every backward kernel is linear in the incoming gradient and a factor of 4 is exact in
    floating point, so scaling dy and daux by 4 must scale every result by exactly 4."""
    cfg, B, L, heads, d = CASES[1]
    dims = moe.EncoderDims(B, L, heads, d)
    inp = make_inputs(cfg, device=DEV)
    w = make_encoder_weights(cfg, heads, d, device=DEV)
    dy, daux = make_upstream(cfg, device=DEV)
    _, _, dx1, g1 = _gpu_backward(cfg, dims, inp, w, dy, daux)
    _, _, dx4, g4 = _gpu_backward(cfg, dims, inp, w, dy * 4, daux * 4)
    assert torch.equal(dx4, dx1 * 4)
    for k in ("w1", "w2", "wg", "wi", "wo"):
        assert torch.equal(g4[k], g1[k] * 4), k
    for i in range(2):
        assert torch.equal(g4["wqkv"][i], g1["wqkv"][i] * 4) and torch.equal(g4["wo_att"][i], g1["wo_att"][i] * 4)
    for i in range(4):
        assert torch.equal(g4["ln_gamma"][i], g1["ln_gamma"][i] * 4)
        assert torch.equal(g4["ln_beta"][i], g1["ln_beta"][i] * 4)
