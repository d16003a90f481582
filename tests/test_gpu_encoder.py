"""GPU parity of the encoder layers around the MoE layer (Section 2.1) against the fp64
oracle, stage by stage through the C ABI, then the fused entry point against the staged calls.

The MoE sub-layer routes discretely on its input, and the GPU's input to it carries the
rounding of everything before; so the dense part is compared with the oracle up to the MoE
layer's input, and the MoE layer is then checked on the GPU's own input (as in the parity
tests of the layer itself)."""
import numpy as np
import pytest
import torch

import paper_2006_16668_amd as moe
from harness import f64, rel_fro, shape_of
from oracle import moe_oracle as orc
from oracle import transformer_oracle as tro
from workloads import ExpertWeightsF64, MoEConfig, make_encoder_weights, make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 5e-5, "bf16": 2e-2}

# (config, sequences B, length L, heads, d)
CASES = [
    (MoEConfig("enc_flash64", G=2, S=512, M=256, H=512, E=8, C=128, act_dtype="bf16", seed=51), 4, 256, 4, 64),
    (MoEConfig("enc_flash128", G=2, S=256, M=256, H=256, E=4, C=128, act_dtype="bf16", seed=52), 2, 256, 2, 128),
    (MoEConfig("enc_long", G=1, S=1024, M=128, H=256, E=4, C=512, act_dtype="bf16", seed=53), 1, 1024, 2, 64),
    # paper-like attention shape (sequences of 1024, key/value dimension 128) at a size the
    # oracle finishes in seconds: several query / key blocks per head, several row tiles per GEMM
    (MoEConfig("enc_mid", G=4, S=1024, M=512, H=1024, E=8, C=256, act_dtype="bf16", seed=56), 4, 1024, 4, 128),
    (MoEConfig("enc_plain_bf16", G=3, S=40, M=72, H=136, E=5, C=20, act_dtype="bf16", seed=54), 4, 30, 3, 24),
    (MoEConfig("enc_f32", G=2, S=48, M=32, H=64, E=4, C=24, act_dtype="f32", seed=55), 3, 32, 2, 16),
]


def _split_qkv(wqkv, A):
    w = f64(wqkv)
    return w[:, :A], w[:, A:2 * A], w[:, 2 * A:]


def _staged(cfg, dims, inp, w):
    """The pair forward as separate C-ABI calls; returns every intermediate."""
    sh = shape_of(cfg)
    dt = sh.torch_dtype
    new = lambda *s: torch.full(s, float("nan"), dtype=dt, device=DEV)
    N3 = (cfg.G, cfg.S, cfg.M)
    aws = torch.empty(moe.moe_attention_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)
    hden = new(cfg.G, cfg.S, cfg.H)
    r = {}
    r["n1"] = new(*N3)
    moe.moe_add_layer_norm(sh, inp.x, None, w["ln_gamma"][0], w["ln_beta"][0], None, r["n1"])
    r["att1"] = new(*N3)
    moe.moe_self_attention(sh, dims, r["n1"], w["wqkv"][0], w["wo_att"][0], r["att1"], aws)
    r["a"], r["n2"] = new(*N3), new(*N3)
    moe.moe_add_layer_norm(sh, inp.x, r["att1"], w["ln_gamma"][1], w["ln_beta"][1], r["a"], r["n2"])
    r["ffn"] = new(*N3)
    moe.moe_dense_ffn(sh, r["n2"], w["w1"], w["w2"], hden, r["ffn"])
    r["b"], r["n3"] = new(*N3), new(*N3)
    moe.moe_add_layer_norm(sh, r["a"], r["ffn"], w["ln_gamma"][2], w["ln_beta"][2], r["b"], r["n3"])
    r["att2"] = new(*N3)
    moe.moe_self_attention(sh, dims, r["n3"], w["wqkv"][1], w["wo_att"][1], r["att2"], aws)
    r["c"], r["n4"] = new(*N3), new(*N3)
    moe.moe_add_layer_norm(sh, r["b"], r["att2"], w["ln_gamma"][3], w["ln_beta"][3], r["c"], r["n4"])
    r["m"] = new(*N3)
    r["aux"] = torch.full((cfg.G,), float("nan"), dtype=torch.float32, device=DEV)
    mws = torch.empty(moe.moe_workspace_bytes(sh), dtype=torch.uint8, device=DEV)
    moe.moe_forward(sh, r["n4"], inp.wg, inp.u, inp.wi, inp.wo, r["m"], r["aux"], mws)
    torch.cuda.synchronize()
    return r


@pytest.mark.parametrize("cfg,B,L,heads,d", CASES, ids=lambda v: v.name if isinstance(v, MoEConfig) else None)
def test_encoder_stages_and_pair(cfg, B, L, heads, d):
    print(f"case {cfg} B={B} L={L} heads={heads} d={d}", flush=True)
    assert B * L == cfg.G * cfg.S
    dims = moe.EncoderDims(B, L, heads, d)
    A = heads * d
    tol = TOL[cfg.act_dtype]
    inp = make_inputs(cfg, device=DEV)
    w = make_encoder_weights(cfg, heads, d, device=DEV)
    r = _staged(cfg, dims, inp, w)
    seq = lambda t: f64(t).reshape(B, L, cfg.M)

    # each stage against the oracle on the GPU's own input of that stage
    ln = lambda v, i: tro.layer_norm(f64(v), f64(w["ln_gamma"][i]), f64(w["ln_beta"][i]))
    assert rel_fro(f64(r["n1"]), ln(inp.x, 0)) < tol / 4
    for i, (u, out) in enumerate((("n1", "att1"), ("n3", "att2"))):
        wq, wk, wv = _split_qkv(w["wqkv"][i], A)
        want = tro.self_attention(seq(r[u]), wq, wk, wv, f64(w["wo_att"][i]), heads)
        got = seq(r[out])
        assert rel_fro(got, want) < tol, out
        rows = np.linalg.norm(got - want, axis=-1) / np.maximum(np.linalg.norm(want, axis=-1), 1e-30)
        assert rows.max() < 4 * tol, (out, rows.max())
    assert rel_fro(f64(r["a"]), f64(inp.x) + f64(r["att1"])) < tol / 4
    assert rel_fro(f64(r["n2"]), ln(r["a"], 1)) < tol / 4
    assert rel_fro(f64(r["ffn"]), tro.dense_ffn(f64(r["n2"]), f64(w["w1"]), f64(w["w2"]))) < tol
    assert rel_fro(f64(r["n4"]), ln(r["c"], 3)) < tol / 4
    m_want, routing, _, _ = orc.moe_forward(f64(r["n4"]), f64(inp.wg), f64(inp.u), ExpertWeightsF64(inp.wi),
                                            ExpertWeightsF64(inp.wo), cfg.C)
    assert rel_fro(f64(r["m"]), m_want) < tol

    # the dense part end to end against the oracle (no discrete decisions up to the MoE input)
    p = {f"ln{i + 1}": (f64(w["ln_gamma"][i]), f64(w["ln_beta"][i])) for i in range(4)}
    for i in (0, 1):
        p[f"wq{i + 1}"], p[f"wk{i + 1}"], p[f"wv{i + 1}"] = _split_qkv(w["wqkv"][i], A)
        p[f"wo{i + 1}"] = f64(w["wo_att"][i])
    p["w1"], p["w2"] = f64(w["w1"]), f64(w["w2"])
    x = seq(inp.x)
    a = x + tro.self_attention(tro.layer_norm(x, *p["ln1"]), p["wq1"], p["wk1"], p["wv1"], p["wo1"], heads)
    b = a + tro.dense_ffn(tro.layer_norm(a, *p["ln2"]), p["w1"], p["w2"])
    c = b + tro.self_attention(tro.layer_norm(b, *p["ln3"]), p["wq2"], p["wk2"], p["wv2"], p["wo2"], heads)
    assert rel_fro(seq(r["c"]), c) < tol
    assert rel_fro(seq(r["n4"]), tro.layer_norm(c, *p["ln4"])) < 2 * tol

    # the fused entry point is exactly the staged sequence
    sh = shape_of(cfg)
    y = torch.full((cfg.G, cfg.S, cfg.M), float("nan"), dtype=sh.torch_dtype, device=DEV)
    aux = torch.full((cfg.G,), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(moe.moe_encoder_workspace_bytes(sh, dims), dtype=torch.uint8, device=DEV)
    weights = dict(w, wg=inp.wg, wi=inp.wi, wo=inp.wo)
    moe.moe_encoder_pair_forward(sh, dims, inp.x, weights, inp.u, y, aux, ws)
    torch.cuda.synchronize()
    y_staged = (r["c"].float() + r["m"].float()).to(sh.torch_dtype)
    assert torch.equal(y, y_staged)
    assert torch.equal(aux, r["aux"])


def test_encoder_argument_errors():
    cfg = CASES[-1][0]
    sh = shape_of(cfg)
    with pytest.raises(moe.MoEError) as ei:               # B*L != G*S
        moe.moe_encoder_workspace_bytes(sh, moe.EncoderDims(3, 31, 2, 16))
    assert ei.value.status == -1
    with pytest.raises(moe.MoEError) as ei:               # head dimension not a multiple of 8
        moe.moe_attention_workspace_bytes(sh, moe.EncoderDims(3, 32, 2, 12))
    assert ei.value.status == -2
