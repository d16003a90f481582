"""HIP path against the fp64 oracle, element by element, through the C ABI.

Tolerances: integer routing bit-exact; gates / weights / auxiliary loss 1e-5
relative (fp32 arithmetic, fp64 oracle); expert and layer outputs 2e-2 relative
in the Frobenius norm with bf16 experts, 1e-5 with fp32 experts.
"""
import numpy as np
import pytest
import torch

import paper_2006_16668_amd as moe
from oracle import moe_oracle as orc
from workloads import CONFIGS, ExpertWeightsF64, MoEConfig, make_inputs

from harness import (assert_gate_floats_close, assert_routing_equal, f64, gpu_forward, gpu_gate,
                     rel_fro, shape_of)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

OUT_TOL = {"bf16": 2e-2, "f32": 1e-5}

# several tiles and ragged tails: S not a multiple of the 64-token chunk, M / H not
# multiples of the 64-wide K step, rows per expert not a multiple of the GEMM tile
SMALL_CASES = [
    CONFIGS["tiny"],
    CONFIGS["small"],
    MoEConfig("ragged_bf16", G=3, S=200, M=72, H=136, E=5, C=37, act_dtype="bf16", seed=11),
    MoEConfig("ragged_f32", G=2, S=131, M=40, H=88, E=7, C=50, act_dtype="f32", seed=12),
    MoEConfig("e130", G=2, S=300, M=64, H=64, E=130, C=6, act_dtype="bf16", seed=13),
    MoEConfig("two_experts", G=2, S=96, M=32, H=48, E=2, C=96, act_dtype="f32", seed=14),
    MoEConfig("capacity_one", G=4, S=70, M=32, H=32, E=6, C=1, act_dtype="bf16", seed=15),
    MoEConfig("one_token", G=5, S=1, M=16, H=24, E=3, C=2, act_dtype="f32", seed=16),
    MoEConfig("wide_rows", G=2, S=520, M=256, H=520, E=3, C=300, act_dtype="bf16", seed=17),
    # one case per width class of the gate kernels (<=32, <=64, <=128, <=256, <=384, <=512, wider)
    MoEConfig("e48", G=2, S=190, M=96, H=32, E=48, C=9, act_dtype="bf16", seed=18),
    MoEConfig("e100", G=3, S=129, M=200, H=32, E=100, C=4, act_dtype="bf16", seed=19),
    MoEConfig("e300", G=1, S=333, M=72, H=32, E=300, C=3, act_dtype="bf16", seed=20),
    MoEConfig("e512", G=2, S=260, M=128, H=32, E=512, C=2, act_dtype="bf16", seed=23),
    MoEConfig("e600", G=1, S=100, M=64, H=32, E=600, C=1, act_dtype="bf16", seed=24),
    MoEConfig("e130_f32", G=1, S=150, M=48, H=32, E=130, C=3, act_dtype="f32", seed=25),
    # exact 256x256 tiles (persistent copy-engine GEMM) with awkward tile counts: fewer tiles
    # than XCDs, a tile count that is no multiple of 8, several row tiles, a single K step
    MoEConfig("tiles_3", G=2, S=300, M=256, H=512, E=3, C=128, act_dtype="bf16", seed=26),
    MoEConfig("tiles_rows", G=2, S=700, M=256, H=256, E=5, C=256, act_dtype="bf16", seed=27),
    MoEConfig("one_k_step", G=1, S=600, M=32, H=256, E=4, C=256, act_dtype="bf16", seed=28),
    MoEConfig("one_k_step_2", G=1, S=600, M=256, H=32, E=4, C=256, act_dtype="bf16", seed=29),
    MoEConfig("many_tiles", G=2, S=1100, M=512, H=768, E=19, C=128, act_dtype="bf16", seed=30),
    # the layer entry point gathers the rows of the first GEMM straight from x for these
    # shapes: shortest K the gather takes, a capacity that is no power of two with row tiles
    # that straddle groups and mostly empty slots; capacity 1; more tiles than compute units
    MoEConfig("gather_k128", G=16, S=100, M=128, H=256, E=8, C=48, act_dtype="bf16", seed=31),
    MoEConfig("gather_c1", G=256, S=4, M=160, H=256, E=3, C=1, act_dtype="bf16", seed=32),
    # more than 512 experts (the paper goes to 2048 per layer): logits as one GEMM on the matrix
    # cores with wg in three bf16 terms, then a per-token softmax / top-2 pass
    MoEConfig("e640_wide", G=2, S=512, M=256, H=32, E=640, C=2, act_dtype="bf16", seed=34),
    MoEConfig("e2048_wide", G=1, S=1024, M=128, H=32, E=2048, C=1, act_dtype="bf16", seed=35),
    # fp32 activations with GEMM-friendly shapes: logits on the matrix cores with x and wg each in
    # three bf16 terms (all nine exact products)
    MoEConfig("f32_mfma_gate", G=2, S=256, M=64, H=64, E=12, C=64, act_dtype="f32", seed=36),
    # fp32 expert GEMMs on the matrix cores: several 128 x 128 tiles with ragged tails in rows,
    # columns and K (rows per expert = 303, no multiple of 4 either)
    MoEConfig("f32_tiles", G=3, S=200, M=136, H=264, E=3, C=101, act_dtype="f32", seed=37),
    # fp32 rows need 16 bytes = 4 elements only
    MoEConfig("f32_quads", G=3, S=90, M=36, H=44, E=5, C=21, act_dtype="f32", seed=48),
    MoEConfig("gather_wrap", G=8, S=400, M=128, H=2048, E=40, C=32, act_dtype="bf16", seed=33),
    # 64 < E <= 128 with enough tokens for the 256-token blocks of the gate (one block per compute
    # unit): blocks whose last chunks are ragged or missing, a feature count that is no multiple
    # of 64
    MoEConfig("e100_blocks256", G=256, S=130, M=72, H=32, E=100, C=3, act_dtype="bf16", seed=49),
    MoEConfig("e128_blocks256", G=128, S=300, M=128, H=32, E=128, C=5, act_dtype="bf16", seed=50),
    # more than 64 chunks per group: the scan over the chunks walks its segments in several batches
    MoEConfig("long_group", G=2, S=4250, M=32, H=16, E=6, C=700, act_dtype="bf16", seed=51),
    # the layer call packs the occupied rows of an expert to the front of its block and multiplies
    # only the 256-row tiles that hold them: skewed routing (full and nearly empty experts), far
    # more capacity than tokens (one tile of several per expert), experts that receive nothing,
    # many groups with few slots each, a row-tile count that straddles bands of eight
    MoEConfig("packed_skew", G=8, S=512, M=256, H=256, E=16, C=64, act_dtype="bf16", seed=38,
              logit_bias_std=1.0),
    MoEConfig("packed_sparse", G=4, S=64, M=256, H=512, E=8, C=192, act_dtype="bf16", seed=39),
    MoEConfig("packed_empty_experts", G=2, S=8, M=256, H=256, E=32, C=128, act_dtype="bf16", seed=40),
    MoEConfig("packed_c16", G=16, S=160, M=256, H=256, E=20, C=16, act_dtype="bf16", seed=46),
    MoEConfig("packed_bands", G=4, S=1500, M=256, H=512, E=5, C=704, act_dtype="bf16", seed=47,
              logit_bias_std=0.7),
]


def _oracle_layer(cfg, inp):
    x, wg, u = inp.host_f64()
    return orc.moe_forward(x, wg, u, ExpertWeightsF64(inp.wi), ExpertWeightsF64(inp.wo), cfg.C)


@pytest.mark.parametrize("cfg", SMALL_CASES, ids=lambda c: c.name)
def test_stages_and_layer_match_oracle(cfg):
    print(f"case {cfg}", flush=True)
    inp = make_inputs(cfg, device=DEV)
    y_want, want, buf_want, out_want = _oracle_layer(cfg, inp)
    sh = shape_of(cfg)

    # --- gating
    r = gpu_gate(cfg, inp.x, inp.wg, inp.u)
    assert_routing_equal(r, want)
    assert_gate_floats_close(r, want, gates=want["gates"])

    # --- dispatch: a copy, so exact
    buf = torch.full((cfg.E, cfg.G, cfg.C, cfg.M), float("nan"), dtype=sh.torch_dtype, device=DEV)
    moe.moe_dispatch(sh, inp.x, r["src_token"], buf)
    torch.cuda.synchronize()
    assert np.array_equal(f64(buf), buf_want)

    # --- experts
    h = torch.empty((cfg.E, cfg.G, cfg.C, cfg.H), dtype=sh.torch_dtype, device=DEV)
    out = torch.full((cfg.E, cfg.G, cfg.C, cfg.M), float("nan"), dtype=sh.torch_dtype, device=DEV)
    moe.moe_expert_ffn(sh, buf, inp.wi, inp.wo, h, out)
    torch.cuda.synchronize()
    tol = OUT_TOL[cfg.act_dtype]
    assert rel_fro(f64(out), out_want) < tol
    # per occupied row as well, so a single broken row cannot hide in the norm
    occ = want["src_token"] >= 0
    if occ.any():
        got_rows, want_rows = f64(out)[occ], out_want[occ]
        row_err = np.linalg.norm(got_rows - want_rows, axis=1) / np.maximum(
            np.linalg.norm(want_rows, axis=1), 1e-30)
        assert row_err.max() < 4 * tol, row_err.max()
    assert (f64(out)[~occ] == 0).all()                 # FFN_e(0) = 0

    # --- combine on the GPU's own expert outputs
    y = torch.full((cfg.G, cfg.S, cfg.M), float("nan"), dtype=sh.torch_dtype, device=DEV)
    moe.moe_combine(sh, out, r["expert_idx"], r["slot"], r["weight"], y)
    torch.cuda.synchronize()
    assert rel_fro(f64(y), y_want) < tol
    dropped = (want["slot"] < 0).all(axis=-1)
    assert (f64(y)[dropped] == 0).all()                # fully dropped token -> zero row

    # --- fused entry point gives the same bits as the staged calls
    y2, aux2 = gpu_forward(cfg, inp)
    assert torch.equal(y2, y)
    assert torch.equal(aux2, r["aux"])

    # --- gate weights packed once by the caller (moe_gate_pack): same bits from both entry points
    nbytes = moe.moe_gate_pack_bytes(sh)
    wgp = torch.empty(nbytes, dtype=torch.uint8, device=DEV) if nbytes else None
    moe.moe_gate_pack(sh, inp.wg, wgp)
    y3 = torch.full_like(y, float("nan"))
    aux3 = torch.full_like(aux2, float("nan"))
    lws = torch.empty(moe.moe_workspace_bytes(sh), dtype=torch.uint8, device=DEV)
    moe.moe_forward_prepacked(sh, inp.x, inp.wg, wgp, inp.u, inp.wi, inp.wo, y3, aux3, lws)
    torch.cuda.synchronize()
    assert torch.equal(y3, y) and torch.equal(aux3, r["aux"])
    r3 = {k: torch.full_like(v, -9) for k, v in r.items() if v is not None}
    gws = torch.empty(moe.moe_gate_workspace_bytes(sh), dtype=torch.uint8, device=DEV)
    moe.moe_gate_prepacked(sh, inp.x, inp.wg, wgp, inp.u, r3["expert_idx"], r3["slot"], r3["weight"],
                           r3["fill"], r3["src_token"], r3["c1"], r3["mean_gate"], r3["aux"],
                           r3["gates"], gws)
    torch.cuda.synchronize()
    for k in r3:
        assert torch.equal(r3[k], r[k]), k

    # --- experts again with fill and a workspace: occupied rows only.  Same bits in every
    # occupied slot; where the kernels pack (moe_forward_packs_rows) the other slots of out are
    # not written, elsewhere the call is the one above
    out2 = torch.full((cfg.E, cfg.G, cfg.C, cfg.M), 77.0, dtype=sh.torch_dtype, device=DEV)
    h2 = torch.empty_like(h)
    fws = torch.empty(max(moe.moe_expert_ffn_workspace_bytes(sh), 256), dtype=torch.uint8, device=DEV)
    moe.moe_expert_ffn(sh, buf, inp.wi, inp.wo, h2, out2, fill=r["fill"], ws=fws)
    torch.cuda.synchronize()
    occ_t = torch.from_numpy(occ).to(DEV)
    assert torch.equal(out2[occ_t], out[occ_t])
    if moe.moe_forward_packs_rows(sh):
        assert (out2[~occ_t] == 77.0).all()
    else:
        assert torch.equal(out2, out)


def test_combine_is_exact_gather_for_identity_like_inputs():
    """Dispatch then combine with out := buf: y = (w0 + w1) x up to one rounding."""
    cfg = MoEConfig("roundtrip", G=2, S=150, M=64, H=64, E=4, C=80, act_dtype="f32", seed=21)
    inp = make_inputs(cfg, device=DEV)
    sh = shape_of(cfg)
    r = gpu_gate(cfg, inp.x, inp.wg, inp.u)
    buf = torch.empty((cfg.E, cfg.G, cfg.C, cfg.M), dtype=torch.float32, device=DEV)
    moe.moe_dispatch(sh, inp.x, r["src_token"], buf)
    y = torch.empty_like(inp.x)
    moe.moe_combine(sh, buf, r["expert_idx"], r["slot"], r["weight"], y)
    torch.cuda.synchronize()
    wsum = f64(r["weight"]).sum(-1, keepdims=True)
    np.testing.assert_allclose(f64(y), wsum * f64(inp.x), rtol=3e-7, atol=1e-30)


def test_zero_gate_weights_tie_break_and_closed_form_aux():
    """wg = 0: every token ties; lowest indices win, expert 0 keeps the first C tokens,
    l_aux = 1/E^2 (closed form)."""
    cfg = MoEConfig("ties", G=2, S=100, M=32, H=32, E=8, C=10, act_dtype="bf16", seed=22)
    inp = make_inputs(cfg, device=DEV, condition=False)
    wg = torch.zeros_like(inp.wg)
    u = torch.zeros_like(inp.u)
    r = gpu_gate(cfg, inp.x, wg, u)
    idx = r["expert_idx"].cpu().numpy()
    assert (idx[..., 0] == 0).all() and (idx[..., 1] == 1).all()
    slot = r["slot"].cpu().numpy()
    want = np.where(np.arange(cfg.S) < cfg.C, np.arange(cfg.S), -1)
    assert (slot[..., 0] == want).all() and (slot[..., 1] == want).all()
    np.testing.assert_allclose(f64(r["aux"]), 1.0 / cfg.E ** 2, rtol=1e-6)
    np.testing.assert_allclose(f64(r["gates"]), 1.0 / cfg.E, rtol=1e-6)


def test_results_are_deterministic():
    cfg = CONFIGS["small"]
    inp = make_inputs(cfg, device=DEV)
    y1, a1 = gpu_forward(cfg, inp)
    y2, a2 = gpu_forward(cfg, inp)
    assert torch.equal(y1, y2) and torch.equal(a1, a2)
    r1 = gpu_gate(cfg, inp.x, inp.wg, inp.u)
    r2 = gpu_gate(cfg, inp.x, inp.wg, inp.u)
    for k in r1:
        assert torch.equal(r1[k], r2[k]), k


def test_argument_errors_enqueue_nothing():
    cfg = CONFIGS["tiny"]
    inp = make_inputs(cfg, device=DEV)
    sh = shape_of(cfg)
    y = torch.zeros_like(inp.x)
    aux = torch.zeros(cfg.G, dtype=torch.float32, device=DEV)
    small_ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_forward(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, small_ws)
    assert ei.value.status == -3
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_workspace_bytes(moe.MoEShape(1, 64, 30, 64, 4, 32, "f32"))   # fp32: M % 4 != 0
    assert ei.value.status == -2
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_workspace_bytes(moe.MoEShape(1, 64, 36, 64, 4, 32, "bf16"))  # bf16: M % 8 != 0
    assert ei.value.status == -2
    assert moe.moe_workspace_bytes(moe.MoEShape(1, 64, 36, 64, 4, 32, "f32")) > 0
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_workspace_bytes(moe.MoEShape(1, 64, 32, 64, 1, 32, "f32"))   # E < 2
    assert ei.value.status == -1
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_workspace_bytes(moe.MoEShape(0, 64, 32, 64, 4, 32, "f32"))   # empty batch
    assert ei.value.status == -1
    torch.cuda.synchronize()
    assert (y == 0).all()


def test_expert_parallel_layout_on_one_gpu():
    """The D-device deployment of Section 3 (groups sharded before the experts, experts
    sharded inside, one exchange each way) replayed on one GPU with the staged entry points:
    every "device" gates and dispatches its own groups over ALL experts, the exchange is a
    tensor permutation, every device runs its E/D experts on the rows of all groups, the
    reverse exchange, and each device combines its own tokens.  Rows are independent in
    every stage, so the result equals the single-device layer bit for bit."""
    cfg = next(c for c in SMALL_CASES if c.name == "small")          # G=4, E=16
    D = 4
    inp = make_inputs(cfg, device=DEV)
    y_ref, aux_ref = gpu_forward(cfg, inp)
    Gl, El = cfg.G // D, cfg.E // D
    dt = shape_of(cfg).torch_dtype
    sh_tok = moe.MoEShape(Gl, cfg.S, cfg.M, cfg.H, cfg.E, cfg.C, cfg.act_dtype)    # a device's tokens, all experts
    sh_exp = moe.MoEShape(cfg.G, cfg.S, cfg.M, cfg.H, El, cfg.C, cfg.act_dtype)    # a device's experts, all groups
    routes, bufs = [], []
    for d in range(D):
        xs, us = inp.x[d * Gl:(d + 1) * Gl].contiguous(), inp.u[d * Gl:(d + 1) * Gl].contiguous()
        sub = cfg.with_(G=Gl)
        r = gpu_gate(sub, xs, inp.wg, us, want_gates=False)
        buf = torch.empty((cfg.E, Gl, cfg.C, cfg.M), dtype=dt, device=DEV)
        moe.moe_dispatch(sh_tok, xs, r["src_token"], buf)
        routes.append(r)
        bufs.append(buf)
    # exchange: device d receives expert block d of every device's buffer -> [El, G, C, M]
    outs = []
    for d in range(D):
        recv = torch.cat([b[d * El:(d + 1) * El] for b in bufs], dim=1).contiguous()
        h = torch.empty((El, cfg.G, cfg.C, cfg.H), dtype=dt, device=DEV)
        out = torch.empty((El, cfg.G, cfg.C, cfg.M), dtype=dt, device=DEV)
        moe.moe_expert_ffn(sh_exp, recv, inp.wi[d * El:(d + 1) * El].contiguous(),
                           inp.wo[d * El:(d + 1) * El].contiguous(), h, out)
        outs.append(out)
    # reverse exchange and combine
    full = torch.cat(outs, dim=0)                                     # [E, G, C, M]
    for d in range(D):
        mine = full[:, d * Gl:(d + 1) * Gl].contiguous()
        y = torch.empty((Gl, cfg.S, cfg.M), dtype=dt, device=DEV)
        r = routes[d]
        moe.moe_combine(sh_tok, mine, r["expert_idx"], r["slot"], r["weight"], y)
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref[d * Gl:(d + 1) * Gl])
        assert torch.equal(r["aux"], aux_ref[d * Gl:(d + 1) * Gl])


def test_forward_and_backward_replay_from_a_hip_graph():
    """The library only enqueues kernels on the caller's stream (no allocation, no
    synchronisation, no memset nodes), so a layer step can be captured once and replayed.
    Replays with fresh inputs in the captured buffers must equal eager calls bit for bit,
    on every replay (eager work and synchronisations in between)."""
    from harness import gpu_forward_backward
    from workloads import make_upstream
    cfg = next(c for c in SMALL_CASES if c.name == "small")
    sh = shape_of(cfg)
    inputs = [make_inputs(cfg.with_(seed=cfg.seed + k), device=DEV) for k in range(3)]
    ups = [make_upstream(cfg.with_(seed=cfg.seed + k), device=DEV) for k in range(3)]
    st = inputs[0]
    x, wg, u = st.x.clone(), st.wg.clone(), st.u.clone()
    wi, wo = st.wi.clone(), st.wo.clone()
    dy, daux = ups[0][0].clone(), ups[0][1].clone()
    y = torch.empty_like(x)
    aux = torch.empty(cfg.G, dtype=torch.float32, device=DEV)
    dx, dwg, dwi, dwo = torch.empty_like(x), torch.empty_like(wg), torch.empty_like(wi), torch.empty_like(wo)
    fws = torch.empty(moe.moe_train_workspace_bytes(sh), dtype=torch.uint8, device=DEV)
    bws = torch.empty(moe.moe_backward_workspace_bytes(sh), dtype=torch.uint8, device=DEV)

    def step():
        moe.moe_forward_train(sh, x, wg, u, wi, wo, y, aux, fws)
        moe.moe_backward(sh, x, wg, wi, wo, dy, daux, fws, dx, dwg, dwi, dwo, bws)

    moe.moe_prepare()                                 # one-time kernel attributes, before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in (1, 2, 0, 1):
        inp, (dyk, dauxk) = inputs[k], ups[k]
        x.copy_(inp.x); wg.copy_(inp.wg); u.copy_(inp.u); wi.copy_(inp.wi); wo.copy_(inp.wo)
        dy.copy_(dyk); daux.copy_(dauxk)
        graph.replay()
        torch.cuda.synchronize()
        got = {"y": y.clone(), "aux": aux.clone(), "dx": dx.clone(), "dwg": dwg.clone(),
               "dwi": dwi.clone(), "dwo": dwo.clone()}
        want = gpu_forward_backward(cfg, inp, dyk, dauxk)            # eager, own buffers
        for name in got:
            assert torch.equal(got[name], want[name]), (k, name)
