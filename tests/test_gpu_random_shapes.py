"""Forward and backward of the layer on randomly drawn small shapes (seeded): the routing
record must equal the oracle's bit for bit, outputs and gradients within the tolerances of the
fixed parity cases.  Catches shape-dependent mistakes (tails, tile counts, width classes of the
gate kernels) that a hand-picked list may miss."""
import numpy as np
import pytest
import torch

from harness import f64, gpu_forward_backward, gpu_gate, rel_fro
from oracle import moe_oracle_backward as orb
from workloads import ExpertWeightsF64, MoEConfig, make_inputs, make_upstream

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _draw(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for k in range(n):
        dt = "bf16" if rng.random() < 0.6 else "f32"
        G = int(rng.integers(1, 5))
        S = int(rng.choice([1, 3, 17, 64, 65, 100, 128, 200, 256, 300, 512]))
        M, H = 8 * int(rng.integers(1, 40)), 8 * int(rng.integers(1, 40))
        if rng.random() < 0.3:
            M, H = 256 * int(rng.integers(1, 3)), 256 * int(rng.integers(1, 3))
        E = int(rng.choice([2, 3, 4, 7, 8, 16, 31, 33, 64, 100, 129, 257]))
        C = int(rng.choice([1, 2, 5, 16, 37, 64, 128, 256]))
        if rng.random() < 0.3 and G in (1, 2, 4):
            C = 256 // G                      # rows per expert = one 256-row GEMM tile
        out.append(MoEConfig(f"random{k}", G=G, S=S, M=M, H=H, E=E, C=C, act_dtype=dt, seed=7000 + k,
                             logit_bias_std=float(rng.choice([0.0, 0.0, 0.5]))))
    return out


@pytest.mark.parametrize("cfg", _draw(24, seed=7), ids=lambda c: c.name)
def test_random_shape(cfg):
    print(cfg, flush=True)
    inp = make_inputs(cfg, device=DEV)
    dy, daux = make_upstream(cfg, device=DEV)
    x, wg, u = inp.host_f64()
    want = orb.moe_backward(x, wg, u, ExpertWeightsF64(inp.wi), ExpertWeightsF64(inp.wo), cfg.C,
                            f64(dy), f64(daux))
    r = want["routing"]
    g = gpu_gate(cfg, inp.x, inp.wg, inp.u)
    for k in ("expert_idx", "slot", "src_token", "fill", "c1"):
        assert np.array_equal(g[k].cpu().numpy(), r[k]), k
    got = gpu_forward_backward(cfg, inp, dy, daux)
    tol = 2e-2 if cfg.act_dtype == "bf16" else 2e-5
    assert rel_fro(f64(got["y"]), want["y"]) < tol
    assert rel_fro(f64(got["dx"]), want["dx"]) < tol
    assert rel_fro(f64(got["dwi"]), np.stack([want["dwi"][e] for e in range(cfg.E)])) < tol
    assert rel_fro(f64(got["dwo"]), np.stack([want["dwo"][e] for e in range(cfg.E)])) < tol
    # with a handful of tokens the gate gradient is a difference of a few rounded dot products
    # (ill-conditioned in bf16): checked from 16 tokens on
    if cfg.N >= 16 or cfg.act_dtype == "f32":
        assert rel_fro(f64(got["dwg"]), want["dwg"]) < tol
    for v in got.values():
        assert torch.isfinite(v.float()).all()
