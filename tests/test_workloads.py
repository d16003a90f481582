"""The seeded input generator: determinism, conditioning, workload structure.  CPU only."""
import numpy as np
import torch

from oracle import moe_oracle as orc
from workloads import CONFIGS, make_inputs


def _gaps(x, wg):
    z = np.sort(x.reshape(-1, x.shape[-1]) @ wg, axis=-1)
    return z[:, -1] - z[:, -2], z[:, -2] - z[:, -3]


def test_same_seed_same_bits_and_other_seed_differs():
    cfg = CONFIGS["tiny"]
    a, b = make_inputs(cfg), make_inputs(cfg)
    for k in ("x", "wg", "u", "wi", "wo"):
        assert torch.equal(getattr(a, k), getattr(b, k))
    c = make_inputs(cfg.with_(seed=cfg.seed + 1))
    assert not torch.equal(a.x, c.x)
    assert a.x.dtype == torch.float32 and a.x.shape == (cfg.G, cfg.S, cfg.M)
    assert a.wi.shape == (cfg.E, cfg.M, cfg.H) and a.wo.shape == (cfg.E, cfg.H, cfg.M)


def test_conditioning_margins_hold_in_fp64():
    cfg = CONFIGS["small"].with_(H=64)          # gating inputs do not depend on H
    inp = make_inputs(cfg)
    assert inp.x.dtype == torch.bfloat16 and inp.wg.dtype == torch.float32
    x, wg, u = inp.host_f64()
    g12, g23 = _gaps(x, wg)
    assert g12.min() > 1e-3 and g23.min() > 1e-3
    thr = 2.0 / (1.0 + np.exp(g12))
    assert np.abs(thr - u.reshape(-1)).min() > 1e-4
    assert (u >= 0).all() and (u < 1).all()
    # the unconditioned draw does violate the margins somewhere: the check bites
    raw = make_inputs(cfg, condition=False)
    rx, rwg, _ = raw.host_f64()
    r12, r23 = _gaps(rx, rwg)
    assert min(r12.min(), r23.min()) <= 1e-3
    # statistics of the recipe
    assert abs(x.std() - 1.0) < 0.02 and abs(wg.std() * np.sqrt(cfg.M) - 1.0) < 0.05
    assert abs(inp.wi.float().std().item() * np.sqrt(cfg.M) - 1.0) < 0.05
    assert abs(inp.wo.float().std().item() * np.sqrt(cfg.H) - 1.0) < 0.05


def test_skewed_workload_drops_15_to_25_percent():
    cfg = CONFIGS["skewed"]
    inp = make_inputs(cfg, with_experts=False)
    x, wg, u = inp.host_f64()
    assert (x[..., -1] == 1.0).all()
    r = orc.top2_gating(orc.softmax_gates(x, wg), u, cfg.C)
    dropped = (r["slot"] == orc.SLOT_OVERFLOW).mean()
    assert 0.15 <= dropped <= 0.25, dropped


def test_balanced_workload_drops_few():
    cfg = CONFIGS["small"]
    inp = make_inputs(cfg, with_experts=False)
    x, wg, u = inp.host_f64()
    r = orc.top2_gating(orc.softmax_gates(x, wg), u, cfg.C)
    assert (r["slot"] == orc.SLOT_OVERFLOW).mean() < 0.03


def test_upstream_and_encoder_weight_generators_are_seeded():
    from workloads import make_encoder_weights, make_upstream
    cfg = CONFIGS["tiny"]
    dy1, da1 = make_upstream(cfg)
    dy2, da2 = make_upstream(cfg)
    assert dy1.shape == (cfg.G, cfg.S, cfg.M) and da1.shape == (cfg.G,)
    assert torch.equal(dy1, dy2) and torch.equal(da1, da2)
    assert not torch.equal(dy1, make_upstream(cfg.with_(seed=cfg.seed + 1))[0])
    small = CONFIGS["small"]
    assert make_upstream(small)[0].dtype == torch.bfloat16
    w1 = make_encoder_weights(small, heads=4, d=16)
    w2 = make_encoder_weights(small, heads=4, d=16)
    assert w1["wqkv"][0].shape == (small.M, 3 * 64) and w1["wo_att"][1].shape == (64, small.M)
    assert w1["w1"].shape == (small.M, small.H) and w1["w1"].dtype == torch.bfloat16
    assert w1["ln_gamma"][3].dtype == torch.float32
    for k in ("wqkv", "wo_att", "ln_gamma", "ln_beta"):
        for a, b in zip(w1[k], w2[k]):
            assert torch.equal(a, b)
    assert not torch.equal(w1["wqkv"][0], w1["wqkv"][1])          # the two attention layers differ
