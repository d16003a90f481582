"""Seeded input generator (torch RNG on whichever device is asked for).

One call draws every input of the layer from one seed and returns torch
tensors on ``device``; the CPU oracle receives exact host copies of the same
stored values (bf16 / fp32 widened to fp64), so both sides always see identical
bits whatever device drew them.

Recipe (all configs): x ~ N(0,1); wg ~ N(0,1/M); wi ~ N(0,1/M); wo ~ N(0,1/H);
u ~ U[0,1).  Activations and expert weights are rounded to ``act_dtype`` before
anyone sees them; wg and u stay fp32.  A config with ``logit_bias_std > 0`` gets
a per-expert logit bias b_e ~ N(0, std^2) realised inside the data (the layer
has no bias input): the last input feature is the constant 1 and the last row
of wg holds b_e.

Conditioning for bit-exact routing.  Routing decisions are discontinuous in
the gate logits, and an fp32 kernel cannot be expected to take the same side
as an fp64 oracle when two candidates are closer than rounding error.  So the
generator inspects the projection z = x . wg in fp64 and
  * redraws every token row whose three largest logits are not separated by
    more than ``margin`` (z(1)-z(2) and z(2)-z(3)), and
  * redraws every uniform u that lies within ``u_margin`` of the threshold it is
    compared with, 2 / (1 + exp(z(1)-z(2))) (twice the renormalised second gate).
This only inspects a plain linear projection of the inputs; no part of the
gating algorithm (capacity, positions, losses) is evaluated here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from .configs import MoEConfig

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclass
class MoEInputs:
    cfg: MoEConfig
    x: torch.Tensor      # [G,S,M] act dtype
    wg: torch.Tensor     # [M,E]   fp32
    u: torch.Tensor      # [G,S]   fp32
    wi: torch.Tensor     # [E,M,H] act dtype
    wo: torch.Tensor     # [E,H,M] act dtype
    redrawn_rows: int = 0
    redrawn_u: int = 0

    def host_f64(self):
        """x, wg, u as float64 numpy arrays (exact widening of the stored values)."""
        return (self.x.detach().to("cpu", torch.float64).numpy(),
                self.wg.detach().to("cpu", torch.float64).numpy(),
                self.u.detach().to("cpu", torch.float64).numpy())


class ExpertWeightsF64:
    """Indexable view of an [E,a,b] tensor: item e -> float64 numpy [a,b] on the host.

    Lets a consumer widen one expert at a time instead of the whole tensor.
    """

    def __init__(self, w: torch.Tensor):
        self.w = w

    def __len__(self):
        return self.w.shape[0]

    def __getitem__(self, e: int) -> np.ndarray:
        return self.w[e].detach().to("cpu", torch.float64).numpy()


def _randn(shape, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def _logit_stats(x2d, wg, chunk=16384):
    """Per token: z(1)-z(2), z(2)-z(3) (inf when E<3) in fp64."""
    wg64 = wg.to(torch.float64)
    gaps12, gaps23 = [], []
    k = min(3, wg.shape[1])
    for i in range(0, x2d.shape[0], chunk):
        z = x2d[i:i + chunk].to(torch.float64) @ wg64
        top = torch.topk(z, k, dim=-1).values
        gaps12.append(top[:, 0] - top[:, 1])
        gaps23.append(top[:, 1] - top[:, 2] if k == 3
                      else torch.full_like(top[:, 0], float("inf")))
    return torch.cat(gaps12), torch.cat(gaps23)


def make_inputs(cfg: MoEConfig, device="cpu", margin=1e-3, u_margin=1e-4,
                condition=True, max_rounds=64, with_experts=True) -> MoEInputs:
    """Draw all inputs of ``cfg`` from ``cfg.seed`` on ``device``.

    ``with_experts=False`` leaves wi / wo as None (gating-only consumers); the
    gating inputs are the same either way because they are drawn first.
    """
    device = torch.device(device)
    dt = _TORCH_DTYPE[cfg.act_dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed)
    G, S, M, H, E = cfg.G, cfg.S, cfg.M, cfg.H, cfg.E
    N = G * S

    wg = _randn((M, E), gen, device) / float(np.sqrt(M))
    biased = cfg.logit_bias_std > 0
    if biased:
        wg[M - 1] = _randn((E,), gen, device) * cfg.logit_bias_std

    def draw_rows(n):
        r = _randn((n, M), gen, device).to(dt)
        if biased:
            r[:, M - 1] = 1.0
        return r

    x = draw_rows(N)
    u = torch.rand((N,), generator=gen, device=device, dtype=torch.float32)

    # expert weights, one expert at a time (the largest config holds 17 GB of them)
    wi = wo = None
    if with_experts:
        egen = torch.Generator(device=device)
        egen.manual_seed(cfg.seed + 7919)
        wi = torch.empty((E, M, H), device=device, dtype=dt)
        wo = torch.empty((E, H, M), device=device, dtype=dt)
        for e in range(E):
            wi[e] = (_randn((M, H), egen, device) / float(np.sqrt(M))).to(dt)
            wo[e] = (_randn((H, M), egen, device) / float(np.sqrt(H))).to(dt)

    redrawn_rows = redrawn_u = 0
    if condition:
        for _ in range(max_rounds):
            g12, g23 = _logit_stats(x, wg)
            bad = (g12 <= margin) | (g23 <= margin)
            nbad = int(bad.sum())
            if nbad == 0:
                break
            x[bad] = draw_rows(nbad)
            redrawn_rows += nbad
        else:
            raise RuntimeError("margin conditioning did not converge")
        g12, _ = _logit_stats(x, wg)
        thr = 2.0 / (1.0 + torch.exp(g12))                  # fp64
        for _ in range(max_rounds):
            bad = (thr - u.to(torch.float64)).abs() <= u_margin
            nbad = int(bad.sum())
            if nbad == 0:
                break
            u[bad] = torch.rand((nbad,), generator=gen, device=device, dtype=torch.float32)
            redrawn_u += nbad
        else:
            raise RuntimeError("uniform conditioning did not converge")

    return MoEInputs(cfg, x.view(G, S, M), wg, u.view(G, S), wi, wo,
                     redrawn_rows, redrawn_u)


def make_upstream(cfg: MoEConfig, device="cpu"):
    """Upstream gradients for the backward pass: dy [G,S,M] ~ N(0,1) rounded to the
    activation type, daux [G] ~ N(0,1) fp32 (a generator of their own, seeded from cfg.seed)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed + 104729)
    dy = _randn((cfg.G, cfg.S, cfg.M), gen, device).to(_TORCH_DTYPE[cfg.act_dtype])
    daux = _randn((cfg.G,), gen, device)
    return dy, daux


def make_encoder_weights(cfg: MoEConfig, heads: int, d: int, device="cpu"):
    """Weights of the two encoder layers around the MoE layer (all but the MoE layer's own):
    layer-norm gains 1 + 0.1 N(0,1) and offsets 0.1 N(0,1) in fp32; attention and dense
    feed-forward matrices N(0, 1/fan_in) rounded to the activation type.  A generator of
    their own, seeded from cfg.seed."""
    device = torch.device(device)
    dt = _TORCH_DTYPE[cfg.act_dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed + 15485863)
    M, H, A = cfg.M, cfg.H, heads * d
    w = {"ln_gamma": [], "ln_beta": [], "wqkv": [], "wo_att": []}
    for _ in range(4):
        w["ln_gamma"].append(1.0 + 0.1 * _randn((M,), gen, device))
        w["ln_beta"].append(0.1 * _randn((M,), gen, device))
    for _ in range(2):
        w["wqkv"].append((_randn((M, 3 * A), gen, device) / float(np.sqrt(M))).to(dt))
        w["wo_att"].append((_randn((A, M), gen, device) / float(np.sqrt(A))).to(dt))
    w["w1"] = (_randn((M, H), gen, device) / float(np.sqrt(M))).to(dt)
    w["w2"] = (_randn((H, M), gen, device) / float(np.sqrt(H))).to(dt)
    return w
