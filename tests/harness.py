"""Shared helpers of the GPU parity tests: run the HIP stages through the C ABI
binding and bring the results back as numpy arrays."""
from __future__ import annotations

import numpy as np
import torch

import paper_2006_16668_amd as moe
from workloads import MoEConfig


def shape_of(cfg: MoEConfig) -> moe.MoEShape:
    return moe.MoEShape(cfg.G, cfg.S, cfg.M, cfg.H, cfg.E, cfg.C, cfg.act_dtype)


def rel_fro(got, want) -> float:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want.ravel())
    num = np.linalg.norm((got - want).ravel())
    return float(num / den) if den > 0 else float(num)


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def gpu_gate(cfg: MoEConfig, x, wg, u, want_gates=True):
    """moe_gate through the C ABI; outputs start as garbage so stale data cannot pass."""
    sh = shape_of(cfg)
    dev = x.device
    G, S, E, C = cfg.G, cfg.S, cfg.E, cfg.C
    i32 = dict(dtype=torch.int32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    r = dict(
        expert_idx=torch.full((G, S, 2), -7, **i32), slot=torch.full((G, S, 2), -7, **i32),
        weight=torch.full((G, S, 2), -7.0, **f32), fill=torch.full((G, E), -7, **i32),
        src_token=torch.full((E, G, C), -7, **i32), c1=torch.full((G, E), -7, **i32),
        mean_gate=torch.full((G, E), -7.0, **f32), aux=torch.full((G,), -7.0, **f32),
        gates=torch.full((G, S, E), -7.0, **f32) if want_gates else None)
    ws = torch.empty(moe.moe_gate_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_gate(sh, x, wg, u, r["expert_idx"], r["slot"], r["weight"], r["fill"], r["src_token"],
                 r["c1"], r["mean_gate"], r["aux"], r["gates"], ws)
    torch.cuda.synchronize()
    return r


def gpu_forward(cfg: MoEConfig, inp):
    sh = shape_of(cfg)
    dev = inp.x.device
    y = torch.full((cfg.G, cfg.S, cfg.M), float("nan"), dtype=sh.torch_dtype, device=dev)
    aux = torch.full((cfg.G,), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty(moe.moe_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_forward(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws)
    torch.cuda.synchronize()
    return y, aux


def gpu_forward_backward(cfg: MoEConfig, inp, dy, daux):
    """moe_forward_train + moe_backward through the C ABI; returns y, aux and the four gradients."""
    sh = shape_of(cfg)
    dev = inp.x.device
    dt = sh.torch_dtype
    nan = float("nan")
    y = torch.full((cfg.G, cfg.S, cfg.M), nan, dtype=dt, device=dev)
    aux = torch.full((cfg.G,), nan, dtype=torch.float32, device=dev)
    fws = torch.empty(moe.moe_train_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_forward_train(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, fws)
    dx = torch.full((cfg.G, cfg.S, cfg.M), nan, dtype=dt, device=dev)
    dwg = torch.full((cfg.M, cfg.E), nan, dtype=torch.float32, device=dev)
    dwi = torch.full((cfg.E, cfg.M, cfg.H), nan, dtype=dt, device=dev)
    dwo = torch.full((cfg.E, cfg.H, cfg.M), nan, dtype=dt, device=dev)
    bws = torch.empty(moe.moe_backward_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_backward(sh, inp.x, inp.wg, inp.wi, inp.wo, dy, daux, fws, dx, dwg, dwi, dwo, bws)
    torch.cuda.synchronize()
    return {"y": y, "aux": aux, "dx": dx, "dwg": dwg, "dwi": dwi, "dwo": dwo}


def assert_routing_equal(r, want):
    """Integer routing tensors: bit-exact."""
    for k in ("expert_idx", "slot", "fill", "src_token", "c1"):
        got = r[k].cpu().numpy().astype(np.int64)
        assert got.shape == want[k].shape, k
        bad = int((got != want[k]).sum())
        assert bad == 0, f"{k}: {bad} of {got.size} entries differ"


def assert_gate_floats_close(r, want, gates=None, rtol=1e-5):
    """fp32 gate outputs against the fp64 oracle: 1e-5 relative."""
    np.testing.assert_allclose(f64(r["weight"]), want["weight"], rtol=rtol, atol=0)
    np.testing.assert_allclose(f64(r["mean_gate"]), want["mean_gate"], rtol=rtol, atol=0)
    np.testing.assert_allclose(f64(r["aux"]), want["aux"], rtol=rtol, atol=0)
    if gates is not None and r.get("gates") is not None:
        # tiny gates: relative to the row maximum's scale is what fp32 softmax can keep
        np.testing.assert_allclose(f64(r["gates"]), gates, rtol=rtol, atol=1e-12)
