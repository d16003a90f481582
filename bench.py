"""Benchmark of the MoE-layer forward pass on one MI355X.

A step is one call of the layer (gating, dispatch, both expert GEMMs, combine)
over one batch of seeded synthetic input that is already resident in HBM; the gate
weights' packed operand form is built once before (moe_gate_pack), the time of
moe_forward, which packs them in every call, is reported beside it.  The
workload is the paper-shaped layer share (G=8, S=4096, M=1024, H=8192, E=32,
C=256, bf16 experts, fp32 gate) unless --config names another one.

Prints ONE JSON line: tokens/s of the whole layer, the roofline of the dominant
kernel (the slower of the two grouped expert GEMMs) measured with HIP events
recorded inside the timed region on the kernels' own stream, per-stage times, and
the fp64 CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

STAGES = ["gate", "dispatch", "expert_gemm1", "expert_gemm2", "combine"]


def measured_traffic(cfg_name):
    """HBM-side bytes per launch of each stage from the committed rocprofv3 --pmc summary of this
    workload (profiles/moe_layer_<workload>_hbm_traffic.md: FETCH_SIZE and WRITE_SIZE in KiB per
    dispatch, scaled by the factors a plain copy of known size gives in the same runs).  Returns
    ({stage: bytes}, source) or ({}, None) when there is no summary; the source string names the
    file and the date it states, so a figure can never outlive its profile unnoticed."""
    import re
    path = os.path.join(ROOT, "profiles", f"moe_layer_{cfg_name}_hbm_traffic.md")
    if not os.path.exists(path):
        return {}, None
    text = open(path).read()
    fs = re.search(r"FETCH_SIZE is scaled by ([0-9]+(?:\.[0-9]+)?), WRITE_SIZE by ([0-9]+(?:\.[0-9]+)?)", text)
    date = re.search(r"Measured: (\S+)", text)
    if not fs:
        return {}, None
    kf, kw = float(fs.group(1)), float(fs.group(2))
    out = {}
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0].strip("`") in STAGES:
            try:
                fetch = float(cells[2].replace(" ", "").replace(",", ""))
                write = float(cells[3].replace(" ", "").replace(",", ""))
            except ValueError:
                continue
            out[cells[0].strip("`")] = (fetch * kf + write * kw) * 1024
    src = f"profiles/{os.path.basename(path)}" + (f" (measured {date.group(1)})" if date else "")
    return out, src


def cpu_baseline(cfg, inp, seconds_hint=20.0):
    """The oracle as it stands, on whole groups of the same workload (groups are
    independent, Section 2.2), as many as fit a ~10-30 s budget."""
    import numpy as np
    import torch
    from oracle import moe_oracle as orc
    from workloads import ExpertWeightsF64
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    wi, wo = ExpertWeightsF64(inp.wi), ExpertWeightsF64(inp.wo)
    x, wg, u = inp.host_f64()
    done, t_total = 0, 0.0
    for g in range(cfg.G):
        t0 = time.perf_counter()
        orc.moe_forward(x[g:g + 1], wg, u[g:g + 1], wi, wo, cfg.C)
        t_total += time.perf_counter() - t0
        done += 1
        if t_total * (done + 1) / done > seconds_hint:
            break
    toks = done * cfg.S
    return {"value": toks / t_total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{done} of {cfg.G} groups ({toks} tokens) of the same workload, whole layer, "
                      f"fp64 numpy, {t_total:.1f} s; includes widening each expert's weights to fp64"}


class PowerSampler:
    """Board power and shader clock from sysfs while a region runs (a thread polling every few
    milliseconds); says whether the card sat at its power cap, which is what sets the clock the
    MFMA-bound kernels run at.  Silent when the files are not there."""

    def __init__(self):
        import glob
        dev = sorted(glob.glob("/sys/class/drm/card*/device"))
        self.dev = dev[0] if dev else None
        hw = sorted(glob.glob(self.dev + "/hwmon/hwmon*")) if self.dev else []
        self.hw = hw[0] if hw else None
        self.samples, self.clocks, self._stop, self._thread = [], [], False, None

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return f.read()
        except OSError:
            return None

    def _poll(self):
        while not self._stop:
            p = self._read(self.hw + "/power1_input") if self.hw else None
            if p:
                self.samples.append(int(p) / 1e6)
            c = self._read(self.dev + "/pp_dpm_sclk") if self.dev else None
            if c:
                cur = [ln for ln in c.splitlines() if ln.strip().endswith("*")]
                if cur:
                    self.clocks.append(int(cur[0].split(":")[1].strip().split("Mhz")[0]))
            time.sleep(0.002)

    def __enter__(self):
        import threading
        self._thread = threading.Thread(target=self._poll, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._thread.join()

    def summary(self):
        if not self.samples:
            return None
        cap = self._read(self.hw + "/power1_cap")
        half = self.samples[len(self.samples) // 2:]      # second half: past the ramp of the sensor's average
        return {"board_power_W_mean": sum(self.samples) / len(self.samples),
                "board_power_W_second_half": sum(half) / len(half),
                "board_power_W_max": max(self.samples),
                "power_cap_W": int(cap) / 1e6 if cap else None,
                "sclk_MHz_mean": sum(self.clocks) / len(self.clocks) if self.clocks else None,
                "sclk_MHz_second_half": (sum(self.clocks[len(self.clocks) // 2:]) /
                                         len(self.clocks[len(self.clocks) // 2:]) if self.clocks else None),
                "sclk_MHz_nominal": 2400, "samples": len(self.samples)}


def yardsticks(cfg, dev):
    """Context for the roofline fractions, measured in the same process on the same box: a
    plain device copy, the vendor library's square bf16 GEMM and its batched GEMMs of exactly
    the two expert-GEMM shapes (torch.bmm, random operands).  Not part of any product path."""
    import torch

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {}
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    out["device_copy_TBps"] = 2 * src.numel() / (timed(lambda: dst.copy_(src), 5) * 1e-3) / 1e12
    del src, dst
    if cfg.act_dtype == "bf16":
        a = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
        b = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
        out["vendor_gemm_8192_cubed_TFLOPs"] = 2 * 8192 ** 3 / (timed(lambda: a @ b, 5) * 1e-3) / 1e12
        del a, b
        rows = cfg.G * cfg.C
        if cfg.E * (rows * cfg.H + cfg.M * cfg.H) * 2 < 40e9:       # operands within 40 GB
            a1 = torch.randn(cfg.E, rows, cfg.M, device=dev, dtype=torch.bfloat16)
            b1 = torch.randn(cfg.E, cfg.M, cfg.H, device=dev, dtype=torch.bfloat16)
            out["vendor_bmm_gemm1_shape_ms"] = timed(lambda: torch.bmm(a1, b1), 5)
            a2 = torch.bmm(a1, b1).relu_()
            del a1, b1
            b2 = torch.randn(cfg.E, cfg.H, cfg.M, device=dev, dtype=torch.bfloat16)
            out["vendor_bmm_gemm2_shape_ms"] = timed(lambda: torch.bmm(a2, b2), 5)
            del a2, b2
    torch.cuda.empty_cache()
    return out


def time_encoder(moe, cfg, sh, inp, K, W, peak):
    """The two encoder layers around the MoE layer at the paper's attention sizes (16 heads of
    key/value dimension 128, sequences of 1024 tokens); stage times from separate timed loops
    of the staged entry points.  Not part of `value`."""
    import torch
    from workloads import make_encoder_weights
    dev = inp.x.device
    heads, d = 16, 128
    L = 1024 if cfg.N % 1024 == 0 else cfg.S
    dims = moe.EncoderDims(cfg.N // L, L, heads, d)
    A = heads * d
    w = make_encoder_weights(cfg, heads, d, device=dev)
    weights = dict(w, wg=inp.wg, wi=inp.wi, wo=inp.wo)
    y = torch.empty_like(inp.x)
    t = torch.empty_like(inp.x)
    aux = torch.empty(cfg.G, dtype=torch.float32, device=dev)
    ws = torch.empty(moe.moe_encoder_workspace_bytes(sh, dims), dtype=torch.uint8, device=dev)
    aws = torch.empty(moe.moe_attention_workspace_bytes(sh, dims), dtype=torch.uint8, device=dev)
    hden = torch.empty((cfg.G, cfg.S, cfg.H), dtype=inp.x.dtype, device=dev)

    def timed(fn):
        for _ in range(W):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(K):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / K

    pair = timed(lambda: moe.moe_encoder_pair_forward(sh, dims, inp.x, weights, inp.u, y, aux, ws))
    att = timed(lambda: moe.moe_self_attention(sh, dims, inp.x, w["wqkv"][0], w["wo_att"][0], t, aws))
    ffn = timed(lambda: moe.moe_dense_ffn(sh, inp.x, w["w1"], w["w2"], hden, t))
    ln = timed(lambda: moe.moe_add_layer_norm(sh, inp.x, t, w["ln_gamma"][0], w["ln_beta"][0], y, t))
    att_flops = 2.0 * cfg.N * cfg.M * 3 * A + 2.0 * cfg.N * A * cfg.M + 4.0 * cfg.N * L * A
    # training: forward that keeps the activations, then the backward pass of both layers
    from workloads import make_upstream
    dy, daux = make_upstream(cfg, device=dev)
    del ws, aws, hden
    fws = torch.empty(moe.moe_encoder_train_workspace_bytes(sh, dims), dtype=torch.uint8, device=dev)
    bws = torch.empty(moe.moe_encoder_backward_workspace_bytes(sh, dims), dtype=torch.uint8, device=dev)
    grads = {k: ([torch.empty_like(v) for v in weights[k]] if isinstance(weights[k], (list, tuple))
                 else torch.empty_like(weights[k])) for k in weights}
    dx = torch.empty_like(inp.x)
    train_fwd = timed(lambda: moe.moe_encoder_pair_forward_train(sh, dims, inp.x, weights, inp.u, y, aux, fws))
    bwd = timed(lambda: moe.moe_encoder_pair_backward(sh, dims, inp.x, weights, dy, daux, fws, dx, grads, bws))
    return {"ms_per_step": pair, "tokens_per_s": cfg.N / (pair * 1e-3),
            "train_forward_ms_per_step": train_fwd, "backward_ms_per_step": bwd,
            "train_tokens_per_s": cfg.N / ((train_fwd + bwd) * 1e-3),
            "dims": {"sequences": dims.B, "length": L, "heads": heads, "d": d},
            "self_attention_ms": att, "self_attention_mfma_frac": att_flops / (att * 1e-3) / 1e12 / peak,
            "dense_ffn_ms": ffn, "dense_ffn_mfma_frac": 4.0 * cfg.N * cfg.M * cfg.H / (ffn * 1e-3) / 1e12 / peak,
            "add_layer_norm_ms": ln,
            "add_layer_norm_hbm_frac": 4.0 * cfg.N * cfg.M * inp.x.element_size() / (ln * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "note": "x -> attention + dense FFN layer -> attention + MoE layer, forward and backward; not part of value"}


def time_backward(moe, cfg, sh, inp, ws, y, aux, K, W, kept_rows, peak):
    """Backward pass of the same layer (not part of `value`): K calls of moe_backward_events
    after one moe_forward_train, stage times from HIP events on the kernels' stream."""
    import torch
    from workloads import make_upstream
    dev = inp.x.device
    dy, daux = make_upstream(cfg, device=dev)
    dx = torch.empty_like(inp.x)
    dwg = torch.empty_like(inp.wg)
    dwi, dwo = torch.empty_like(inp.wi), torch.empty_like(inp.wo)
    bws = torch.empty(moe.moe_backward_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_forward_train(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws)
    n_ev = moe.binding.BACKWARD_EVENTS
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(K)]
    for evs in events:
        for e in evs:
            e.record()
    args = (sh, inp.x, inp.wg, inp.wi, inp.wo, dy, daux, ws, dx, dwg, dwi, dwo, bws)
    for _ in range(W):
        moe.moe_backward(*args)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        moe.moe_backward_events(*args, events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    names = ["combine_bwd", "dgrad2_dh", "wgrad2_dwo", "dgrad1_dbuf", "wgrad1_dwi", "gate_bwd_dwg", "dx"]
    stage_ms = {n: sum(events[k][i].elapsed_time(events[k][i + 1]) for k in range(K)) / K
                for i, n in enumerate(names)}
    gemm_ms = sum(stage_ms[n] for n in names[1:5])
    flops = 4 * 2.0 * cfg.M * cfg.H * kept_rows          # four GEMMs over the kept rows
    return {"ms_per_step": (t1 - t0) * 1e3 / K, "stages_ms": stage_ms,
            "gemm_mfma_frac": flops / (gemm_ms * 1e-3) / 1e12 / peak,
            "note": "moe_backward after moe_forward_train on the same inputs; not part of value"}


def time_f32_layer(moe, cfg, K, W):
    """The same workload with fp32 activations and expert weights (the precision the paper
    trained in, Section 4): forward and backward of the layer, whose expert GEMMs run as fp32
    MFMA.  Not part of `value`."""
    import dataclasses
    import torch
    from workloads import make_inputs, make_upstream
    dev = "cuda:0"
    c32 = dataclasses.replace(cfg, name=cfg.name + "_f32", act_dtype="f32")
    inp = make_inputs(c32, device=dev)
    sh = moe.MoEShape(c32.G, c32.S, c32.M, c32.H, c32.E, c32.C, "f32")
    y = torch.empty_like(inp.x)
    aux = torch.empty(c32.G, dtype=torch.float32, device=dev)
    ws = torch.empty(moe.moe_train_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(moe.binding.FORWARD_EVENTS)]
    for e in evs:
        e.record()
    for _ in range(W):
        moe.moe_forward(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws)
    torch.cuda.synchronize()
    names = ["gate", "dispatch", "expert_gemm1", "expert_gemm2", "combine"]
    stage = {n: 0.0 for n in names}
    t0 = time.perf_counter()
    for _ in range(K):
        moe.moe_forward_events(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws, evs)
    torch.cuda.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / K
    for i, n in enumerate(names):                  # stage times of the last call
        stage[n] = evs[i].elapsed_time(evs[i + 1])
    padded = c32.E * c32.G * c32.C
    gemm_ms = stage["expert_gemm1"] + stage["expert_gemm2"]
    dy, daux = make_upstream(c32, device=dev)
    dx, dwg = torch.empty_like(inp.x), torch.empty_like(inp.wg)
    dwi, dwo = torch.empty_like(inp.wi), torch.empty_like(inp.wo)
    bws = torch.empty(moe.moe_backward_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_forward_train(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws)
    args = (sh, inp.x, inp.wg, inp.wi, inp.wo, dy, daux, ws, dx, dwg, dwi, dwo, bws)
    moe.moe_backward(*args)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        moe.moe_backward(*args)
    torch.cuda.synchronize()
    bwd_ms = (time.perf_counter() - t0) * 1e3 / K
    return {"forward_ms_per_step": fwd_ms, "forward_tokens_per_s": c32.N / (fwd_ms * 1e-3),
            "stages_ms": stage, "backward_ms_per_step": bwd_ms,
            # every slot is multiplied (no skipping of empty rows), so padded rows are the work
            "ffn_mfma_f32_frac_padded_rows": 4.0 * c32.M * c32.H * padded / (gemm_ms * 1e-3) / 1e12 / PEAK_F32_TFLOPS,
            "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s",
            "note": "same workload in fp32 (v_mfma_f32_32x32x2_f32); not part of value"}


def gemm_rows(moe, cfg, sh, fill):
    """Rows per GEMM launch: occupied slots (the algorithmic work), every slot of the buffer, and
    the rows the launches really multiply (whole 256-row tiles of each expert's packed rows when
    the layer packs them, else every slot)."""
    import torch
    kept = int(fill.sum().item())
    padded = cfg.E * cfg.G * cfg.C
    multiplied = padded
    if moe.moe_forward_fuses_dispatch(sh) and hasattr(moe, "moe_forward_packs_rows") \
            and moe.moe_forward_packs_rows(sh):
        per_e = fill.sum(dim=0)
        multiplied = int((((per_e + 255) // 256) * 256).sum().item())
    return kept, padded, multiplied


def measure_forward(moe, cfg, inp, K, W, power=False):
    """K timed calls of moe_forward_events after W warm-up calls of moe_forward; stage times from
    HIP events recorded inside the timed calls on the kernels' own stream."""
    import torch
    dev = inp.x.device
    sh = moe.MoEShape(cfg.G, cfg.S, cfg.M, cfg.H, cfg.E, cfg.C, cfg.act_dtype)
    y = torch.empty_like(inp.x)
    aux = torch.empty(cfg.G, dtype=torch.float32, device=dev)
    # (sized for the training forward, which the backward measurement runs in the same buffer)
    ws = torch.empty(moe.moe_train_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    # occupied expert rows (algorithmic work of the GEMMs counts kept rows only)
    i32 = dict(dtype=torch.int32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    fill = torch.empty((cfg.G, cfg.E), **i32)
    gws = torch.empty(moe.moe_gate_workspace_bytes(sh), dtype=torch.uint8, device=dev)
    moe.moe_gate(sh, inp.x, inp.wg, inp.u, torch.empty((cfg.G, cfg.S, 2), **i32),
                 torch.empty((cfg.G, cfg.S, 2), **i32), torch.empty((cfg.G, cfg.S, 2), **f32), fill,
                 torch.empty((cfg.E, cfg.G, cfg.C), **i32), torch.empty((cfg.G, cfg.E), **i32),
                 torch.empty((cfg.G, cfg.E), **f32), torch.empty((cfg.G,), **f32), None, gws)
    torch.cuda.synchronize()
    kept_rows, padded_rows, multiplied_rows = gemm_rows(moe, cfg, sh, fill)
    del gws

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(moe.binding.FORWARD_EVENTS)]
              for _ in range(K)]
    for evs in events:                      # create the handles
        for e in evs:
            e.record()
    # the gate weights are a parameter: their MFMA operand form is built once, outside the timed
    # region (moe_gate_pack), as a server or a training step would after each weight update
    nbytes = moe.moe_gate_pack_bytes(sh)
    wgp = torch.empty(nbytes, dtype=torch.uint8, device=dev) if nbytes else None
    moe.moe_gate_pack(sh, inp.wg, wgp)
    for _ in range(W):
        moe.moe_forward_prepacked(sh, inp.x, inp.wg, wgp, inp.u, inp.wi, inp.wo, y, aux, ws)
    torch.cuda.synchronize()
    # the timed region: K calls of the layer with the six stage marks recorded between the
    # kernels, on the kernels' stream
    t0 = time.perf_counter()
    for k in range(K):
        moe.moe_forward_prepacked(sh, inp.x, inp.wg, wgp, inp.u, inp.wi, inp.wo, y, aux, ws, events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # the same K calls without the marks (an event record leaves a gap of about a microsecond
    # between two kernels)
    v0 = time.perf_counter()
    for k in range(K):
        moe.moe_forward_prepacked(sh, inp.x, inp.wg, wgp, inp.u, inp.wi, inp.wo, y, aux, ws)
    torch.cuda.synchronize()
    plain_ms = (time.perf_counter() - v0) * 1e3 / K
    # and with wg packed inside every call (moe_forward)
    u0 = time.perf_counter()
    for k in range(K):
        moe.moe_forward(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws)
    torch.cuda.synchronize()
    repack_ms = (time.perf_counter() - u0) * 1e3 / K
    pw = None
    if power:
        # power / clock state under this load: a separate, longer, untimed run of the same calls
        with PowerSampler() as ps:
            for _ in range(max(K, int(1500.0 / max((t1 - t0) * 1e3 / K, 0.05)))):      # about 1.5 s
                moe.moe_forward_prepacked(sh, inp.x, inp.wg, wgp, inp.u, inp.wi, inp.wo, y, aux, ws)
            torch.cuda.synchronize()
        pw = ps.summary()
    per_call = {n: sorted(events[k][i].elapsed_time(events[k][i + 1]) for k in range(K))
                for i, n in enumerate(STAGES)}
    return {"sh": sh, "ws": ws, "y": y, "aux": aux, "wall_s": t1 - t0, "power": pw,
            "ms_per_step_packing_wg_in_call": repack_ms, "ms_per_step_without_stage_events": plain_ms,
            "kept_rows": kept_rows, "padded_rows": padded_rows, "multiplied_rows": multiplied_rows,
            "stage_ms": {n: sum(v) / K for n, v in per_call.items()},
            "stage_median": {n: v[K // 2] for n, v in per_call.items()},
            "stage_min": {n: v[0] for n, v in per_call.items()}}


def stage_rooflines(moe, cfg, m):
    """Per stage: algorithmic flops and bytes of one launch, which roofline binds it (the larger of
    flops / MFMA peak and bytes / HBM peak) and the achieved fraction of each."""
    elt = 2 if cfg.act_dtype == "bf16" else 4
    peak = PEAK_BF16_TFLOPS if cfg.act_dtype == "bf16" else PEAK_F32_TFLOPS
    kept, N, row_b = m["kept_rows"], cfg.N, cfg.M * elt
    w_bytes = cfg.E * cfg.M * cfg.H * elt
    work = {  # stage: (flops, bytes) of one launch; GEMM work counts the occupied rows only
        # the gate's logits run as three bf16 MFMA passes (wg in three exact bf16 terms)
        "gate": (2.0 * (3 if cfg.act_dtype == "bf16" else 1) * N * cfg.M * cfg.E,
                 N * row_b + cfg.M * cfg.E * 4 + N * 28),
        "dispatch": (0.0, (kept + m["padded_rows"]) * row_b),     # read kept rows, write every slot
        "expert_gemm1": (2.0 * cfg.M * cfg.H * kept, w_bytes + kept * row_b + kept * cfg.H * elt),
        "expert_gemm2": (2.0 * cfg.M * cfg.H * kept, w_bytes + kept * cfg.H * elt + kept * row_b),
        "combine": (0.0, (kept + N) * row_b),
    }
    if moe.moe_forward_fuses_dispatch(m["sh"]):
        del work["dispatch"]                 # no dispatch kernel ran: the stage is an empty gap
    out = {}
    for n, (fl, by) in work.items():
        t = m["stage_ms"][n] * 1e-3
        t_mfma, t_hbm = fl / (peak * 1e12), by / (PEAK_HBM_GBS * 1e9)
        out[n] = {"ms": m["stage_ms"][n], "bound": "mfma" if t_mfma > t_hbm else "hbm",
                  "mfma_frac": fl / t / 1e12 / peak, "hbm_frac": by / t / 1e9 / PEAK_HBM_GBS,
                  "frac_of_bound": max(t_mfma, t_hbm) / t,
                  "algorithmic_GB": by / 1e9, "algorithmic_TFLOP": fl / 1e12}
    return out


def headline_roofline(moe, cfg, m, roofs):
    """The `roofline` object of the JSON line: the slower of the two expert GEMM launches, against
    the roofline that bounds it (bf16 MFMA unless the weights' HBM traffic takes longer)."""
    peak = PEAK_BF16_TFLOPS if cfg.act_dtype == "bf16" else PEAK_F32_TFLOPS
    dom = max(("expert_gemm1", "expert_gemm2"), key=lambda n: m["stage_ms"][n])
    r = roofs[dom]
    traffic, source = measured_traffic(cfg.name)
    kern = ("expert_gemm_bf16_dma_kernel" if cfg.act_dtype == "bf16" else "gemm_f32_mfma_kernel") + f" ({dom})"
    t = m["stage_ms"][dom] * 1e-3
    if r["bound"] == "mfma":
        out = {"bound": "mfma", "kernel": kern, "achieved": r["mfma_frac"] * peak, "peak": peak,
               "unit": "TFLOP/s", "frac": r["mfma_frac"]}
    else:
        out = {"bound": "hbm", "kernel": kern, "achieved": r["hbm_frac"] * PEAK_HBM_GBS,
               "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": r["hbm_frac"],
               "mfma_frac": r["mfma_frac"]}
    out["traffic"] = traffic.get(dom)
    out["traffic_source"] = source
    out["achieved_padded_rows_TFLOPs"] = 2.0 * cfg.M * cfg.H * m["padded_rows"] / t / 1e12
    out["achieved_multiplied_rows_TFLOPs"] = 2.0 * cfg.M * cfg.H * m["multiplied_rows"] / t / 1e12
    return out


def workload_name(cfg):
    return (f"{cfg.name}: G={cfg.G} S={cfg.S} M={cfg.M} H={cfg.H} E={cfg.E} C={cfg.C}, top-2, "
            f"{cfg.act_dtype} experts, fp32 gate")


def other_config(moe, name, K, W):
    """One more workload of the target list (forward only), measured like the headline one."""
    import torch
    from workloads import CONFIGS, make_inputs
    cfg = CONFIGS[name]
    inp = make_inputs(cfg, device="cuda:0")
    m = measure_forward(moe, cfg, inp, K, W)
    roofs = stage_rooflines(moe, cfg, m)
    peak = PEAK_BF16_TFLOPS if cfg.act_dtype == "bf16" else PEAK_F32_TFLOPS
    gemm_s = (m["stage_ms"]["expert_gemm1"] + m["stage_ms"]["expert_gemm2"]) * 1e-3
    out = {"workload": workload_name(cfg), "tokens": cfg.N, "steps": K, "warmup": W,
           "tokens_per_s": cfg.N * K / m["wall_s"], "ms_per_step": m["wall_s"] * 1e3 / K,
           "ms_per_step_packing_wg_in_call": m["ms_per_step_packing_wg_in_call"],
           "ms_per_step_without_stage_events": m["ms_per_step_without_stage_events"],
           "kept_rows": m["kept_rows"], "padded_rows": m["padded_rows"],
           "multiplied_rows": m["multiplied_rows"],
           "stages_ms": m["stage_ms"], "stages_ms_min": m["stage_min"],
           "ffn_mfma_frac": 4.0 * cfg.M * cfg.H * m["kept_rows"] / gemm_s / 1e12 / peak,
           "ffn_hbm_frac": (roofs["expert_gemm1"]["algorithmic_GB"] + roofs["expert_gemm2"]["algorithmic_GB"])
                           / gemm_s / PEAK_HBM_GBS,
           "stages": roofs, "roofline": headline_roofline(moe, cfg, m, roofs)}
    del inp, m
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="paper")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hip-graph", action="store_true",
                    help="also time the forward as replays of one captured HIP graph (reported as "
                         "an extra field; the metric itself is always the eager call sequence)")
    ap.add_argument("--no-encoder", action="store_true",
                    help="skip the extra measurement of the encoder layers around the MoE layer")
    ap.add_argument("--no-yardsticks", action="store_true",
                    help="skip the copy / vendor-GEMM context measurements")
    ap.add_argument("--no-f32", action="store_true",
                    help="skip the extra measurement of the same workload in fp32")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip the extra (untimed for the metric) measurement of the backward pass")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the forward measurement of the other paper-shaped workloads "
                         "(skewed, many_experts) that the default run appends")
    ap.add_argument("--only-forward", action="store_true",
                    help="the timed forward of --config and nothing else (for profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (yardstick for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters); not part of the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the layer on ONE GPU (one device's share of tokens); "
                 "the cross-device exchange is out of scope, so --gpus must be 1")
    if args.only_forward:
        args.no_cpu_baseline = args.no_encoder = args.no_yardsticks = args.no_f32 = True
        args.no_backward = args.no_other_configs = True

    import torch
    import paper_2006_16668_amd as moe
    from workloads import CONFIGS, make_inputs

    cfg = CONFIGS[args.config]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    inp = make_inputs(cfg, device=dev)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    K, W = args.steps, args.warmup
    m = measure_forward(moe, cfg, inp, K, W, power=not args.only_forward)
    sh, ws, y, aux = m["sh"], m["ws"], m["y"], m["aux"]
    kept_rows, padded_rows = m["kept_rows"], m["padded_rows"]
    stage_ms = dict(m["stage_ms"])
    roofs = stage_rooflines(moe, cfg, m)
    peak = PEAK_BF16_TFLOPS if cfg.act_dtype == "bf16" else PEAK_F32_TFLOPS
    flops_launch = 2.0 * cfg.M * cfg.H * kept_rows            # per GEMM launch, kept rows only
    if moe.moe_forward_fuses_dispatch(sh):
        stage_ms["dispatch_fused_into_gemm1"] = True
    out = {
        "metric": "MoE-layer forward tokens/sec on 1 MI355X", "value": cfg.N * K / m["wall_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": m["wall_s"] * 1e3 / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.act_dtype, "data": "synthetic",
        "config": {"workload": workload_name(cfg), "tokens": cfg.N, "kept_rows": kept_rows,
                   "padded_rows": padded_rows, "multiplied_rows": m["multiplied_rows"],
                   "entry_point": "moe_forward_prepacked (gate weights in MFMA operand form, packed once "
                                  "by moe_gate_pack outside the timed region)"},
        "ms_per_step_packing_wg_in_call": m["ms_per_step_packing_wg_in_call"],
        "ms_per_step_without_stage_events": m["ms_per_step_without_stage_events"],
        "roofline": headline_roofline(moe, cfg, m, roofs),
        "power_state": m["power"],
        "stages_ms": stage_ms, "stages_ms_median": m["stage_median"], "stages_ms_min": m["stage_min"],
        "gate_mfma_frac": roofs["gate"]["mfma_frac"] if cfg.act_dtype == "bf16" else None,
        "stages_hbm_frac": {n: roofs[n]["hbm_frac"] for n in ("gate", "dispatch", "combine") if n in roofs},
        "ffn_mfma_frac": 2 * flops_launch / ((stage_ms["expert_gemm1"] + stage_ms["expert_gemm2"]) * 1e-3)
                         / 1e12 / peak,
        "stages": roofs,
    }
    if args.hip_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            moe.moe_forward(sh, inp.x, inp.wg, inp.u, inp.wi, inp.wo, y, aux, ws)
        for _ in range(W):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(K):
            graph.replay()
        torch.cuda.synchronize()
        out["hip_graph_ms_per_step"] = (time.perf_counter() - g0) * 1e3 / K
    if not args.no_encoder and cfg.act_dtype == "bf16":
        out["encoder_pair"] = time_encoder(moe, cfg, sh, inp, K, W, peak)
    if not args.no_yardsticks:
        out["yardsticks"] = yardsticks(cfg, dev)
    if not args.no_backward:
        out["backward"] = time_backward(moe, cfg, sh, inp, ws, y, aux, K, W, kept_rows, peak)
    del ws, y, m
    torch.cuda.empty_cache()
    if not args.no_f32 and cfg.act_dtype == "bf16":
        out["f32_layer"] = time_f32_layer(moe, cfg, min(K, 5), min(W, 2))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp)
    if not args.no_other_configs:
        # the other workloads the throughput target is stated for; `value` stays the headline one
        del inp
        torch.cuda.empty_cache()
        out["other_configs"] = {n: other_config(moe, n, K, W)
                                for n in ("paper", "skewed", "many_experts") if n != cfg.name}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
