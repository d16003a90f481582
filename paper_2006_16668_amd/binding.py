"""ctypes binding of libmoe_gfx950.so: argument marshalling only.

The functions have the names and argument order of the C ABI.  Tensors are torch
tensors on the GPU (torch serves as allocator and stream provider); the wrappers
check dtype / shape / contiguity, pass ``data_ptr()`` and the current stream,
and raise ``MoEError`` on a negative status.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmoe_gfx950.so"
_lib = None

MOE_F32, MOE_BF16 = 0, 1
SLOT_OVERFLOW, SLOT_NOT_SAMPLED = -1, -2

EXPORTS = ("moe_status_string", "moe_prepare", "moe_gate_workspace_bytes", "moe_workspace_bytes", "moe_train_workspace_bytes", "moe_gate",
           "moe_gate_noalloc", "moe_gate_noalloc_max_bytes", "moe_dispatch",
           "moe_gate_pack_bytes", "moe_gate_pack", "moe_gate_prepacked", "moe_forward_prepacked",
           "moe_expert_ffn_workspace_bytes", "moe_forward_packs_rows", "moe_expert_ffn", "moe_combine", "moe_forward", "moe_forward_events",
           "moe_forward_fuses_dispatch", "moe_forward_train", "moe_backward_workspace_bytes",
           "moe_backward", "moe_backward_events", "moe_add_layer_norm",
           "moe_attention_workspace_bytes", "moe_encoder_workspace_bytes", "moe_self_attention",
           "moe_dense_ffn", "moe_encoder_pair_forward", "moe_encoder_train_workspace_bytes",
           "moe_encoder_backward_workspace_bytes", "moe_encoder_pair_forward_train",
           "moe_encoder_pair_backward")
FORWARD_EVENTS = 6
BACKWARD_EVENTS = 8


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {moe_status_string(status)} ({status})")


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("G", "S", "M", "H", "E", "C", "act_dtype")]


class _EncoderDims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "L", "heads", "d")]


class _EncoderWeights(ctypes.Structure):
    _fields_ = [("ln_gamma", ctypes.c_void_p * 4), ("ln_beta", ctypes.c_void_p * 4),
                ("wqkv", ctypes.c_void_p * 2), ("wo_att", ctypes.c_void_p * 2),
                ("w1", ctypes.c_void_p), ("w2", ctypes.c_void_p), ("wg", ctypes.c_void_p),
                ("wi", ctypes.c_void_p), ("wo", ctypes.c_void_p)]


@dataclass(frozen=True)
class EncoderDims:
    """B sequences of length L (B*L == G*S), attention heads and key/value dimension d."""
    B: int
    L: int
    heads: int
    d: int

    def _c(self):
        return _EncoderDims(self.B, self.L, self.heads, self.d)


@dataclass(frozen=True)
class MoEShape:
    """G groups, S tokens per group, M model dim, H hidden dim, E experts, C capacity."""
    G: int
    S: int
    M: int
    H: int
    E: int
    C: int
    act_dtype: str = "bf16"   # "f32" | "bf16"

    @property
    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.act_dtype]

    def _c(self) -> _Config:
        return _Config(self.G, self.S, self.M, self.H, self.E, self.C,
                       {"f32": MOE_F32, "bf16": MOE_BF16}[self.act_dtype])


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library() -> ctypes.CDLL:
    """Load the HIP library (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2006_16668_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    cfgp = ctypes.POINTER(_Config)
    lib.moe_status_string.restype = ctypes.c_char_p
    lib.moe_status_string.argtypes = [i32]
    for name, args in {
        "moe_gate_workspace_bytes": [cfgp, ctypes.POINTER(sz)],
        "moe_workspace_bytes": [cfgp, ctypes.POINTER(sz)],
        "moe_train_workspace_bytes": [cfgp, ctypes.POINTER(sz)],
        "moe_forward_fuses_dispatch": [cfgp, ctypes.POINTER(i32)],
        "moe_gate": [cfgp] + [vp] * 13 + [sz, vp],
        "moe_gate_noalloc": [cfgp] + [vp] * 13,
        "moe_gate_pack_bytes": [cfgp, ctypes.POINTER(sz)],
        "moe_gate_pack": [cfgp, vp, vp, vp],
        "moe_gate_prepacked": [cfgp] + [vp] * 14 + [sz, vp],
        "moe_forward_prepacked": [cfgp] + [vp] * 9 + [sz, vp, ctypes.POINTER(ctypes.c_void_p)],
        "moe_gate_noalloc_max_bytes": [ctypes.POINTER(sz)],
        "moe_dispatch": [cfgp, vp, vp, vp, vp],
        "moe_expert_ffn": [cfgp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "moe_expert_ffn_workspace_bytes": [cfgp, ctypes.POINTER(sz)],
        "moe_forward_packs_rows": [cfgp, ctypes.POINTER(i32)],
        "moe_combine": [cfgp, vp, vp, vp, vp, vp, vp],
        "moe_forward": [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "moe_forward_events": [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp,
                               ctypes.POINTER(ctypes.c_void_p)],
        "moe_forward_train": [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "moe_add_layer_norm": [cfgp, vp, vp, vp, vp, vp, vp, vp],
        "moe_attention_workspace_bytes": [cfgp, ctypes.POINTER(_EncoderDims), ctypes.POINTER(sz)],
        "moe_encoder_workspace_bytes": [cfgp, ctypes.POINTER(_EncoderDims), ctypes.POINTER(sz)],
        "moe_self_attention": [cfgp, ctypes.POINTER(_EncoderDims), vp, vp, vp, vp, vp, sz, vp],
        "moe_dense_ffn": [cfgp, vp, vp, vp, vp, vp, vp],
        "moe_encoder_pair_forward": [cfgp, ctypes.POINTER(_EncoderDims), vp,
                                     ctypes.POINTER(_EncoderWeights), vp, vp, vp, vp, sz, vp],
        "moe_encoder_train_workspace_bytes": [cfgp, ctypes.POINTER(_EncoderDims), ctypes.POINTER(sz)],
        "moe_encoder_backward_workspace_bytes": [cfgp, ctypes.POINTER(_EncoderDims), ctypes.POINTER(sz)],
        "moe_encoder_pair_forward_train": [cfgp, ctypes.POINTER(_EncoderDims), vp,
                                           ctypes.POINTER(_EncoderWeights), vp, vp, vp, vp, sz, vp],
        "moe_encoder_pair_backward": [cfgp, ctypes.POINTER(_EncoderDims), vp,
                                      ctypes.POINTER(_EncoderWeights), vp, vp, vp, sz, vp,
                                      ctypes.POINTER(_EncoderWeights), vp, sz, vp],
        "moe_backward_workspace_bytes": [cfgp, ctypes.POINTER(sz)],
        "moe_backward": [cfgp] + [vp] * 7 + [sz] + [vp] * 5 + [sz, vp],
        "moe_backward_events": [cfgp] + [vp] * 7 + [sz] + [vp] * 5 + [sz, vp,
                                                                     ctypes.POINTER(ctypes.c_void_p)],
    }.items():
        fn = getattr(lib, name)
        fn.restype = i32
        fn.argtypes = args
    _lib = lib
    return lib


def moe_prepare():
    """One-time set-up of the current device (kernel attributes); optional."""
    lib = load_library()
    lib.moe_prepare.restype = ctypes.c_int
    lib.moe_prepare.argtypes = []
    _check(lib.moe_prepare(), "moe_prepare")


def moe_status_string(status: int) -> str:
    return load_library().moe_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise MoEError(status, where)


def _ptr(t, dtype, shape, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _ws(ws, name="ws"):
    if not isinstance(ws, torch.Tensor) or not ws.is_cuda or ws.dtype != torch.uint8 \
            or not ws.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous uint8 GPU tensor")
    return ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def moe_gate_workspace_bytes(shape: MoEShape) -> int:
    n = ctypes.c_size_t(0)
    c = shape._c()
    _check(load_library().moe_gate_workspace_bytes(ctypes.byref(c), ctypes.byref(n)),
           "moe_gate_workspace_bytes")
    return n.value


def moe_forward_fuses_dispatch(shape: MoEShape) -> bool:
    n = ctypes.c_int(0)
    c = shape._c()
    _check(load_library().moe_forward_fuses_dispatch(ctypes.byref(c), ctypes.byref(n)),
           "moe_forward_fuses_dispatch")
    return bool(n.value)


def moe_workspace_bytes(shape: MoEShape) -> int:
    n = ctypes.c_size_t(0)
    c = shape._c()
    _check(load_library().moe_workspace_bytes(ctypes.byref(c), ctypes.byref(n)),
           "moe_workspace_bytes")
    return n.value


def moe_train_workspace_bytes(shape: MoEShape) -> int:
    n = ctypes.c_size_t(0)
    c = shape._c()
    _check(load_library().moe_train_workspace_bytes(ctypes.byref(c), ctypes.byref(n)),
           "moe_train_workspace_bytes")
    return n.value


def moe_gate(shape: MoEShape, x, wg, u, expert_idx, slot, weight, fill, src_token, c1, mean_gate,
             aux, gates_opt, ws):
    G, S, M, E, C = shape.G, shape.S, shape.M, shape.E, shape.C
    i32, f32 = torch.int32, torch.float32
    c = shape._c()
    wsp, wsn = _ws(ws)
    _check(load_library().moe_gate(
        ctypes.byref(c), _ptr(x, shape.torch_dtype, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"),
        _ptr(u, f32, (G, S), "u"), _ptr(expert_idx, i32, (G, S, 2), "expert_idx"),
        _ptr(slot, i32, (G, S, 2), "slot"), _ptr(weight, f32, (G, S, 2), "weight"),
        _ptr(fill, i32, (G, E), "fill"), _ptr(src_token, i32, (E, G, C), "src_token"),
        _ptr(c1, i32, (G, E), "c1"), _ptr(mean_gate, f32, (G, E), "mean_gate"),
        _ptr(aux, f32, (G,), "aux"), _ptr(gates_opt, f32, (G, S, E), "gates_opt"),
        wsp, wsn, _stream()), "moe_gate")


def moe_gate_pack_bytes(shape: MoEShape) -> int:
    n = ctypes.c_size_t(0)
    c = shape._c()
    _check(load_library().moe_gate_pack_bytes(ctypes.byref(c), ctypes.byref(n)), "moe_gate_pack_bytes")
    return n.value


def moe_gate_pack(shape: MoEShape, wg, wg_packed):
    """wg [M,E] fp32 -> wg_packed (uint8 tensor of moe_gate_pack_bytes, or None when that is 0)."""
    c = shape._c()
    dst = _ws(wg_packed, "wg_packed")[0] if wg_packed is not None else None
    _check(load_library().moe_gate_pack(
        ctypes.byref(c), _ptr(wg, torch.float32, (shape.M, shape.E), "wg"), dst, _stream()),
        "moe_gate_pack")


def moe_gate_prepacked(shape: MoEShape, x, wg, wg_packed, u, expert_idx, slot, weight, fill, src_token,
                       c1, mean_gate, aux, gates_opt, ws):
    G, S, M, E, C = shape.G, shape.S, shape.M, shape.E, shape.C
    i32, f32 = torch.int32, torch.float32
    c = shape._c()
    wsp, wsn = _ws(ws)
    pk = _ws(wg_packed, "wg_packed")[0] if wg_packed is not None else None
    _check(load_library().moe_gate_prepacked(
        ctypes.byref(c), _ptr(x, shape.torch_dtype, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"), pk,
        _ptr(u, f32, (G, S), "u"), _ptr(expert_idx, i32, (G, S, 2), "expert_idx"),
        _ptr(slot, i32, (G, S, 2), "slot"), _ptr(weight, f32, (G, S, 2), "weight"),
        _ptr(fill, i32, (G, E), "fill"), _ptr(src_token, i32, (E, G, C), "src_token"),
        _ptr(c1, i32, (G, E), "c1"), _ptr(mean_gate, f32, (G, E), "mean_gate"),
        _ptr(aux, f32, (G,), "aux"), _ptr(gates_opt, f32, (G, S, E), "gates_opt"),
        wsp, wsn, _stream()), "moe_gate_prepacked")


def moe_forward_prepacked(shape: MoEShape, x, wg, wg_packed, u, wi, wo, y, aux, ws, events=None):
    """moe_forward (events=None) / moe_forward_events with gate weights packed by moe_gate_pack."""
    G, S, M, H, E = shape.G, shape.S, shape.M, shape.H, shape.E
    dt, f32 = shape.torch_dtype, torch.float32
    handles = None
    if events is not None:
        if len(events) != FORWARD_EVENTS:
            raise ValueError(f"need {FORWARD_EVENTS} events")
        handles = (ctypes.c_void_p * FORWARD_EVENTS)(*[ctypes.c_void_p(e.cuda_event) for e in events])
    c = shape._c()
    wsp, wsn = _ws(ws)
    pk = _ws(wg_packed, "wg_packed")[0] if wg_packed is not None else None
    _check(load_library().moe_forward_prepacked(
        ctypes.byref(c), _ptr(x, dt, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"), pk,
        _ptr(u, f32, (G, S), "u"), _ptr(wi, dt, (E, M, H), "wi"), _ptr(wo, dt, (E, H, M), "wo"),
        _ptr(y, dt, (G, S, M), "y"), _ptr(aux, f32, (G,), "aux"), wsp, wsn, _stream(), handles),
        "moe_forward_prepacked")


def moe_gate_noalloc_max_bytes() -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().moe_gate_noalloc_max_bytes(ctypes.byref(n)), "moe_gate_noalloc_max_bytes")
    return n.value


def moe_gate_noalloc(shape: MoEShape, x, wg, u, expert_idx, slot, weight, fill, src_token, c1,
                     mean_gate, aux, gates_opt):
    """moe_gate whose scratch is the library's own per-GPU array (no workspace argument)."""
    G, S, M, E, C = shape.G, shape.S, shape.M, shape.E, shape.C
    i32, f32 = torch.int32, torch.float32
    c = shape._c()
    _check(load_library().moe_gate_noalloc(
        ctypes.byref(c), _ptr(x, shape.torch_dtype, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"),
        _ptr(u, f32, (G, S), "u"), _ptr(expert_idx, i32, (G, S, 2), "expert_idx"),
        _ptr(slot, i32, (G, S, 2), "slot"), _ptr(weight, f32, (G, S, 2), "weight"),
        _ptr(fill, i32, (G, E), "fill"), _ptr(src_token, i32, (E, G, C), "src_token"),
        _ptr(c1, i32, (G, E), "c1"), _ptr(mean_gate, f32, (G, E), "mean_gate"),
        _ptr(aux, f32, (G,), "aux"), _ptr(gates_opt, f32, (G, S, E), "gates_opt"),
        _stream()), "moe_gate_noalloc")


def moe_dispatch(shape: MoEShape, x, src_token, buf):
    G, S, M, E, C = shape.G, shape.S, shape.M, shape.E, shape.C
    c = shape._c()
    _check(load_library().moe_dispatch(
        ctypes.byref(c), _ptr(x, shape.torch_dtype, (G, S, M), "x"),
        _ptr(src_token, torch.int32, (E, G, C), "src_token"),
        _ptr(buf, shape.torch_dtype, (E, G, C, M), "buf"), _stream()), "moe_dispatch")


def moe_forward_packs_rows(shape: MoEShape) -> bool:
    n = ctypes.c_int(0)
    c = shape._c()
    _check(load_library().moe_forward_packs_rows(ctypes.byref(c), ctypes.byref(n)),
           "moe_forward_packs_rows")
    return bool(n.value)


def moe_expert_ffn_workspace_bytes(shape: MoEShape) -> int:
    n = ctypes.c_size_t(0)
    c = shape._c()
    _check(load_library().moe_expert_ffn_workspace_bytes(ctypes.byref(c), ctypes.byref(n)),
           "moe_expert_ffn_workspace_bytes")
    return n.value


def moe_expert_ffn(shape: MoEShape, buf, wi, wo, h_ws, out, fill=None, ws=None):
    """Positional arguments in the order they had before ``fill`` and ``ws`` existed; the C call
    takes (cfg, buf, fill, wi, wo, h_ws, out, ws, ws_bytes, stream)."""
    G, M, H, E, C = shape.G, shape.M, shape.H, shape.E, shape.C
    dt = shape.torch_dtype
    c = shape._c()
    wsp, wsn = _ws(ws) if ws is not None else (None, ctypes.c_size_t(0))
    _check(load_library().moe_expert_ffn(
        ctypes.byref(c), _ptr(buf, dt, (E, G, C, M), "buf"), _ptr(fill, torch.int32, (G, E), "fill"),
        _ptr(wi, dt, (E, M, H), "wi"),
        _ptr(wo, dt, (E, H, M), "wo"), _ptr(h_ws, dt, (E, G, C, H), "h_ws"),
        _ptr(out, dt, (E, G, C, M), "out"), wsp, wsn, _stream()), "moe_expert_ffn")


def moe_combine(shape: MoEShape, out, expert_idx, slot, weight, y):
    G, S, M, E, C = shape.G, shape.S, shape.M, shape.E, shape.C
    dt = shape.torch_dtype
    c = shape._c()
    _check(load_library().moe_combine(
        ctypes.byref(c), _ptr(out, dt, (E, G, C, M), "out"),
        _ptr(expert_idx, torch.int32, (G, S, 2), "expert_idx"),
        _ptr(slot, torch.int32, (G, S, 2), "slot"), _ptr(weight, torch.float32, (G, S, 2), "weight"),
        _ptr(y, dt, (G, S, M), "y"), _stream()), "moe_combine")


def moe_forward(shape: MoEShape, x, wg, u, wi, wo, y, aux, ws):
    G, S, M, H, E = shape.G, shape.S, shape.M, shape.H, shape.E
    dt, f32 = shape.torch_dtype, torch.float32
    c = shape._c()
    wsp, wsn = _ws(ws)
    _check(load_library().moe_forward(
        ctypes.byref(c), _ptr(x, dt, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"),
        _ptr(u, f32, (G, S), "u"), _ptr(wi, dt, (E, M, H), "wi"), _ptr(wo, dt, (E, H, M), "wo"),
        _ptr(y, dt, (G, S, M), "y"), _ptr(aux, f32, (G,), "aux"), wsp, wsn, _stream()),
        "moe_forward")


def moe_forward_events(shape: MoEShape, x, wg, u, wi, wo, y, aux, ws, events):
    """moe_forward that records ``events`` (FORWARD_EVENTS torch.cuda.Event objects, timing
    enabled, each recorded at least once before so that its handle exists) at the stage
    boundaries, on the stream the kernels run on."""
    G, S, M, H, E = shape.G, shape.S, shape.M, shape.H, shape.E
    dt, f32 = shape.torch_dtype, torch.float32
    if len(events) != FORWARD_EVENTS:
        raise ValueError(f"need {FORWARD_EVENTS} events")
    handles = (ctypes.c_void_p * FORWARD_EVENTS)(*[ctypes.c_void_p(e.cuda_event) for e in events])
    c = shape._c()
    wsp, wsn = _ws(ws)
    _check(load_library().moe_forward_events(
        ctypes.byref(c), _ptr(x, dt, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"),
        _ptr(u, f32, (G, S), "u"), _ptr(wi, dt, (E, M, H), "wi"), _ptr(wo, dt, (E, H, M), "wo"),
        _ptr(y, dt, (G, S, M), "y"), _ptr(aux, f32, (G,), "aux"), wsp, wsn, _stream(), handles),
        "moe_forward_events")


def moe_forward_train(shape: MoEShape, x, wg, u, wi, wo, y, aux, ws):
    """moe_forward that also keeps the softmax gates in ``ws`` for moe_backward."""
    G, S, M, H, E = shape.G, shape.S, shape.M, shape.H, shape.E
    dt, f32 = shape.torch_dtype, torch.float32
    c = shape._c()
    wsp, wsn = _ws(ws)
    _check(load_library().moe_forward_train(
        ctypes.byref(c), _ptr(x, dt, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"),
        _ptr(u, f32, (G, S), "u"), _ptr(wi, dt, (E, M, H), "wi"), _ptr(wo, dt, (E, H, M), "wo"),
        _ptr(y, dt, (G, S, M), "y"), _ptr(aux, f32, (G,), "aux"), wsp, wsn, _stream()),
        "moe_forward_train")


def moe_backward_workspace_bytes(shape: MoEShape) -> int:
    n = ctypes.c_size_t(0)
    c = shape._c()
    _check(load_library().moe_backward_workspace_bytes(ctypes.byref(c), ctypes.byref(n)),
           "moe_backward_workspace_bytes")
    return n.value


def _backward_args(shape, x, wg, wi, wo, dy, daux, fwd_ws, dx, dwg, dwi, dwo, ws):
    G, S, M, H, E = shape.G, shape.S, shape.M, shape.H, shape.E
    dt, f32 = shape.torch_dtype, torch.float32
    fp, fn = _ws(fwd_ws, "fwd_ws")
    wsp, wsn = _ws(ws)
    return (_ptr(x, dt, (G, S, M), "x"), _ptr(wg, f32, (M, E), "wg"), _ptr(wi, dt, (E, M, H), "wi"),
            _ptr(wo, dt, (E, H, M), "wo"), _ptr(dy, dt, (G, S, M), "dy"), _ptr(daux, f32, (G,), "daux"),
            fp, fn, _ptr(dx, dt, (G, S, M), "dx"), _ptr(dwg, f32, (M, E), "dwg"),
            _ptr(dwi, dt, (E, M, H), "dwi"), _ptr(dwo, dt, (E, H, M), "dwo"), wsp, wsn, _stream())


def moe_backward(shape: MoEShape, x, wg, wi, wo, dy, daux, fwd_ws, dx, dwg, dwi, dwo, ws):
    """Gradients of the layer; ``fwd_ws`` is the workspace moe_forward_train has filled."""
    c = shape._c()
    _check(load_library().moe_backward(
        ctypes.byref(c), *_backward_args(shape, x, wg, wi, wo, dy, daux, fwd_ws, dx, dwg, dwi, dwo, ws)),
        "moe_backward")


def moe_backward_events(shape: MoEShape, x, wg, wi, wo, dy, daux, fwd_ws, dx, dwg, dwi, dwo, ws, events):
    """moe_backward that records BACKWARD_EVENTS torch.cuda.Event objects at its stage boundaries."""
    if len(events) != BACKWARD_EVENTS:
        raise ValueError(f"need {BACKWARD_EVENTS} events")
    handles = (ctypes.c_void_p * BACKWARD_EVENTS)(*[ctypes.c_void_p(e.cuda_event) for e in events])
    c = shape._c()
    _check(load_library().moe_backward_events(
        ctypes.byref(c), *_backward_args(shape, x, wg, wi, wo, dy, daux, fwd_ws, dx, dwg, dwi, dwo, ws),
        handles), "moe_backward_events")


# ---- encoder layers around the MoE layer
def moe_add_layer_norm(shape: MoEShape, x, delta, gamma, beta, sum_out, norm_out):
    G, S, M = shape.G, shape.S, shape.M
    dt, f32 = shape.torch_dtype, torch.float32
    c = shape._c()
    _check(load_library().moe_add_layer_norm(
        ctypes.byref(c), _ptr(x, dt, (G, S, M), "x"), _ptr(delta, dt, (G, S, M), "delta"),
        _ptr(gamma, f32, (M,), "gamma"), _ptr(beta, f32, (M,), "beta"),
        _ptr(sum_out, dt, (G, S, M), "sum_out"), _ptr(norm_out, dt, (G, S, M), "norm_out"), _stream()),
        "moe_add_layer_norm")


def _ws_query(fn_name, shape: MoEShape, dims: EncoderDims) -> int:
    n = ctypes.c_size_t(0)
    c, d = shape._c(), dims._c()
    _check(getattr(load_library(), fn_name)(ctypes.byref(c), ctypes.byref(d), ctypes.byref(n)), fn_name)
    return n.value


def moe_attention_workspace_bytes(shape: MoEShape, dims: EncoderDims) -> int:
    return _ws_query("moe_attention_workspace_bytes", shape, dims)


def moe_encoder_workspace_bytes(shape: MoEShape, dims: EncoderDims) -> int:
    return _ws_query("moe_encoder_workspace_bytes", shape, dims)


def moe_self_attention(shape: MoEShape, dims: EncoderDims, u, wqkv, wo_att, out, ws):
    G, S, M = shape.G, shape.S, shape.M
    A = dims.heads * dims.d
    dt = shape.torch_dtype
    c, d = shape._c(), dims._c()
    wsp, wsn = _ws(ws)
    _check(load_library().moe_self_attention(
        ctypes.byref(c), ctypes.byref(d), _ptr(u, dt, (G, S, M), "u"), _ptr(wqkv, dt, (M, 3 * A), "wqkv"),
        _ptr(wo_att, dt, (A, M), "wo_att"), _ptr(out, dt, (G, S, M), "out"), wsp, wsn, _stream()),
        "moe_self_attention")


def moe_dense_ffn(shape: MoEShape, u, w1, w2, h_ws, out):
    G, S, M, H = shape.G, shape.S, shape.M, shape.H
    dt = shape.torch_dtype
    c = shape._c()
    _check(load_library().moe_dense_ffn(
        ctypes.byref(c), _ptr(u, dt, (G, S, M), "u"), _ptr(w1, dt, (M, H), "w1"), _ptr(w2, dt, (H, M), "w2"),
        _ptr(h_ws, dt, (G, S, H), "h_ws"), _ptr(out, dt, (G, S, M), "out"), _stream()), "moe_dense_ffn")


def _encoder_weights(shape: MoEShape, dims: EncoderDims, weights: dict) -> _EncoderWeights:
    """The C struct of device pointers (weights, or gradients of the same shapes)."""
    M, H, E = shape.M, shape.H, shape.E
    A = dims.heads * dims.d
    dt, f32 = shape.torch_dtype, torch.float32
    w = _EncoderWeights()
    for i in range(4):
        w.ln_gamma[i] = _ptr(weights["ln_gamma"][i], f32, (M,), "ln_gamma").value
        w.ln_beta[i] = _ptr(weights["ln_beta"][i], f32, (M,), "ln_beta").value
    for i in range(2):
        w.wqkv[i] = _ptr(weights["wqkv"][i], dt, (M, 3 * A), "wqkv").value
        w.wo_att[i] = _ptr(weights["wo_att"][i], dt, (A, M), "wo_att").value
    w.w1 = _ptr(weights["w1"], dt, (M, H), "w1").value
    w.w2 = _ptr(weights["w2"], dt, (H, M), "w2").value
    w.wg = _ptr(weights["wg"], f32, (M, E), "wg").value
    w.wi = _ptr(weights["wi"], dt, (E, M, H), "wi").value
    w.wo = _ptr(weights["wo"], dt, (E, H, M), "wo").value
    return w


def _encoder_forward(fn_name, shape, dims, x, weights, u, y, aux, ws):
    G, S, M = shape.G, shape.S, shape.M
    dt, f32 = shape.torch_dtype, torch.float32
    w = _encoder_weights(shape, dims, weights)
    c, d = shape._c(), dims._c()
    wsp, wsn = _ws(ws)
    _check(getattr(load_library(), fn_name)(
        ctypes.byref(c), ctypes.byref(d), _ptr(x, dt, (G, S, M), "x"), ctypes.byref(w),
        _ptr(u, f32, (G, S), "u"), _ptr(y, dt, (G, S, M), "y"), _ptr(aux, f32, (G,), "aux"),
        wsp, wsn, _stream()), fn_name)


def moe_encoder_pair_forward(shape: MoEShape, dims: EncoderDims, x, weights: dict, u, y, aux, ws):
    """weights: ln_gamma / ln_beta (4 tensors [M] fp32 each), wqkv / wo_att (2 each), w1, w2,
    wg, wi, wo."""
    _encoder_forward("moe_encoder_pair_forward", shape, dims, x, weights, u, y, aux, ws)


def moe_encoder_train_workspace_bytes(shape: MoEShape, dims: EncoderDims) -> int:
    return _ws_query("moe_encoder_train_workspace_bytes", shape, dims)


def moe_encoder_backward_workspace_bytes(shape: MoEShape, dims: EncoderDims) -> int:
    return _ws_query("moe_encoder_backward_workspace_bytes", shape, dims)


def moe_encoder_pair_forward_train(shape: MoEShape, dims: EncoderDims, x, weights: dict, u, y, aux, ws):
    """As moe_encoder_pair_forward; ws (moe_encoder_train_workspace_bytes) keeps what
    moe_encoder_pair_backward reads."""
    _encoder_forward("moe_encoder_pair_forward_train", shape, dims, x, weights, u, y, aux, ws)


def moe_encoder_pair_backward(shape: MoEShape, dims: EncoderDims, x, weights: dict, dy, daux, fwd_ws,
                              dx, grads: dict, ws):
    """grads: a dict of output tensors with the keys and shapes of ``weights``."""
    G, S, M = shape.G, shape.S, shape.M
    dt, f32 = shape.torch_dtype, torch.float32
    w = _encoder_weights(shape, dims, weights)
    g = _encoder_weights(shape, dims, grads)
    c, d = shape._c(), dims._c()
    fwp, fwn = _ws(fwd_ws)
    wsp, wsn = _ws(ws)
    _check(load_library().moe_encoder_pair_backward(
        ctypes.byref(c), ctypes.byref(d), _ptr(x, dt, (G, S, M), "x"), ctypes.byref(w),
        _ptr(dy, dt, (G, S, M), "dy"), _ptr(daux, f32, (G,), "daux"), fwp, fwn,
        _ptr(dx, dt, (G, S, M), "dx"), ctypes.byref(g), wsp, wsn, _stream()),
        "moe_encoder_pair_backward")
