"""The C-ABI library loads and exports every symbol the header declares (no GPU)."""
import ctypes
import os
import re

import paper_2006_16668_amd as moe
from paper_2006_16668_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe_gfx950.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text))


def test_header_symbols_are_exported():
    names = _declared()
    assert names == set(binding.EXPORTS)
    lib = ctypes.CDLL(moe.library_path())
    for n in names:
        assert getattr(lib, n) is not None


def test_host_only_entry_points():
    assert moe.moe_status_string(0) == "MOE_OK"
    assert "workspace" in moe.moe_status_string(-3)
    assert "unknown" in moe.moe_status_string(-99)
    sh = moe.MoEShape(8, 4096, 1024, 8192, 32, 256, "bf16")
    rows = sh.E * sh.G * sh.C
    need = rows * (sh.M + sh.H) * 2               # out + h (the rows of buf are gathered from x)
    got = moe.moe_workspace_bytes(sh)
    assert need < got < need + (16 << 20)
    # training keeps the softmax gates and one bit per element of h for the backward pass
    extra = sh.G * sh.S * sh.E * 4 + rows * sh.H // 8
    assert got + extra <= moe.moe_train_workspace_bytes(sh) < got + extra + (1 << 20)
    assert 0 < moe.moe_gate_workspace_bytes(sh) < got
    # the paper-size bf16 layer gathers inside the first GEMM; fp32 and short rows do not
    assert moe.moe_forward_fuses_dispatch(sh) is True
    assert moe.moe_forward_fuses_dispatch(moe.MoEShape(1, 64, 32, 64, 4, 32, "f32")) is False
    assert moe.moe_forward_fuses_dispatch(moe.MoEShape(1, 600, 32, 256, 4, 256, "bf16")) is False
    # the workspace of the fp32 layer is twice as wide in its activation buffers
    assert moe.moe_workspace_bytes(moe.MoEShape(1, 64, 32, 64, 4, 32, "f32")) > 128 * (64 + 64) * 4
