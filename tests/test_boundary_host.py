"""The C-ABI library loads, exports what include/moemix.h declares, and its host-side argument checks
answer with the documented codes.  No kernel is launched here (runs without a GPU)."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2407_14417_amd import binding as mm

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def L():
    if not (ROOT / "paper_2407_14417_amd" / "libmoemix.so").exists():
        from paper_2407_14417_amd import buildlib
        buildlib.build()
    return mm.lib()


def test_every_declared_symbol_is_exported(L):
    header = (ROOT / "include" / "moemix.h").read_text()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", header))
    assert declared == set(mm.EXPORTS), declared ^ set(mm.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.moe_version() >= 1000


def _layer(d=256, f=512, E=4, k=2, gate=1, experts=None):
    ex = experts if experts is not None else (mm.CExpert * E)()
    return mm.CLayer(d, f, E, k, gate, None, ex), ex


def test_workspace_bytes_is_monotone_and_rejects_nonsense(L):
    lay, _ = _layer()
    a = L.moe_workspace_bytes(ctypes.byref(lay), 1)
    b = L.moe_workspace_bytes(ctypes.byref(lay), 16)
    assert 0 < a < b and a % 256 == 0 and b % 256 == 0
    # at least the hidden rows and the expert outputs must fit
    assert b >= 16 * 2 * 512 * 2 + 16 * 2 * 256 * 4
    assert L.moe_workspace_bytes(ctypes.byref(lay), 0) == 0
    assert L.moe_workspace_bytes(None, 4) == 0


@pytest.mark.parametrize("kwargs,code", [
    (dict(d=250), mm.MOE_ESHAPE), (dict(f=100), mm.MOE_ESHAPE), (dict(E=33), mm.MOE_ESHAPE),
    (dict(k=5), mm.MOE_ESHAPE), (dict(k=0), mm.MOE_ESHAPE), (dict(gate=None), mm.MOE_EINVAL),
])
def test_bad_layers_are_rejected_on_the_host(L, kwargs, code):
    E = kwargs.get("E", 4)
    lay, _ = _layer(**{**kwargs, "experts": (mm.CExpert * max(E, 1))()})
    assert L.moe_route(ctypes.byref(lay), 1, 1, 1, 1, None) == code
    assert L.moe_last_error()
    assert L.moe_layer_forward(ctypes.byref(lay), 1, 1, 1, None, None, 256, 1 << 30, None) == code


def test_misaligned_matrices_are_rejected_on_the_host(L):
    """Weights, scales and zeros are read with 128-bit loads: a resident expert whose pointers are not 16-byte
    aligned is refused before any launch."""
    ex = (mm.CExpert * 4)()
    for e in range(4):
        ex[e].prec, ex[e].resident = mm.PREC_FP16, 1
        for m in (ex[e].w1, ex[e].w3, ex[e].w2):
            m.data = 4096
    lay, _ = _layer(experts=ex)
    assert L.moe_workspace_bytes(ctypes.byref(lay), 4) > 0
    ex[2].w3.data = 4096 + 8
    assert L.moe_route(ctypes.byref(lay), 1, 1, 1, 1, None) == mm.MOE_EINVAL
    assert b"16-byte aligned" in L.moe_last_error()
    ex[2].w3.data = 4096
    ex[1].prec = mm.PREC_INT4G64
    for m in (ex[1].w1, ex[1].w3, ex[1].w2):
        m.scale, m.zero = 8192, 8192 + 2
    assert L.moe_route(ctypes.byref(lay), 1, 1, 1, 1, None) == mm.MOE_EINVAL


def test_null_and_size_arguments(L):
    lay, _ = _layer()
    assert L.moe_route(ctypes.byref(lay), None, 1, 1, 1, None) == mm.MOE_EINVAL
    assert L.moe_route(ctypes.byref(lay), 1, 0, 1, 1, None) == mm.MOE_ESHAPE
    assert L.moe_layer_forward(ctypes.byref(lay), 256, 4, 256, None, None, None, 0, None) == mm.MOE_EWORKSPACE
    assert L.moe_layer_forward(ctypes.byref(lay), 256, 4, 256, None, None, 256, 1024, None) == mm.MOE_EWORKSPACE
    assert L.moe_layer_forward(ctypes.byref(lay), 256, 4, 256, None, None, 257, 1 << 30, None) == mm.MOE_EWORKSPACE
    assert b"needed" in L.moe_last_error() or b"aligned" in L.moe_last_error()
    assert L.moe_dequant_int4(None, 1, 64, 1, None) == mm.MOE_EINVAL
    m = mm.CMat(1, 1, 1)
    assert L.moe_dequant_int4(ctypes.byref(m), 4, 96, 1, None) == mm.MOE_ESHAPE
    assert L.moe_quantize_int4(1, 4, 100, 1, 1, 1, None) == mm.MOE_ESHAPE
    assert L.moe_synth_fill_f16(None, 8, 0, 0, 0, 1.0, 0, None) == mm.MOE_EINVAL
    assert L.moe_synth_fill_f16(1, 8, 0, 0, 0, 1.0, 7, None) == mm.MOE_EINVAL


def test_explicit_non_resident_expert_fails_on_the_host(L):
    ex = (mm.CExpert * 4)()
    for e in ex:
        e.prec, e.resident = mm.PREC_FP16, 1
        e.w1.data = e.w3.data = e.w2.data = 256
    ex[2].resident = 0
    lay, _ = _layer(experts=ex)
    assert L.moe_expert_ffn_mixed(ctypes.byref(lay), 2, 256, 1, 256, 256, 1 << 30, None) == mm.MOE_ENOTRESIDENT
    assert L.moe_expert_ffn_mixed(ctypes.byref(lay), 9, 256, 1, 256, 256, 1 << 30, None) == mm.MOE_EINVAL
    ex[1].prec = mm.PREC_INT4G64          # 4-bit expert without scale/zero
    assert L.moe_route(ctypes.byref(lay), 256, 1, 256, 256, None) == mm.MOE_EINVAL
