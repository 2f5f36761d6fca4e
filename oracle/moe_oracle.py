"""ctypes front end of the CPU oracle (``moe_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
benchmark's cpu_baseline leg import this module.  It marshals numpy arrays to
the C functions and nothing else; all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import subprocess
from dataclasses import dataclass
from pathlib import Path
from typing import List, Optional, Sequence

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "moe_oracle.c"
_LIB = _HERE / "libmoe_oracle.so"
GROUP = 64


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP over independent rows, no fast-math, no FMA contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                               "-o", str(_LIB), str(_SRC), "-lm"])
    return _LIB


class _Mat(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("zero", ctypes.c_void_p)]


class _Expert(ctypes.Structure):
    _fields_ = [("prec_int4", ctypes.c_int), ("resident", ctypes.c_int), ("w1", _Mat), ("w3", _Mat), ("w2", _Mat)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(str(build()))
        vp, i32, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        L.orc_half_to_float.argtypes = [ctypes.c_uint16]
        L.orc_half_to_float.restype = ctypes.c_float
        L.orc_float_to_half.argtypes = [ctypes.c_float]
        L.orc_float_to_half.restype = ctypes.c_uint16
        L.orc_double_to_half.argtypes = [f64]
        L.orc_double_to_half.restype = ctypes.c_uint16
        L.orc_quantize_int4.argtypes = [vp, i32, i32, vp, vp, vp]
        L.orc_dequant_int4.argtypes = [vp, vp, vp, i32, i32, vp]
        L.orc_quantize_int8.argtypes = [vp, i32, i32, vp, vp, vp]
        L.orc_dequant_int8.argtypes = [vp, vp, vp, i32, i32, vp]
        L.orc_route.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, vp, vp]
        L.orc_permute.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.orc_expert_ffn.argtypes = [i32, ctypes.POINTER(_Mat), ctypes.POINTER(_Mat), ctypes.POINTER(_Mat),
                                     vp, i32, i32, i32, vp, vp]
        L.orc_layer_forward.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, ctypes.POINTER(_Expert), vp, vp, vp]
        L.orc_rmsnorm.argtypes = [vp, vp, i32, i32, f64, vp]
        L.orc_rmsnorm.restype = None
        L.orc_residual_add.argtypes = [vp, vp, i32, i32]
        L.orc_residual_add.restype = None
        L.orc_chain_layer.argtypes = [vp, i32, i32, i32, i32, i32, vp, f64, vp, vp, ctypes.POINTER(_Expert), vp, vp, vp]
        L.orc_expert_ffn_f32.argtypes = [i32, ctypes.POINTER(_Mat), ctypes.POINTER(_Mat), ctypes.POINTER(_Mat),
                                         vp, i32, i32, i32, i32, vp, vp]
        L.orc_route_f32.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, vp]
        L.orc_layer_forward_f32.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, ctypes.POINTER(_Expert), i32, vp, vp,
                                            vp, vp]
        L.orc_chain_layer_f32.argtypes = [vp, i32, i32, i32, i32, i32, vp, ctypes.c_float, vp, vp,
                                          ctypes.POINTER(_Expert), i32, vp, vp]
        L.orc_max_threads.restype = i32
        L.orc_set_threads.argtypes = [i32]
        L.orc_set_threads.restype = None
        _lib = L
    return _lib


def _f16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


# ------------------------------------------------------------------ data holders

@dataclass
class Mat:
    """One weight matrix [out, in]: fp16 ``data``; packed uint8 ``data`` [out, in/2] + fp16 ``scale``/``zero`` (4-bit);
    or uint8 ``data`` [out, in] + fp16 ``scale``/``zero`` with ``bits`` = 8."""
    data: np.ndarray
    scale: Optional[np.ndarray] = None
    zero: Optional[np.ndarray] = None
    bits: int = 4                      # of a quantized matrix (ignored when scale is None)

    @property
    def int4(self) -> bool:
        return self.scale is not None and self.bits == 4

    @property
    def int8(self) -> bool:
        return self.scale is not None and self.bits == 8

    @property
    def prec(self) -> int:
        """Precision code of the C oracle: 0 = 16-bit, 1 = 4-bit, 2 = 8-bit."""
        return 0 if self.scale is None else (2 if self.bits == 8 else 1)

    @property
    def in_features(self) -> int:
        return self.data.shape[1] * (2 if self.int4 else 1)

    def c(self) -> _Mat:
        return _Mat(_ptr(self.data), _ptr(self.scale), _ptr(self.zero))


@dataclass
class Expert:
    w1: Mat
    w3: Mat
    w2: Mat
    resident: bool = True

    @property
    def int4(self) -> bool:
        return self.w1.int4

    @property
    def int8(self) -> bool:
        return self.w1.int8

    @property
    def prec(self) -> int:
        return self.w1.prec

    def c(self) -> _Expert:
        return _Expert(self.prec, int(self.resident), self.w1.c(), self.w3.c(), self.w2.c())


# ------------------------------------------------------------------ scalar helpers (for pins)

def half_to_float(bits: int) -> float:
    return float(lib().orc_half_to_float(bits))


def float_to_half(v: float) -> int:
    return int(lib().orc_float_to_half(v))


def double_to_half(v: float) -> int:
    return int(lib().orc_double_to_half(v))


# ------------------------------------------------------------------ format

def quantize_int4(w: np.ndarray) -> Mat:
    """fp16 [out,in] -> 4-bit Mat (asymmetric uint4, group 64 along ``in``, fp16 scale and zero)."""
    w = _f16(w)
    out, inn = w.shape
    q = np.zeros((out, inn // 2), dtype=np.uint8)
    s = np.zeros((out, inn // GROUP), dtype=np.float16)
    z = np.zeros((out, inn // GROUP), dtype=np.float16)
    rc = lib().orc_quantize_int4(w.ctypes.data, out, inn, q.ctypes.data, s.ctypes.data, z.ctypes.data)
    if rc != 0:
        raise ValueError("orc_quantize_int4: shape not a multiple of the group size")
    return Mat(q, s, z)


def quantize_int8(w: np.ndarray) -> Mat:
    """fp16 [out,in] -> 8-bit Mat (asymmetric uint8, group 64 along ``in``, fp16 scale and zero)."""
    w = _f16(w)
    out, inn = w.shape
    q = np.zeros((out, inn), dtype=np.uint8)
    s = np.zeros((out, inn // GROUP), dtype=np.float16)
    z = np.zeros((out, inn // GROUP), dtype=np.float16)
    rc = lib().orc_quantize_int8(w.ctypes.data, out, inn, q.ctypes.data, s.ctypes.data, z.ctypes.data)
    if rc != 0:
        raise ValueError("orc_quantize_int8: shape not a multiple of the group size")
    return Mat(q, s, z, bits=8)


def dequant_int8(m: Mat) -> np.ndarray:
    out, inn = m.data.shape
    w = np.zeros((out, inn), dtype=np.float16)
    rc = lib().orc_dequant_int8(m.data.ctypes.data, m.scale.ctypes.data, m.zero.ctypes.data, out, inn, w.ctypes.data)
    if rc != 0:
        raise ValueError("orc_dequant_int8: bad shape")
    return w


def dequant_int4(m: Mat) -> np.ndarray:
    out, half_in = m.data.shape
    w = np.zeros((out, half_in * 2), dtype=np.float16)
    rc = lib().orc_dequant_int4(m.data.ctypes.data, m.scale.ctypes.data, m.zero.ctypes.data, out, half_in * 2,
                                w.ctypes.data)
    if rc != 0:
        raise ValueError("orc_dequant_int4: bad shape")
    return w


# ------------------------------------------------------------------ block

def route(x: np.ndarray, wg: np.ndarray, k: int, bias: Optional[np.ndarray] = None, want_logits: bool = False):
    x, wg = _f16(x), _f16(wg)
    T, d = x.shape
    E = wg.shape[0]
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float32)
    logits = np.zeros((T, E), dtype=np.float64) if want_logits else None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    rc = lib().orc_route(x.ctypes.data, T, d, wg.ctypes.data, _ptr(bias), E, k, idx.ctypes.data, gate.ctypes.data,
                         _ptr(logits))
    if rc != 0:
        raise ValueError("orc_route: bad arguments")
    return (idx, gate, logits) if want_logits else (idx, gate)


def permute(idx: np.ndarray, E: int):
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    counts = np.zeros(E, dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    perm = np.zeros(T * k, dtype=np.int32)
    rc = lib().orc_permute(idx.ctypes.data, T, k, E, counts.ctypes.data, offsets.ctypes.data, perm.ctypes.data)
    if rc != 0:
        raise ValueError("orc_permute: expert index out of range")
    return counts, offsets, perm


def expert_ffn(e: Expert, x_rows: np.ndarray, want_h: bool = False):
    x_rows = _f16(x_rows)
    n, d = x_rows.shape
    f = e.w2.in_features
    y = np.zeros((n, d), dtype=np.float64)
    h = np.zeros((n, f), dtype=np.float64) if want_h else None
    m1, m3, m2 = e.w1.c(), e.w3.c(), e.w2.c()
    rc = lib().orc_expert_ffn(e.prec, ctypes.byref(m1), ctypes.byref(m3), ctypes.byref(m2), x_rows.ctypes.data,
                              n, d, f, y.ctypes.data, _ptr(h))
    if rc != 0:
        raise ValueError("orc_expert_ffn: bad shape")
    return (y, h) if want_h else y


def _expert_array(experts: Sequence[Expert]):
    arr = (_Expert * len(experts))()
    for i, e in enumerate(experts):
        arr[i] = e.c()
    return arr


def _d_ff(experts: Sequence[Expert]) -> int:
    """d_ff read off the first expert that is resident (placeholders of absent experts carry no shape)."""
    e = next((x for x in experts if x.resident), experts[0])
    return e.w2.in_features


def layer_forward(x: np.ndarray, wg: np.ndarray, experts: Sequence[Expert], k: int,
                  bias: Optional[np.ndarray] = None):
    """Returns (out double [T,d], idx int32 [T,k], gate fp32 [T,k]).  Raises LookupError if a routed expert is
    not resident."""
    x, wg = _f16(x), _f16(wg)
    T, d = x.shape
    E = len(experts)
    out = np.zeros((T, d), dtype=np.float64)
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    arr = _expert_array(experts)
    rc = lib().orc_layer_forward(x.ctypes.data, T, d, _d_ff(experts), E, k, wg.ctypes.data, _ptr(bias), arr,
                                 out.ctypes.data, idx.ctypes.data, gate.ctypes.data)
    if rc == -3:
        raise LookupError("a routed expert is not resident")
    if rc != 0:
        raise ValueError("orc_layer_forward: bad arguments")
    return out, idx, gate


def rmsnorm(h: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    h, g = _f16(h), _f16(g)
    T, d = h.shape
    n = np.zeros((T, d), dtype=np.float16)
    lib().orc_rmsnorm(h.ctypes.data, g.ctypes.data, T, d, eps, n.ctypes.data)
    return n


def residual_add(h: np.ndarray, moe_out: np.ndarray) -> np.ndarray:
    h = _f16(h).copy()
    moe_out = np.ascontiguousarray(moe_out, dtype=np.float64)
    T, d = h.shape
    lib().orc_residual_add(h.ctypes.data, moe_out.ctypes.data, T, d)
    return h


def chain_layer(h: np.ndarray, rms_gain: np.ndarray, eps: float, wg: np.ndarray, experts: Sequence[Expert], k: int,
                bias: Optional[np.ndarray] = None):
    """One (RMSNorm -> MoE -> residual) block.  Returns (h_new fp16, idx, gate, normed input fp16)."""
    h = _f16(h).copy()
    rms_gain, wg = _f16(rms_gain), _f16(wg)
    T, d = h.shape
    E = len(experts)
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float32)
    normed = np.zeros((T, d), dtype=np.float16)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    arr = _expert_array(experts)
    rc = lib().orc_chain_layer(h.ctypes.data, T, d, _d_ff(experts), E, k, rms_gain.ctypes.data, eps, wg.ctypes.data,
                               _ptr(bias), arr, idx.ctypes.data, gate.ctypes.data, normed.ctypes.data)
    if rc == -3:
        raise LookupError("a routed expert is not resident")
    if rc != 0:
        raise ValueError("orc_chain_layer: bad arguments")
    return h, idx, gate, normed


# ------------------------------------------------------------------ second mode: fp32 accumulators, fp16 intermediates

def expert_ffn_f32(e: Expert, x_rows: np.ndarray, exact_weights: bool = False, want_h: bool = False):
    """The expert with fp32 accumulators and the hidden row rounded to fp16.  Returns y fp32 [n,d] (and h fp16)."""
    x_rows = _f16(x_rows)
    n, d = x_rows.shape
    f = e.w2.in_features
    y = np.zeros((n, d), dtype=np.float32)
    h = np.zeros((n, f), dtype=np.float16) if want_h else None
    m1, m3, m2 = e.w1.c(), e.w3.c(), e.w2.c()
    rc = lib().orc_expert_ffn_f32(e.prec, ctypes.byref(m1), ctypes.byref(m3), ctypes.byref(m2),
                                  x_rows.ctypes.data, n, d, f, int(exact_weights), y.ctypes.data, _ptr(h))
    if rc != 0:
        raise ValueError("orc_expert_ffn_f32: bad shape")
    return (y, h) if want_h else y


def route_f32(x: np.ndarray, wg: np.ndarray, k: int, bias: Optional[np.ndarray] = None):
    x, wg = _f16(x), _f16(wg)
    T, d = x.shape
    E = wg.shape[0]
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    rc = lib().orc_route_f32(x.ctypes.data, T, d, wg.ctypes.data, _ptr(bias), E, k, idx.ctypes.data, gate.ctypes.data)
    if rc != 0:
        raise ValueError("orc_route_f32: bad arguments")
    return idx, gate


def layer_forward_f32(x: np.ndarray, wg: np.ndarray, experts: Sequence[Expert], k: int,
                      bias: Optional[np.ndarray] = None, exact_weights: bool = False,
                      residual: Optional[np.ndarray] = None):
    """The block in the second mode.  Returns (out fp16 [T,d], idx, gate)."""
    x, wg = _f16(x), _f16(wg)
    T, d = x.shape
    out = np.zeros((T, d), dtype=np.float16)
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    if residual is not None:
        residual = _f16(residual)
    arr = _expert_array(experts)
    rc = lib().orc_layer_forward_f32(x.ctypes.data, T, d, _d_ff(experts), len(experts), k, wg.ctypes.data, _ptr(bias),
                                     arr, int(exact_weights), _ptr(residual), out.ctypes.data, idx.ctypes.data,
                                     gate.ctypes.data)
    if rc == -3:
        raise LookupError("a routed expert is not resident")
    if rc != 0:
        raise ValueError("orc_layer_forward_f32: bad arguments")
    return out, idx, gate


def chain_layer_f32(h: np.ndarray, rms_gain: np.ndarray, eps: float, wg: np.ndarray, experts: Sequence[Expert], k: int,
                    bias: Optional[np.ndarray] = None, exact_weights: bool = False):
    """One (RMSNorm -> block -> residual) step in the second mode.  Returns (h_new fp16, idx, gate)."""
    h = _f16(h).copy()
    rms_gain, wg = _f16(rms_gain), _f16(wg)
    T, d = h.shape
    idx = np.zeros((T, k), dtype=np.int32)
    gate = np.zeros((T, k), dtype=np.float32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    arr = _expert_array(experts)
    rc = lib().orc_chain_layer_f32(h.ctypes.data, T, d, _d_ff(experts), len(experts), k, rms_gain.ctypes.data, eps,
                                   wg.ctypes.data, _ptr(bias), arr, int(exact_weights), idx.ctypes.data,
                                   gate.ctypes.data)
    if rc == -3:
        raise LookupError("a routed expert is not resident")
    if rc != 0:
        raise ValueError("orc_chain_layer_f32: bad arguments")
    return h, idx, gate


def max_threads() -> int:
    return int(lib().orc_max_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(n)
