"""Seeded synthetic inputs for the mixed-precision MoE block.

Stand-ins for what the paper's evaluation (§4.1) takes from a trained Mixtral
8x7B checkpoint and from text corpora: tensors have the model's shapes and a
stated value distribution, nothing else.  This module holds none of the MoE
arithmetic (no matmul, no softmax, no quantizer); it only maps
(seed, stream, element index) to an fp16 value, so both the CPU oracle's tests
and the HIP path's tests/bench can draw bit-identical tensors from it.  The
device-side fill kernel of the HIP library follows the same recipe.

Recipe, element ``i`` of stream ``stream`` under ``seed`` (all 64-bit wraparound)::

    mix64(z): z += 0x9E3779B97F4A7C15; z = (z ^ z>>30)*0xBF58476D1CE4E5B9;
              z = (z ^ z>>27)*0x94D049BB133111EB; return z ^ z>>31      (splitmix64)
    key      = mix64(mix64(seed) + stream)
    h0, h1   = mix64(key + 2i), mix64(key + 2i + 1)
    normal : S = sum of the eight 16-bit fields of h0 and h1; c = 2S - 8*65535
             value = fp16_rne(float32(c) * scale),  scale = fp32(sigma / sqrt((8/3)*(65536**2-1)))
    uniform: c = 2*(h0 >> 40) - (2**24 - 1)
             value = fp16_rne(float32(c) * scale),  scale = fp32(a / 2**24)

The "normal" stream is a sum of eight uniforms: exact variance sigma^2, tails
cut at about 4.9 sigma.  It needs no transcendental function, which is what
makes it bit-reproducible on any IEEE machine.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_HERE = Path(__file__).resolve().parent
_HOST_SRC = _HERE / "csrc" / "synth_host.c"
_HOST_LIB = _HERE / "libmoesynth_host.so"

# Stream ids: one per tensor kind, so tensors never share random numbers.
STREAM_X = 1
STREAM_WG = 2
STREAM_RMS = 3
STREAM_EXPERT_BASE = 1 << 20          # + ((layer*4096 + expert) * 4 + {0:w1, 1:w3, 2:w2})


def expert_stream(layer: int, expert: int, which: int) -> int:
    """Stream id of matrix ``which`` (0=w1, 1=w3, 2=w2) of ``expert`` in ``layer``."""
    return STREAM_EXPERT_BASE + ((layer * 4096 + expert) * 4 + which)


def x_stream(retry: int = 0) -> int:
    """Stream id for activations.  Token row t occupies elements [t*d, (t+1)*d);
    ``retry`` > 0 names an independent stream from which a single row is redrawn."""
    return STREAM_X + (retry << 32)


def normal_scale(sigma: float) -> np.float32:
    return np.float32(sigma / np.sqrt((8.0 / 3.0) * (65536.0 ** 2 - 1.0)))


def uniform_scale(a: float) -> np.float32:
    return np.float32(a / 2.0 ** 24)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z + np.uint64(0x9E3779B97F4A7C15)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def key_of(seed: int, stream: int) -> int:
    with np.errstate(over="ignore"):
        k = _mix64(_mix64(np.array([seed], dtype=np.uint64)) + np.uint64(stream))
    return int(k[0])


def _normal_numpy(n: int, first: int, seed: int, stream: int, scale: np.float32) -> np.ndarray:
    out = np.empty(n, dtype=np.float16)
    key = np.uint64(key_of(seed, stream))
    step = 1 << 20
    with np.errstate(over="ignore"):
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            i = np.arange(first + lo, first + hi, dtype=np.uint64)
            h0 = _mix64(key + np.uint64(2) * i)
            h1 = _mix64(key + np.uint64(2) * i + np.uint64(1))
            s = np.zeros(hi - lo, dtype=np.int64)
            for b in range(4):
                sh = np.uint64(16 * b)
                s += ((h0 >> sh) & np.uint64(0xFFFF)).astype(np.int64)
                s += ((h1 >> sh) & np.uint64(0xFFFF)).astype(np.int64)
            c = (2 * s - 8 * 65535).astype(np.float32)
            out[lo:hi] = (c * scale).astype(np.float16)
    return out


def _uniform_numpy(n: int, first: int, seed: int, stream: int, scale: np.float32) -> np.ndarray:
    out = np.empty(n, dtype=np.float16)
    key = np.uint64(key_of(seed, stream))
    step = 1 << 20
    with np.errstate(over="ignore"):
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            i = np.arange(first + lo, first + hi, dtype=np.uint64)
            h0 = _mix64(key + np.uint64(2) * i)
            c = (2 * (h0 >> np.uint64(40)).astype(np.int64) - ((1 << 24) - 1)).astype(np.float32)
            out[lo:hi] = (c * scale).astype(np.float16)
    return out


_host = None
_host_tried = False


def build_host_lib(force: bool = False) -> Path:
    """Compile the C accelerator of this generator (gcc, OpenMP)."""
    if force or not _HOST_LIB.exists() or _HOST_LIB.stat().st_mtime < _HOST_SRC.stat().st_mtime:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", str(_HOST_LIB), str(_HOST_SRC)])
    return _HOST_LIB


def _host_lib():
    """The C accelerator if it can be had; None means the numpy path is used."""
    global _host, _host_tried
    if _host_tried:
        return _host
    _host_tried = True
    if os.environ.get("MOEMIX_SYNTH_NUMPY") == "1":
        return None
    try:
        lib = ctypes.CDLL(str(build_host_lib()))
    except (OSError, subprocess.CalledProcessError):
        return None
    for name in ("synth_fill_normal_f16", "synth_fill_uniform_f16"):
        fn = getattr(lib, name)
        fn.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_uint64,
                       ctypes.c_uint64, ctypes.c_float]
        fn.restype = None
    _host = lib
    return lib


def _fill(kind: str, shape, seed: int, stream: int, scale: np.float32, first: int, use_numpy: bool) -> np.ndarray:
    n = int(np.prod(shape))
    lib = None if use_numpy else _host_lib()
    if lib is None:
        flat = (_normal_numpy if kind == "normal" else _uniform_numpy)(n, first, seed, stream, scale)
    else:
        flat = np.empty(n, dtype=np.float16)
        fn = lib.synth_fill_normal_f16 if kind == "normal" else lib.synth_fill_uniform_f16
        fn(flat.ctypes.data, n, first, seed, stream, float(scale))
    return flat.reshape(shape)


def normal_f16(shape, sigma: float, seed: int, stream: int, first: int = 0, use_numpy: bool = False) -> np.ndarray:
    """fp16 tensor of the "normal" stream with standard deviation ``sigma``."""
    return _fill("normal", shape, seed, stream, normal_scale(sigma), first, use_numpy)


def uniform_f16(shape, a: float, seed: int, stream: int, first: int = 0, use_numpy: bool = False) -> np.ndarray:
    """fp16 tensor of the uniform stream on (-a, a)."""
    return _fill("uniform", shape, seed, stream, uniform_scale(a), first, use_numpy)


def precision_mask(n_experts_total: int, n_int4: int, seed: int) -> np.ndarray:
    """Seeded random choice of which experts are 4-bit (paper §3: the quantized
    attribute is assigned to experts at random).  Returns uint8 [n_experts_total],
    1 = 4-bit.  Fisher-Yates shuffle of 0..n-1 driven by the mix64 stream; the
    first ``n_int4`` entries of the shuffled order are quantized."""
    order = list(range(n_experts_total))
    key = key_of(seed, 0x5EED_0A5C)
    with np.errstate(over="ignore"):
        r = _mix64(np.uint64(key) + np.arange(n_experts_total, dtype=np.uint64))
    for i in range(n_experts_total - 1, 0, -1):
        j = int(r[i] % np.uint64(i + 1))
        order[i], order[j] = order[j], order[i]
    mask = np.zeros(n_experts_total, dtype=np.uint8)
    mask[order[:n_int4]] = 1
    return mask


def zipf_bias(n_experts: int, s: float = 1.2) -> np.ndarray:
    """Per-expert logit offsets ln(p_e), p_e proportional to (e+1)^-s, as fp32.
    Workload shaping for the skewed prefill configuration, not method arithmetic."""
    p = np.arange(1, n_experts + 1, dtype=np.float64) ** (-s)
    p /= p.sum()
    return np.log(p).astype(np.float32)
