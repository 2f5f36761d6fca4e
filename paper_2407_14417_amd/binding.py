"""Thin ctypes binding of ``libmoemix.so``: same names as the C-ABI in ``include/moemix.h``.

Argument marshalling only.  Tensors are ``torch`` CUDA tensors used as device
memory (``data_ptr()``) and the current torch stream is passed through; every
step of the MoE block runs inside the library's kernels.  There is no fallback:
if the library is not built, :func:`lib` raises.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from pathlib import Path
from typing import List, Optional, Sequence

_LIB_PATH = Path(__file__).resolve().parent / "libmoemix.so"

MOE_OK, MOE_EINVAL, MOE_ESHAPE, MOE_ENOTRESIDENT, MOE_EWORKSPACE, MOE_EHIP = 0, -1, -2, -3, -4, -5
PREC_FP16, PREC_INT4G64, PREC_INT8G64 = 0, 1, 2
GROUP = 64
STATUS_BAD_INDEX = 1 << 1
STATUS_NOT_RESIDENT = 1 << 3

EXPORTS = (
    "moe_workspace_bytes", "moe_route", "moe_permute", "moe_expert_ffn_mixed", "moe_layer_forward",
    "moe_chain_forward", "moe_dequant_int4", "moe_quantize_int4", "moe_synth_fill_f16", "moe_read_status",
    "moe_last_error", "moe_version", "moe_trace_kernel", "moe_plan", "moe_swap_slot_bytes", "moe_layer_forward_swap",
    "moe_stream_read", "moe_static_scratch_bytes", "moe_layer_forward_static",
    "moe_dequant_int8", "moe_quantize_int8",
)


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moemix error {code}: {msg}")
        self.code = code


class CMat(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("zero", ctypes.c_void_p)]


class CExpert(ctypes.Structure):
    _fields_ = [("prec", ctypes.c_int32), ("resident", ctypes.c_int32), ("w1", CMat), ("w3", CMat), ("w2", CMat)]


class CLayer(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("w_gate", ctypes.c_void_p), ("gate_bias", ctypes.c_void_p),
                ("experts", ctypes.POINTER(CExpert))]


class CPlanRequest(ctypes.Structure):
    _fields_ = [("mem_gpu", ctypes.c_uint64), ("size_non_expert", ctypes.c_uint64), ("size_e16", ctypes.c_uint64),
                ("size_e4", ctypes.c_uint64), ("swap_bytes", ctypes.c_uint64), ("seed", ctypes.c_uint64),
                ("num_experts", ctypes.c_int32), ("preference", ctypes.c_int32), ("num_e4", ctypes.c_int32)]


class CPlanResult(ctypes.Structure):
    _fields_ = [("num_e16", ctypes.c_int32), ("num_e4", ctypes.c_int32), ("resident_e16", ctypes.c_int32),
                ("resident_e4", ctypes.c_int32), ("bytes_resident", ctypes.c_uint64)]


class CSwap(ctypes.Structure):
    _fields_ = [("host_experts", ctypes.POINTER(CExpert)), ("swap", ctypes.c_void_p), ("slot_bytes", ctypes.c_size_t),
                ("n_slots", ctypes.c_int32), ("host_idx", ctypes.c_void_p), ("copy_stream", ctypes.c_void_p),
                ("copied_event", ctypes.c_void_p), ("computed_event", ctypes.c_void_p)]


PREFER_THROUGHPUT, PREFER_QUALITY = 0, 1

_lib = None


def lib():
    """The loaded HIP library.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise RuntimeError(f"{_LIB_PATH} is missing: run __graft_entry__.build() (hipcc, gfx950) first")
        # torch first: its HIP runtime owns the streams and the memory that are passed in, and the library
        # must bind to that same runtime instance rather than load a second one
        import torch  # noqa: F401
        L = ctypes.CDLL(str(_LIB_PATH))
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        LP = ctypes.POINTER(CLayer)
        L.moe_workspace_bytes.argtypes = [LP, i32]
        L.moe_workspace_bytes.restype = sz
        L.moe_route.argtypes = [LP, vp, i32, vp, vp, vp]
        L.moe_permute.argtypes = [LP, vp, i32, vp, vp, vp, vp, sz, vp]
        L.moe_expert_ffn_mixed.argtypes = [LP, i32, vp, i32, vp, vp, sz, vp]
        L.moe_layer_forward.argtypes = [LP, vp, i32, vp, vp, vp, vp, sz, vp]
        L.moe_chain_forward.argtypes = [LP, ctypes.POINTER(vp), i32, ctypes.c_float, vp, i32, vp, vp, sz, vp]
        L.moe_dequant_int4.argtypes = [ctypes.POINTER(CMat), i32, i32, vp, vp]
        L.moe_quantize_int4.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.moe_dequant_int8.argtypes = [ctypes.POINTER(CMat), i32, i32, vp, vp]
        L.moe_quantize_int8.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.moe_synth_fill_f16.argtypes = [vp, sz, sz, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_float, i32, vp]
        L.moe_read_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int)]
        L.moe_trace_kernel.argtypes = [i32, vp, vp]
        L.moe_plan.argtypes = [ctypes.POINTER(CPlanRequest), ctypes.POINTER(CPlanResult), vp, vp]
        L.moe_swap_slot_bytes.argtypes = [LP]
        L.moe_swap_slot_bytes.restype = sz
        L.moe_layer_forward_swap.argtypes = [LP, ctypes.POINTER(CSwap), vp, i32, vp, vp, vp, vp, sz, vp,
                                             ctypes.POINTER(ctypes.c_int32)]
        L.moe_stream_read.argtypes = [vp, sz, vp, vp]
        L.moe_static_scratch_bytes.argtypes = []
        L.moe_static_scratch_bytes.restype = sz
        L.moe_layer_forward_static.argtypes = [LP, vp, i32, vp, vp, vp, vp]
        L.moe_last_error.restype = ctypes.c_char_p
        L.moe_version.restype = i32
        for name in EXPORTS:
            if name not in ("moe_workspace_bytes", "moe_last_error", "moe_version", "moe_swap_slot_bytes",
                            "moe_static_scratch_bytes"):
                getattr(L, name).restype = i32
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != MOE_OK:
        raise MoeError(rc, lib().moe_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


# ---------------------------------------------------------------- descriptors

@dataclass
class Mat:
    """One weight matrix in device memory: fp16 ``data`` [out,in], or uint8 ``data`` [out,in/2] + fp16 scale/zero."""
    data: "torch.Tensor"
    scale: Optional["torch.Tensor"] = None
    zero: Optional["torch.Tensor"] = None

    def c(self) -> CMat:
        return CMat(_ptr(self.data), _ptr(self.scale), _ptr(self.zero))

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.data, self.scale, self.zero) if t is not None)


@dataclass
class Expert:
    prec: int
    w1: Optional[Mat]
    w3: Optional[Mat]
    w2: Optional[Mat]
    resident: bool = True

    def c(self) -> CExpert:
        null = CMat(None, None, None)
        return CExpert(self.prec, int(self.resident), self.w1.c() if self.w1 else null,
                       self.w3.c() if self.w3 else null, self.w2.c() if self.w2 else null)

    def nbytes(self) -> int:
        return sum(m.nbytes() for m in (self.w1, self.w3, self.w2) if m is not None)


class Layer:
    """Host descriptor of one MoE block; keeps the tensors alive that its device pointers name."""

    def __init__(self, d_model: int, d_ff: int, top_k: int, w_gate, experts: Sequence[Expert], gate_bias=None):
        self.d_model, self.d_ff, self.top_k = d_model, d_ff, top_k
        self.w_gate, self.gate_bias, self.experts = w_gate, gate_bias, list(experts)
        self._arr = (CExpert * len(self.experts))(*[e.c() for e in self.experts])
        self.c = CLayer(d_model, d_ff, len(self.experts), top_k, _ptr(w_gate), _ptr(gate_bias), self._arr)

    @property
    def n_experts(self) -> int:
        return len(self.experts)


def workspace_bytes(layer: Layer, n_tokens: int) -> int:
    return int(lib().moe_workspace_bytes(ctypes.byref(layer.c), n_tokens))


def alloc_workspace(layer: Layer, n_tokens: int):
    import torch
    n = workspace_bytes(layer, n_tokens)
    if n == 0:
        raise MoeError(MOE_EINVAL, "moe_workspace_bytes rejected the arguments")
    return torch.empty(n, dtype=torch.uint8, device="cuda")


# ---------------------------------------------------------------- entry points (same names as the C-ABI)

def moe_route(layer: Layer, x, topk_idx, topk_gate) -> None:
    _check(lib().moe_route(ctypes.byref(layer.c), _ptr(x), x.shape[0], _ptr(topk_idx), _ptr(topk_gate), _stream()))


def moe_permute(layer: Layer, topk_idx, counts, offsets, perm, ws) -> None:
    _check(lib().moe_permute(ctypes.byref(layer.c), _ptr(topk_idx), topk_idx.shape[0], _ptr(counts), _ptr(offsets),
                             _ptr(perm), _ptr(ws), ws.numel(), _stream()))


def moe_expert_ffn_mixed(layer: Layer, expert: int, x_rows, y, ws) -> None:
    _check(lib().moe_expert_ffn_mixed(ctypes.byref(layer.c), expert, _ptr(x_rows), x_rows.shape[0], _ptr(y), _ptr(ws),
                                      0 if ws is None else ws.numel(), _stream()))


def moe_layer_forward(layer: Layer, x, out, ws, topk_idx_out=None, topk_gate_out=None) -> None:
    _check(lib().moe_layer_forward(ctypes.byref(layer.c), _ptr(x), x.shape[0], _ptr(out), _ptr(topk_idx_out),
                                   _ptr(topk_gate_out), _ptr(ws), 0 if ws is None else ws.numel(), _stream()))


def moe_static_scratch_bytes() -> int:
    return int(lib().moe_static_scratch_bytes())


def moe_layer_forward_static(layer: Layer, x, out, topk_idx_out=None, topk_gate_out=None) -> None:
    _check(lib().moe_layer_forward_static(ctypes.byref(layer.c), _ptr(x), x.shape[0], _ptr(out), _ptr(topk_idx_out),
                                          _ptr(topk_gate_out), _stream()))


class Swap:
    """Swap space and host-side expert copies for moe_layer_forward_swap.  `host_experts[e]` is an Expert whose
    tensors are pinned host tensors (or None for experts that are resident in `layer`)."""

    def __init__(self, layer: Layer, host_experts: Sequence[Optional[Expert]], n_slots: int, n_tokens: int):
        import torch
        self.layer, self.host_experts, self.n_slots = layer, list(host_experts), n_slots
        null = CExpert(PREC_FP16, 0, CMat(None, None, None), CMat(None, None, None), CMat(None, None, None))
        self._arr = (CExpert * layer.n_experts)(*[e.c() if e is not None else null for e in self.host_experts])
        self.slot_bytes = int(lib().moe_swap_slot_bytes(ctypes.byref(layer.c)))
        self.space = torch.empty(max(1, n_slots * self.slot_bytes), dtype=torch.uint8, device="cuda")
        self.host_idx = torch.empty(n_tokens * layer.top_k, dtype=torch.int32).pin_memory()
        self.copy_stream = torch.cuda.Stream()
        self.copied, self.computed = torch.cuda.Event(), torch.cuda.Event()
        # torch creates the underlying hipEvent_t lazily, on the first record
        self.copied.record(self.copy_stream)
        self.computed.record(self.copy_stream)
        self.c = CSwap(self._arr, _ptr(self.space), self.slot_bytes, n_slots, self.host_idx.data_ptr(),
                       self.copy_stream.cuda_stream, self.copied.cuda_event, self.computed.cuda_event)


def moe_layer_forward_swap(layer: Layer, swap: Swap, x, out, ws, topk_idx_out=None, topk_gate_out=None) -> int:
    """Returns the number of experts copied in by this call."""
    missed = ctypes.c_int32(0)
    _check(lib().moe_layer_forward_swap(ctypes.byref(layer.c), ctypes.byref(swap.c), _ptr(x), x.shape[0], _ptr(out),
                                        _ptr(topk_idx_out), _ptr(topk_gate_out), _ptr(ws), ws.numel(), _stream(),
                                        ctypes.byref(missed)))
    return missed.value


class Chain:
    """Host arrays for moe_chain_forward, built once."""

    def __init__(self, layers: Sequence[Layer], rms_gains: Sequence):
        self.layers, self.rms_gains = list(layers), list(rms_gains)
        self.c_layers = (CLayer * len(self.layers))(*[l.c for l in self.layers])
        self.c_gains = (ctypes.c_void_p * len(self.layers))(*[_ptr(g) for g in self.rms_gains])


def moe_chain_forward(chain: Chain, eps: float, h, ws, topk_idx_out=None) -> None:
    _check(lib().moe_chain_forward(chain.c_layers, chain.c_gains, len(chain.layers), eps, _ptr(h), h.shape[0],
                                   _ptr(topk_idx_out), _ptr(ws), ws.numel(), _stream()))


def moe_dequant_int4(m: Mat, out: int, inn: int, w_fp16) -> None:
    cm = m.c()
    _check(lib().moe_dequant_int4(ctypes.byref(cm), out, inn, _ptr(w_fp16), _stream()))


def moe_quantize_int4(w_fp16, packed, scale, zero) -> None:
    out, inn = w_fp16.shape
    _check(lib().moe_quantize_int4(_ptr(w_fp16), out, inn, _ptr(packed), _ptr(scale), _ptr(zero), _stream()))


def moe_dequant_int8(m: Mat, out: int, inn: int, w_fp16) -> None:
    cm = m.c()
    _check(lib().moe_dequant_int8(ctypes.byref(cm), out, inn, _ptr(w_fp16), _stream()))


def moe_quantize_int8(w_fp16, codes, scale, zero) -> None:
    out, inn = w_fp16.shape
    _check(lib().moe_quantize_int8(_ptr(w_fp16), out, inn, _ptr(codes), _ptr(scale), _ptr(zero), _stream()))


def moe_synth_fill_f16(dst, first: int, seed: int, stream_id: int, scale: float, kind: int) -> None:
    _check(lib().moe_synth_fill_f16(_ptr(dst), dst.numel(), first, seed, stream_id, scale, kind, _stream()))


def moe_read_status(ws) -> int:
    """Status bits of the last call on workspace ``ws`` (None: of the last moe_layer_forward_static call)."""
    v = ctypes.c_int(0)
    _check(lib().moe_read_status(_ptr(ws), _stream(), ctypes.byref(v)))
    return v.value


KERNEL_ROUTE, KERNEL_PERMUTE, KERNEL_UP, KERNEL_DOWN, KERNEL_COMBINE, KERNEL_STREAM_READ = range(6)


def moe_trace_kernel(kernel: int, start_event: Optional[int], stop_event: Optional[int]) -> None:
    """Arms a one-shot event bracket around the next launch of ``kernel``; (None, None) drops an unused one."""
    _check(lib().moe_trace_kernel(kernel, start_event, stop_event))


def moe_stream_read(src, nbytes: int, sink) -> None:
    _check(lib().moe_stream_read(_ptr(src), nbytes, _ptr(sink), _stream()))


def moe_plan(mem_gpu: int, size_non_expert: int, size_e16: int, size_e4: int, num_experts: int, preference: int,
             num_e4: int = 0, seed: int = 0, swap_bytes: int = 0):
    """Returns (CPlanResult, quantized list, resident list); host-only."""
    req = CPlanRequest(mem_gpu, size_non_expert, size_e16, size_e4, swap_bytes, seed, num_experts, preference, num_e4)
    res = CPlanResult()
    q = (ctypes.c_uint8 * max(num_experts, 1))()
    r = (ctypes.c_uint8 * max(num_experts, 1))()
    rc = lib().moe_plan(ctypes.byref(req), ctypes.byref(res), q, r)
    if rc != MOE_OK:
        raise MoeError(rc, "moe_plan rejected the request")
    return res, list(q)[:num_experts], list(r)[:num_experts]


def moe_version() -> int:
    return int(lib().moe_version())


# ---------------------------------------------------------------- conveniences built only from the calls above

def quantize_mat(w_fp16) -> Mat:
    """Device-side 16-bit -> 4-bit switch of one matrix (moe_quantize_int4)."""
    import torch
    out, inn = w_fp16.shape
    packed = torch.empty((out, inn // 2), dtype=torch.uint8, device=w_fp16.device)
    scale = torch.empty((out, inn // GROUP), dtype=torch.float16, device=w_fp16.device)
    zero = torch.empty((out, inn // GROUP), dtype=torch.float16, device=w_fp16.device)
    moe_quantize_int4(w_fp16, packed, scale, zero)
    return Mat(packed, scale, zero)


def quantize_mat8(w_fp16) -> Mat:
    """Device-side 16-bit -> 8-bit switch of one matrix (moe_quantize_int8)."""
    import torch
    out, inn = w_fp16.shape
    codes = torch.empty((out, inn), dtype=torch.uint8, device=w_fp16.device)
    scale = torch.empty((out, inn // GROUP), dtype=torch.float16, device=w_fp16.device)
    zero = torch.empty((out, inn // GROUP), dtype=torch.float16, device=w_fp16.device)
    moe_quantize_int8(w_fp16, codes, scale, zero)
    return Mat(codes, scale, zero)
