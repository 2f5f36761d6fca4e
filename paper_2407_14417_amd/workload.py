"""Device-resident synthetic MoE layers for tests and the benchmark.

Weights are drawn directly in device memory with the library's seeded fill
(``moe_synth_fill_f16``, the same streams as :mod:`synth` on the host) and, for
4-bit experts, quantized in place with ``moe_quantize_int4``.  Nothing here
computes any part of the MoE block.
"""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as mm
from . import synth

SIGMA_W = 0.02


def fill_normal(shape, sigma: float, seed: int, stream_id: int, first: int = 0) -> torch.Tensor:
    t = torch.empty(shape, dtype=torch.float16, device="cuda")
    mm.moe_synth_fill_f16(t, first, seed, stream_id, float(synth.normal_scale(sigma)), 0)
    return t


def fill_uniform(shape, a: float, seed: int, stream_id: int, first: int = 0) -> torch.Tensor:
    t = torch.empty(shape, dtype=torch.float16, device="cuda")
    mm.moe_synth_fill_f16(t, first, seed, stream_id, float(synth.uniform_scale(a)), 1)
    return t


def device_expert(d: int, f: int, seed: int, layer: int, expert: int, int4: bool, int8: bool = False) -> mm.Expert:
    """Expert ``expert`` of ``layer``: w1, w3 [f,d], w2 [d,f] ~ N(0, 0.02), 16-bit or quantized to 4 or 8 bits."""
    mats = []
    for which, shape in enumerate(((f, d), (f, d), (d, f))):
        w = fill_normal(shape, SIGMA_W, seed, synth.expert_stream(layer, expert, which))
        if int4 or int8:
            m = mm.quantize_mat(w) if int4 else mm.quantize_mat8(w)
            del w
        else:
            m = mm.Mat(w)
        mats.append(m)
    prec = mm.PREC_INT4G64 if int4 else (mm.PREC_INT8G64 if int8 else mm.PREC_FP16)
    return mm.Expert(prec, mats[0], mats[1], mats[2])


def device_layer(d: int, f: int, n_experts: int, top_k: int, int4_experts: Sequence[int], seed: int = 0,
                 layer: int = 0, router: str = "normal", zipf: Optional[float] = None,
                 int8_experts: Sequence[int] = ()) -> mm.Layer:
    """One synthetic MoE block in device memory.  ``router``: "normal" = N(0, 0.02) gate matrix,
    "uniform" = U(+-0.02*sqrt(3)); ``zipf``: exponent of the per-expert logit offsets ln p_e, p_e ~ (e+1)^-s."""
    stream = synth.STREAM_WG + 16 * layer
    if router == "uniform":
        wg = fill_uniform((n_experts, d), SIGMA_W * 3 ** 0.5, seed, stream)
    else:
        wg = fill_normal((n_experts, d), SIGMA_W, seed, stream)
    bias = None if zipf is None else torch.from_numpy(synth.zipf_bias(n_experts, zipf)).cuda()
    experts = [device_expert(d, f, seed, layer, e, e in set(int4_experts), e in set(int8_experts))
               for e in range(n_experts)]
    return mm.Layer(d, f, top_k, wg, experts, bias)


def device_tokens(T: int, d: int, seed: int = 0, retry: int = 0) -> torch.Tensor:
    """x ~ N(0, 1), fp16 [T, d], the host generator's activation stream."""
    return fill_normal((T, d), 1.0, seed, synth.x_stream(retry))


def stored_bytes(layer: mm.Layer, experts: Sequence[int]) -> int:
    """Bytes of the stored weights of the given experts plus the gate matrix: the 'effective weight bytes'
    a block call has to stream when exactly these experts receive tokens."""
    return sum(layer.experts[e].nbytes() for e in set(int(e) for e in experts)) + layer.w_gate.numel() * 2
