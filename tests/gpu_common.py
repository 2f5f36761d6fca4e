"""Upload of host workloads (numpy, oracle descriptors) into device descriptors of the binding."""
from __future__ import annotations

import numpy as np
import torch

from paper_2407_14417_amd import binding as mm


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def prec_of(e) -> int:
    """Library precision code of an oracle expert."""
    return mm.PREC_INT4G64 if e.int4 else (mm.PREC_INT8G64 if e.int8 else mm.PREC_FP16)


def device_mat(m) -> mm.Mat:
    if m.scale is None:
        return mm.Mat(dev(m.data))
    return mm.Mat(dev(m.data), dev(m.scale), dev(m.zero))


def device_expert(e) -> mm.Expert:
    if e is None:
        return mm.Expert(mm.PREC_FP16, None, None, None, resident=False)
    return mm.Expert(prec_of(e), device_mat(e.w1), device_mat(e.w3), device_mat(e.w2), resident=e.resident)


def device_layer(wl) -> mm.Layer:
    cfg = wl.cfg
    bias = None if wl.bias is None else dev(wl.bias)
    return mm.Layer(cfg.d, cfg.f, cfg.k, dev(wl.wg), [device_expert(e) for e in wl.experts], bias)


def pinned(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).pin_memory()


def host_expert(e) -> mm.Expert:
    """The same expert in pinned host memory (what the expert-miss path copies from)."""
    def mat(m):
        if m.scale is None:
            return mm.Mat(pinned(m.data))
        return mm.Mat(pinned(m.data), pinned(m.scale), pinned(m.zero))
    return mm.Expert(prec_of(e), mat(e.w1), mat(e.w3), mat(e.w2), resident=False)


def device_layer_with_offloaded(wl, offloaded):
    """(layer whose experts in `offloaded` are marked not resident and hold no device data, host-side experts)."""
    cfg = wl.cfg
    bias = None if wl.bias is None else dev(wl.bias)
    experts, hosts = [], []
    for i, e in enumerate(wl.experts):
        if i in offloaded:
            experts.append(mm.Expert(prec_of(e), None, None, None, resident=False))
            hosts.append(host_expert(e))
        else:
            experts.append(device_expert(e))
            hosts.append(None)
    return mm.Layer(cfg.d, cfg.f, cfg.k, dev(wl.wg), experts, bias), hosts
