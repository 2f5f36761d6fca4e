#!/usr/bin/env python3
"""Benchmark of the mixed-precision MoE block on one MI355X.

Workload (the configuration the headline metric is quoted on): Mixtral-shaped single MoE layer,
batch-1 decode -- d_model 4096, d_ff 14336, 8 SwiGLU experts, top-2, one token per step, experts 0-3
16-bit and 4-7 4-bit (uint4, group 64).  A step is one moe_layer_forward call: gating, top-k, both
routed experts, weighted average.  To keep the last-level cache from serving weights, steps rotate over
a pool of independent layers (1.8 GB each) and every step has its own token, so the routed pair (and
its precision mix) changes from step to step.  All inputs are synthetic and resident in HBM before the
timed region.

Prints ONE JSON line; `value` is layer tokens/s, `effective_weight_GBps` the stored bytes of the experts
that received tokens (plus the gate matrix) per second.  `roofline` is measured live with HIP events
around every launch of the dominant kernel; `cpu_baseline` times the CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0
D, F, E, K = 4096, 14336, 8, 2
INT4_EXPERTS = (4, 5, 6, 7)


class HipEvents:
    """hipEvent_t pairs through the HIP runtime that torch has already loaded."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.hip.hipEventDestroy(ev)


def cpu_baseline(seed: int, n_tokens: int):
    """The oracle, as it stands, on the host cores: the same decode workload, first `n_tokens` steps of
    pool layer 0.  Only the routed experts are generated on the host (set-up is not timed)."""
    import numpy as np
    from oracle import moe_oracle as orc
    from paper_2407_14417_amd import synth

    sigma = 0.02
    wg = synth.normal_f16((E, D), sigma, seed, synth.STREAM_WG)
    x = synth.normal_f16((n_tokens, D), 1.0, seed, synth.x_stream(0))
    idx, _ = orc.route(x, wg, K)
    need = sorted(set(int(e) for e in idx.reshape(-1)))
    dummy = orc.Mat(np.zeros((1, 1), dtype=np.float16))
    experts = []
    for e in range(E):
        if e not in need:
            experts.append(orc.Expert(dummy, dummy, dummy, resident=False))
            continue
        ws = [synth.normal_f16(s, sigma, seed, synth.expert_stream(0, e, i))
              for i, s in enumerate(((F, D), (F, D), (D, F)))]
        if e in INT4_EXPERTS:
            experts.append(orc.Expert(*[orc.quantize_int4(w) for w in ws]))
        else:
            experts.append(orc.Expert(*[orc.Mat(w) for w in ws]))
    t0 = time.perf_counter()
    for t in range(n_tokens):
        orc.layer_forward(x[t:t + 1], wg, experts, K)
    dt = time.perf_counter() - t0
    return {"value": n_tokens / dt, "unit": "tokens/s", "cores": orc.max_threads(), "kind": "oracle",
            "sample": f"{n_tokens} decode steps (T=1) of pool layer 0, routed experts only, "
                      f"{dt:.1f} s of oracle time; OpenMP over output rows"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--pool", type=int, default=8, help="independent layers the steps rotate over")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--cpu-tokens", type=int, default=8, help="oracle sample size (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2407_14417_amd import binding as mm
    from paper_2407_14417_amd import workload

    mm.lib()                                    # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    steps, warmup, pool = args.steps, args.warmup, args.pool

    layers = [workload.device_layer(D, F, E, K, INT4_EXPERTS, seed=args.seed, layer=l) for l in range(pool)]
    n_tok = steps + warmup
    x_all = workload.device_tokens(n_tok, D, seed=args.seed)
    out_all = torch.empty((n_tok, D), dtype=torch.float16, device="cuda")
    idx_all = torch.empty((n_tok, K), dtype=torch.int32, device="cuda")
    ws = mm.alloc_workspace(layers[0], 1)
    torch.cuda.synchronize()

    def step(i: int) -> None:
        mm.moe_layer_forward(layers[i % pool], x_all[i:i + 1], out_all[i:i + 1], ws, idx_all[i:i + 1], None)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for i in range(warmup):
            step(i)
        stream.synchronize()
        graph = None
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(warmup, n_tok):
                    step(i)
            graph.replay()                      # one untimed replay: graph upload
            stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if graph is not None:
            graph.replay()
        else:
            for i in range(warmup, n_tok):
                step(i)
        stream.synchronize()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

        # ---- roofline leg: the same steps, eagerly, the two matrix kernels of every step between HIP events
        ev = HipEvents()
        traced = {"up": mm.KERNEL_UP, "down": mm.KERNEL_DOWN, "route": mm.KERNEL_ROUTE}
        pairs = {n: [(ev.create(), ev.create()) for _ in range(steps)] for n in traced}
        for j, i in enumerate(range(warmup, n_tok)):
            for n, kid in traced.items():
                mm.moe_trace_kernel(kid, pairs[n][j][0], pairs[n][j][1])
            step(i)
        stream.synchronize()
        ms = {n: np.array([ev.elapsed_ms(a, b) for a, b in pairs[n]]) for n in traced}
        for n in traced:
            for a, b in pairs[n]:
                ev.destroy(a)
                ev.destroy(b)

    idx = idx_all[warmup:].cpu().numpy()
    per_step_bytes = np.array([workload.stored_bytes(layers[(warmup + j) % pool], idx[j]) for j in range(steps)], dtype=np.float64)
    # up-projection: w1 and w3 of both routed experts = 2/3 of their stored bytes; down-projection: w2 = 1/3
    gate_bytes = E * D * 2
    up_bytes = (per_step_bytes - gate_bytes) * (2.0 / 3.0)
    down_bytes = (per_step_bytes - gate_bytes) * (1.0 / 3.0)
    up_ms = ms["up"]
    n_int4 = np.array([sum(int(e) in INT4_EXPERTS for e in idx[j]) for j in range(steps)])
    by_pair = {}
    for kind, name in ((0, "fp16+fp16"), (1, "fp16+int4"), (2, "int4+int4")):
        sel = n_int4 == kind
        if sel.any():
            by_pair[name] = {"launches": int(sel.sum()), "avg_us": float(up_ms[sel].mean() * 1e3),
                             "GBps": float(up_bytes[sel].sum() / (up_ms[sel].sum() * 1e-3) / 1e9),
                             "down_avg_us": float(ms["down"][sel].mean() * 1e3),
                             "down_GBps": float(down_bytes[sel].sum() / (ms["down"][sel].sum() * 1e-3) / 1e9)}
    achieved = float(up_bytes.sum() / (up_ms.sum() * 1e-3) / 1e9)
    other = {"down_projection": {"avg_launch_us": float(ms["down"].mean() * 1e3),
                                 "GBps": float(down_bytes.sum() / (ms["down"].sum() * 1e-3) / 1e9)},
             "route": {"avg_launch_us": float(ms["route"].mean() * 1e3)}}

    result = {
        "metric": "MoE-layer tokens/s + effective weight HBM GB/s (% of peak), Mixtral shape",
        "value": steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 weights / uint4-g64 weights, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "Mixtral-shaped single MoE layer, batch-1 decode: d_model=4096, d_ff=14336, 8 experts, "
                               "top-2, 1 token/step, experts 0-3 fp16, 4-7 uint4 g64",
                   "pool_layers": pool, "launch": "eager" if graph is None else "hip-graph replay of all steps",
                   "routed_pairs": {k: v["launches"] for k, v in by_pair.items()}},
        "effective_weight_GBps": float(per_step_bytes.sum() / elapsed / 1e9),
        "pct_of_hbm_peak": float(per_step_bytes.sum() / elapsed / 1e9 / HBM_PEAK_GBPS * 100.0),
        "roofline": {"bound": "hbm", "kernel": "expert up-projection (w1, w3 of both routed experts, SiLU-gate)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": None, "avg_launch_us": float(up_ms.mean() * 1e3), "by_pair": by_pair,
                     "other_kernels": other},
    }
    if args.cpu_tokens > 0:
        result["cpu_baseline"] = cpu_baseline(args.seed, args.cpu_tokens)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
