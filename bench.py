#!/usr/bin/env python3
"""Benchmark of the mixed-precision MoE block on one MI355X.

Default workload (the configuration the headline metric is quoted on): Mixtral-shaped single MoE layer,
batch-1 decode -- d_model 4096, d_ff 14336, 8 SwiGLU experts, top-2, one token per step, experts 0-3
16-bit and 4-7 4-bit (uint4, group 64).  A step is one moe_layer_forward call: gating, top-k, the routed
experts, weighted average.  To keep the last-level cache from serving weights, steps rotate over a pool of
independent layers and every step has its own tokens, so the routed experts (and their precision mix)
change from step to step.  All inputs are synthetic and resident in HBM before the timed region.

Other workloads of the same layer shape (`--workload`): `batched` (16 tokens per step, all experts 4-bit,
uniform-random gate matrix), `prefill` (512 tokens per step, experts 0-1 16-bit and 2-7 4-bit, Zipf(1.2)
logit offsets), `chain` (32 x (RMSNorm -> block -> residual), 1 token, a seeded random half of the 256
experts 4-bit; a step is one pass through all 32 blocks).

Prints ONE JSON line; `value` is tokens/s, `effective_weight_GBps` the stored bytes of the experts that
received tokens (plus the gate matrix) per second.  `roofline` is measured live with HIP events around every
launch of the dominant kernel (the up-projection: 2/3 of the weights); `cpu_baseline` times the CPU oracle
on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
D, F, E, K = 4096, 14336, 8, 2
SIGMA = 0.02

WORKLOADS = {
    "decode": dict(T=1, int4=(4, 5, 6, 7), router="normal", zipf=None, pool=8, steps=400, warmup=40, bound="hbm",
                   name="Mixtral-shaped single MoE layer, batch-1 decode: d_model=4096, d_ff=14336, 8 experts, "
                        "top-2, 1 token/step, experts 0-3 fp16, 4-7 uint4 g64"),
    "batched": dict(T=16, int4=tuple(range(8)), router="uniform", zipf=None, pool=4, steps=200, warmup=20,
                    bound="hbm",
                    name="Mixtral-shaped layer, fully quantized batched decode: 8 experts all uint4 g64, top-2, "
                         "16 tokens/step, uniform-random gate matrix"),
    "prefill": dict(T=512, int4=(2, 3, 4, 5, 6, 7), router="normal", zipf=1.2, pool=4, steps=100, warmup=10,
                    bound="mfma",
                    name="Mixtral-shaped prefill layer: 512 tokens/step, 8 experts top-2, experts 0-1 fp16, 2-7 "
                         "uint4 g64, Zipf(1.2) logit offsets"),
    "offload": dict(T=1, steps=60, warmup=6, bound="hbm",
                    name="Mixtral-shaped single MoE layer, batch-1 decode with the expert-miss path: the planner "
                         "decides from a memory budget which of the 8 experts are 4-bit and which stay in device "
                         "memory; missed experts are copied from pinned host memory into a swap slot"),
    "chain": dict(T=1, layers=32, steps=40, warmup=4, bound="hbm",
                  name="32-layer chained MoE decode step: 32 x (RMSNorm 1e-5 -> 8-expert top-2 block -> residual), "
                       "1 token, 128 of 256 experts uint4 g64 by seeded random mask"),
}


def traffic_ratio(profile_name: str, key: str):
    """HBM bytes fetched per launch over algorithmic bytes per launch, as measured with rocprofv3 --pmc FETCH_SIZE
    (scaled by the same counter's reading for a plain copy of known size) and recorded in profiles/<name>:
    a line `TRAFFIC_OVER_ALGORITHMIC <key> = <ratio>`.  None if no such record exists."""
    f = ROOT / "profiles" / profile_name
    if not f.exists():
        return None
    for line in f.read_text().splitlines():
        parts = line.split()
        if len(parts) == 4 and parts[0] == "TRAFFIC_OVER_ALGORITHMIC" and parts[1] == key and parts[2] == "=":
            return float(parts[3])
    return None


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


def cpu_baseline(wl: dict, seed: int, n_tokens: int):
    """The oracle, as it stands, on the host cores: the first `n_tokens` tokens of the workload's token stream
    through pool layer 0.  Only the routed experts are generated on the host (set-up is not timed)."""
    import numpy as np
    from oracle import moe_oracle as orc
    from paper_2407_14417_amd import synth

    if wl["router"] == "uniform":
        wg = synth.uniform_f16((E, D), SIGMA * 3 ** 0.5, seed, synth.STREAM_WG)
    else:
        wg = synth.normal_f16((E, D), SIGMA, seed, synth.STREAM_WG)
    bias = None if wl["zipf"] is None else synth.zipf_bias(E, wl["zipf"])
    x = synth.normal_f16((n_tokens, D), 1.0, seed, synth.x_stream(0))
    idx, _ = orc.route(x, wg, K, bias)
    need = sorted(set(int(e) for e in idx.reshape(-1)))
    dummy = orc.Mat(np.zeros((1, 1), dtype=np.float16))
    experts = []
    for e in range(E):
        if e not in need:
            experts.append(orc.Expert(dummy, dummy, dummy, resident=False))
            continue
        ws = [synth.normal_f16(s, SIGMA, seed, synth.expert_stream(0, e, i))
              for i, s in enumerate(((F, D), (F, D), (D, F)))]
        if e in wl["int4"]:
            experts.append(orc.Expert(*[orc.quantize_int4(w) for w in ws]))
        else:
            experts.append(orc.Expert(*[orc.Mat(w) for w in ws]))
    T = wl["T"]
    t0 = time.perf_counter()
    for t in range(0, n_tokens, T):
        orc.layer_forward(x[t:t + T], wg, experts, K, bias)
    dt = time.perf_counter() - t0
    return {"value": n_tokens / dt, "unit": "tokens/s", "cores": orc.max_threads(), "kind": "oracle",
            "sample": f"first {n_tokens} tokens of the workload in calls of {min(T, n_tokens)}, pool layer 0, routed "
                      f"experts only, {dt:.1f} s of oracle time; OpenMP over output rows"}


def run_layer_workload(args, wl, mm, workload, torch, np):
    T, pool = wl["T"], args.pool or wl["pool"]
    steps, warmup = args.steps or wl["steps"], args.warmup if args.warmup is not None else wl["warmup"]
    layers = [workload.device_layer(D, F, E, K, wl["int4"], seed=args.seed, layer=l, router=wl["router"],
                                    zipf=wl["zipf"]) for l in range(pool)]
    n_tok = steps + warmup
    x_all = workload.device_tokens(n_tok * T, D, seed=args.seed).reshape(n_tok, T, D)
    out_all = torch.empty((n_tok, T, D), dtype=torch.float16, device="cuda")
    idx_all = torch.empty((n_tok, T, K), dtype=torch.int32, device="cuda")
    ws = mm.alloc_workspace(layers[0], T)
    torch.cuda.synchronize()

    def step(i: int) -> None:
        mm.moe_layer_forward(layers[i % pool], x_all[i], out_all[i], ws, idx_all[i], None)

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

        # ---- roofline leg: the same steps, eagerly, the kernels of every step between HIP events
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
        assert mm.moe_read_status(ws) == 0

    idx = idx_all[warmup:].cpu().numpy()
    per_step_bytes = np.array([workload.stored_bytes(layers[(warmup + j) % pool], idx[j].reshape(-1))
                               for j in range(steps)], dtype=np.float64)
    # up-projection: w1 and w3 of the routed experts = 2/3 of their stored bytes; down-projection: w2 = 1/3
    gate_bytes = E * D * 2
    up_bytes = (per_step_bytes - gate_bytes) * (2.0 / 3.0)
    down_bytes = (per_step_bytes - gate_bytes) * (1.0 / 3.0)
    up_ms, down_ms = ms["up"], ms["down"]
    up_flops = 2.0 * 2.0 * D * F * T * K          # 2 flops per weight of w1, w3 per routed (token, expert) pair
    down_flops = 2.0 * D * F * T * K
    extra = {}
    if T == 1:
        n_int4 = np.array([sum(int(e) in wl["int4"] for e in idx[j, 0]) for j in range(steps)])
        by_pair = {}
        for kind, name in ((0, "fp16+fp16"), (1, "fp16+int4"), (2, "int4+int4")):
            sel = n_int4 == kind
            if sel.any():
                by_pair[name] = {"launches": int(sel.sum()), "avg_us": float(up_ms[sel].mean() * 1e3),
                                 "GBps": float(up_bytes[sel].sum() / (up_ms[sel].sum() * 1e-3) / 1e9),
                                 "down_avg_us": float(down_ms[sel].mean() * 1e3),
                                 "down_GBps": float(down_bytes[sel].sum() / (down_ms[sel].sum() * 1e-3) / 1e9)}
        extra["by_pair"] = by_pair
    else:
        counts = np.stack([np.bincount(idx[j].reshape(-1), minlength=E) for j in range(steps)])
        extra["rows_per_expert_mean"] = [float(c) for c in counts.mean(axis=0)]
        extra["active_experts_mean"] = float((counts > 0).sum(axis=1).mean())
    up_GBps = float(up_bytes.sum() / (up_ms.sum() * 1e-3) / 1e9)
    up_TFLOPs = float(up_flops * steps / (up_ms.sum() * 1e-3) / 1e12)
    other = {"down_projection": {"avg_launch_us": float(down_ms.mean() * 1e3),
                                 "GBps": float(down_bytes.sum() / (down_ms.sum() * 1e-3) / 1e9),
                                 "TFLOPs": float(down_flops * steps / (down_ms.sum() * 1e-3) / 1e12)},
             "route": {"avg_launch_us": float(ms["route"].mean() * 1e3)}}
    if wl["bound"] == "hbm":
        roof = {"bound": "hbm", "kernel": "expert up-projection (w1, w3 of the routed experts, SiLU-gate)",
                "achieved": up_GBps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": up_GBps / HBM_PEAK_GBPS,
                "traffic": None, "avg_launch_us": float(up_ms.mean() * 1e3), "TFLOPs": up_TFLOPs}
    else:
        roof = {"bound": "mfma", "kernel": "expert up-projection (w1, w3 of the routed experts, SiLU-gate), "
                                           "grouped fp16 MFMA product",
                "achieved": up_TFLOPs, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": up_TFLOPs / MFMA_F16_PEAK_TFLOPS, "traffic": None,
                "avg_launch_us": float(up_ms.mean() * 1e3), "GBps": up_GBps,
                "frac_of_hbm_peak_on_bytes": up_GBps / HBM_PEAK_GBPS}
    ratio = traffic_ratio({"decode": "decode_b1_hbm_traffic.md"}.get(args.workload, "none"), "up_projection")
    if ratio is not None:
        roof["traffic"] = ratio * float(up_bytes.mean())          # bytes per launch, like `achieved`
        roof["traffic_source"] = "profiles/decode_b1_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE, copy-calibrated): " \
                                 f"fetched/algorithmic = {ratio}"
    roof["algorithmic_bytes_per_launch"] = float(up_bytes.mean())
    roof.update(extra)
    roof["other_kernels"] = other
    return {
        "value": steps * T / elapsed, "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3,
        "config": {"workload": wl["name"], "tokens_per_step": T, "pool_layers": pool,
                   "launch": "eager" if graph is None else "hip-graph replay of all steps"},
        "effective_weight_GBps": float(per_step_bytes.sum() / elapsed / 1e9),
        "pct_of_hbm_peak": float(per_step_bytes.sum() / elapsed / 1e9 / HBM_PEAK_GBPS * 100.0),
        "TFLOPs": float((up_flops + down_flops) * steps / elapsed / 1e12),
        "roofline": roof,
    }


def run_chain_workload(args, wl, mm, workload, torch, np):
    from paper_2407_14417_amd import synth
    L = wl["layers"]
    steps, warmup = args.steps or wl["steps"], args.warmup if args.warmup is not None else wl["warmup"]
    mask = synth.precision_mask(E * L, E * L // 2, args.seed)
    layers = []
    for l in range(L):
        layers.append(workload.device_layer(D, F, E, K, tuple(e for e in range(E) if mask[l * E + e]),
                                            seed=args.seed, layer=l))
    gains = [torch.ones(D, dtype=torch.float16, device="cuda") for _ in range(L)]
    chain = mm.Chain(layers, gains)
    n_tok = steps + warmup
    h_all = workload.device_tokens(n_tok, D, seed=args.seed).reshape(n_tok, 1, D)
    idx_all = torch.empty((n_tok, L, 1, K), dtype=torch.int32, device="cuda")
    ws = mm.alloc_workspace(layers[0], 1)
    torch.cuda.synchronize()

    def step(i: int) -> None:
        mm.moe_chain_forward(chain, 1e-5, h_all[i], ws, idx_all[i])

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
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if graph is not None:
            graph.replay()                      # the chain updates h in place: every replay needs fresh tokens,
        else:                                   # so the one timed replay is also the first
            for i in range(warmup, n_tok):
                step(i)
        stream.synchronize()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        assert mm.moe_read_status(ws) == 0
    idx = idx_all[warmup:].cpu().numpy()
    per_step_bytes = np.array([sum(workload.stored_bytes(layers[l], idx[j, l, 0]) for l in range(L))
                               for j in range(steps)], dtype=np.float64)
    GBps = float(per_step_bytes.sum() / elapsed / 1e9)
    return {
        "value": steps / elapsed, "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3,
        "config": {"workload": wl["name"], "tokens_per_step": 1, "layers": L,
                   "resident_GB": float(sum(e.nbytes() for l in layers for e in l.experts) / 1e9),
                   "launch": "eager" if graph is None else "hip-graph replay of all steps"},
        "effective_weight_GBps": GBps, "pct_of_hbm_peak": GBps / HBM_PEAK_GBPS * 100.0,
        "roofline": {"bound": "hbm", "kernel": "whole step (32 x route, up-projection, down-projection)",
                     "achieved": GBps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": GBps / HBM_PEAK_GBPS,
                     "traffic": None, "bytes_per_step_GB": float(per_step_bytes.mean() / 1e9)},
    }


def run_offload_workload(args, wl, mm, workload, torch, np):
    """Decode steps through moe_layer_forward_swap.  The planner (moe_plan, quality preference) turns --mem-mb and
    --num-e4 into the precision mask and the residency of the 8 experts of every pool layer."""
    steps, warmup = args.steps or wl["steps"], args.warmup if args.warmup is not None else wl["warmup"]
    pool = args.pool or 2
    size_e16, size_e4 = 3 * D * F * 2, 3 * (D * F // 2 + 2 * (D * F // 64) * 2)
    size_ne = E * D * 2
    slot = size_e16 if args.num_e4 < E else size_e4
    plan, quantized, resident = mm.moe_plan(int(args.mem_mb * 1e6), size_ne, size_e16, size_e4, E, mm.PREFER_QUALITY,
                                            args.num_e4, args.seed, args.slots * slot)
    layers, swaps = [], []
    for l in range(pool):
        experts, hosts = [], []
        for e in range(E):
            de = workload.device_expert(D, F, args.seed, l, e, bool(quantized[e]))
            if resident[e]:
                experts.append(de)
                hosts.append(None)
            else:
                def to_host(m):
                    return mm.Mat(*[None if t is None else t.cpu().pin_memory() for t in (m.data, m.scale, m.zero)])
                hosts.append(mm.Expert(de.prec, to_host(de.w1), to_host(de.w3), to_host(de.w2), resident=False))
                experts.append(mm.Expert(de.prec, None, None, None, resident=False))
                del de
        from paper_2407_14417_amd import synth
        wg = workload.fill_normal((E, D), SIGMA, args.seed, synth.STREAM_WG + 16 * l)
        layer = mm.Layer(D, F, K, wg, experts, None)
        layers.append(layer)
        swaps.append(mm.Swap(layer, hosts, args.slots, 1))
    n_tok = steps + warmup
    x_all = workload.device_tokens(n_tok, D, seed=args.seed).reshape(n_tok, 1, D)
    out_all = torch.empty((n_tok, 1, D), dtype=torch.float16, device="cuda")
    ws = mm.alloc_workspace(layers[0], 1)
    torch.cuda.synchronize()
    misses = 0
    for i in range(warmup):
        mm.moe_layer_forward_swap(layers[i % pool], swaps[i % pool], x_all[i], out_all[i], ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(warmup, n_tok):
        misses += mm.moe_layer_forward_swap(layers[i % pool], swaps[i % pool], x_all[i], out_all[i], ws)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert mm.moe_read_status(ws) == 0
    return {
        "value": steps / elapsed, "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3,
        "config": {"workload": wl["name"], "tokens_per_step": 1, "pool_layers": pool, "launch": "eager",
                   "mem_budget_MB": args.mem_mb, "num_e4": int(plan.num_e4), "resident_e4": int(plan.resident_e4),
                   "resident_e16": int(plan.resident_e16), "swap_slots": args.slots,
                   "resident_MB": plan.bytes_resident / 1e6},
        "expert_misses_per_token": misses / steps,
        "roofline": {"bound": "pcie", "kernel": "host-to-device copy of missed experts", "achieved": None, "peak": None,
                     "unit": "GB/s", "frac": None, "traffic": None},
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0 = the workload's default)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="decode")
    ap.add_argument("--pool", type=int, default=0, help="independent layers the steps rotate over (0 = default)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--cpu-tokens", type=int, default=-1, help="oracle sample size (0 = skip, -1 = default)")
    ap.add_argument("--int4-experts", default=None,
                    help="comma-separated expert indices that are 4-bit instead of the workload's own mask "
                         "(e.g. 0,1,2,3,4,5,6,7 times the all-4-bit pair at batch 1)")
    ap.add_argument("--mem-mb", type=float, default=2000.0, help="offload workload: device memory budget of the layer")
    ap.add_argument("--num-e4", type=int, default=4, help="offload workload: number of 4-bit experts (of 8)")
    ap.add_argument("--slots", type=int, default=2, help="offload workload: swap slots")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run a plain device-to-device copy of this many MiB three times: the known-size kernel "
                         "that rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled by")
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
    wl = dict(WORKLOADS[args.workload])
    if args.int4_experts is not None and "int4" in wl:       # measurement variant: another precision mask
        wl["int4"] = tuple(int(e) for e in args.int4_experts.split(",") if e != "")
        wl["name"] += f" [precision mask overridden: 4-bit experts {list(wl['int4'])}]"
    if args.workload == "chain":
        res = run_chain_workload(args, wl, mm, workload, torch, np)
    elif args.workload == "offload":
        res = run_offload_workload(args, wl, mm, workload, torch, np)
    else:
        res = run_layer_workload(args, wl, mm, workload, torch, np)

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    result = {
        "metric": "MoE-layer tokens/s + effective weight HBM GB/s (% of peak), Mixtral shape",
        "value": res.pop("value"),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": res.pop("steps"),
        "warmup": res.pop("warmup"),
        "ms_per_step": res.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 (products of f16 weights and activations accumulated in f32; uint4-g64 weights expanded to f16)",
        "data": "synthetic",
    }
    result.update(res)
    cpu_tokens = args.cpu_tokens
    if cpu_tokens < 0:
        cpu_tokens = {"decode": 48, "batched": 48, "prefill": 64, "chain": 0, "offload": 0}[args.workload]
    if cpu_tokens > 0:
        result["cpu_baseline"] = cpu_baseline(wl, args.seed, cpu_tokens)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
