#!/usr/bin/env python3
"""Benchmark of the mixed-precision MoE block on one MI355X.

Headline workload (the configuration the metric is quoted on): Mixtral-shaped single MoE layer, batch-1 decode
-- d_model 4096, d_ff 14336, 8 SwiGLU experts, top-2, one token per step, experts 0-3 16-bit and 4-7 4-bit
(uint4, group 64).  A step is one moe_layer_forward call: gating, top-k, the routed experts, weighted average.
To keep the last-level cache from serving weights, steps rotate over a pool of independent layers and every step
has its own token, so the routed experts (and their precision mix) change from step to step.  All inputs are
synthetic and resident in HBM before the timed region.

Timing: the K steps are captured in one HIP graph; the graph is replayed R >= 10 times (at least 200 timed steps
in all), every replay between two HIP events recorded on the launch stream; `ms_per_step` is the median replay
divided by K, p10/p90 are reported beside it.  `roofline` is measured live with HIP events around every launch
of the dominant kernel (the up-projection: 2/3 of the weights) in an eager pass over the same steps.

Besides the headline the same JSON line carries, under `configs`, the other workloads of the same layer shape,
each timed the same way and each with the parity metrics of one of its steps against the CPU oracle:
`decode_int4_only` / `decode_fp16_only` / `decode_int8_only` (batch-1 decode with every expert 4-bit / 16-bit / 8-bit:
the all-4-bit pair is the case the >= 70 % of HBM peak target is stated for), `batched` (16 tokens per step, all experts 4-bit,
uniform-random gate matrix), `prefill` (512 tokens per step, experts 0-1 16-bit and 2-7 4-bit, Zipf(1.2) logit
offsets), `chain` (32 x (RMSNorm -> block -> residual), 1 token, a seeded random half of the 256 experts 4-bit; a
step is one pass through all 32 blocks).  `stream_ceiling` is a plain streaming-read kernel at the byte counts of
the 4-bit and the 16-bit up-projection; `cpu_baseline` times the CPU oracle on a bounded sample of the headline
workload.  `--workload X` makes X the headline instead; `--configs none` drops the extra legs.
"""
from __future__ import annotations

import argparse
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
MIN_REPLAYS, MIN_TIMED_STEPS = 10, 200

WORKLOADS = {
    "decode": dict(T=1, int4=(4, 5, 6, 7), router="normal", zipf=None, pool=8, steps=40, warmup=8, bound="hbm",
                   name="Mixtral-shaped single MoE layer, batch-1 decode: d_model=4096, d_ff=14336, 8 experts, "
                        "top-2, 1 token/step, experts 0-3 fp16, 4-7 uint4 g64"),
    "decode_int4_only": dict(T=1, int4=tuple(range(8)), router="normal", zipf=None, pool=8, steps=40, warmup=8,
                             bound="hbm",
                             name="batch-1 decode, same layer shape, every expert uint4 g64 (the all-4-bit routed pair)"),
    "decode_fp16_only": dict(T=1, int4=(), router="normal", zipf=None, pool=4, steps=40, warmup=8, bound="hbm",
                             name="batch-1 decode, same layer shape, every expert fp16"),
    "decode_int8_only": dict(T=1, int4=(), int8=tuple(range(8)), router="normal", zipf=None, pool=6, steps=40, warmup=8,
                             bound="hbm",
                             name="batch-1 decode, same layer shape, every expert uint8 g64 (the precision of the "
                                  "paper's homogeneous 8-bit model)"),
    "batched": dict(T=16, int4=tuple(range(8)), router="uniform", zipf=None, pool=4, steps=20, warmup=4,
                    bound="hbm",
                    name="Mixtral-shaped layer, fully quantized batched decode: 8 experts all uint4 g64, top-2, "
                         "16 tokens/step, uniform-random gate matrix"),
    "prefill": dict(T=512, int4=(2, 3, 4, 5, 6, 7), router="normal", zipf=1.2, pool=4, steps=12, warmup=4,
                    bound="mfma",
                    name="Mixtral-shaped prefill layer: 512 tokens/step, 8 experts top-2, experts 0-1 fp16, 2-7 "
                         "uint4 g64, Zipf(1.2) logit offsets"),
    "offload": dict(T=1, steps=60, warmup=6, bound="hbm",
                    name="Mixtral-shaped single MoE layer, batch-1 decode with the expert-miss path: the planner "
                         "decides from a memory budget which of the 8 experts are 4-bit and which stay in device "
                         "memory; missed experts are copied from pinned host memory into a swap slot"),
    "chain": dict(T=1, layers=32, steps=6, warmup=2, bound="hbm",
                  name="32-layer chained MoE decode step: 32 x (RMSNorm 1e-5 -> 8-expert top-2 block -> residual), "
                       "1 token, 128 of 256 experts uint4 g64 by seeded random mask"),
}
EXTRA_CONFIGS = ("decode_int4_only", "decode_fp16_only", "decode_int8_only", "batched", "prefill", "chain")


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


# ---------------------------------------------------------------- timing

def percentiles(ms_per_replay, steps):
    import numpy as np
    a = np.asarray(ms_per_replay, dtype=np.float64) / steps
    return {"median": float(np.median(a)), "p10": float(np.percentile(a, 10)), "p90": float(np.percentile(a, 90)),
            "min": float(a.min()), "max": float(a.max())}


def timed_replays(torch, stream, step, first, steps, warmup, no_graph):
    """Warm-up steps [first - warmup, first), then steps [first, first + steps) captured in one HIP graph and
    replayed; every replay sits between two HIP events recorded on `stream`.  Returns the list of replay times
    in ms and the launch mode."""
    replays = max(MIN_REPLAYS, -(-MIN_TIMED_STEPS // steps))
    with torch.cuda.stream(stream):
        for i in range(first - warmup, first):
            step(i)
        stream.synchronize()
        graph = None
        if not no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(first, first + steps):
                    step(i)
            graph.replay()                      # one untimed replay: graph upload
            stream.synchronize()
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
        torch.cuda.synchronize()
        for a, b in events:
            a.record(stream)
            if graph is not None:
                graph.replay()
            else:
                for i in range(first, first + steps):
                    step(i)
            b.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in events], ("eager" if graph is None else "hip-graph replay of all steps")


# ---------------------------------------------------------------- oracle legs

def host_layer(wl, seed, layer, need):
    """Oracle-side tensors of pool layer `layer`: gate matrix, bias, and the experts in `need` (others absent)."""
    import numpy as np
    from oracle import moe_oracle as orc
    from paper_2407_14417_amd import synth
    stream = synth.STREAM_WG + 16 * layer
    if wl["router"] == "uniform":
        wg = synth.uniform_f16((E, D), SIGMA * 3 ** 0.5, seed, stream)
    else:
        wg = synth.normal_f16((E, D), SIGMA, seed, stream)
    bias = None if wl["zipf"] is None else synth.zipf_bias(E, wl["zipf"])
    dummy = orc.Mat(np.zeros((1, 1), dtype=np.float16))
    experts = []
    for e in range(E):
        if e not in need:
            experts.append(orc.Expert(dummy, dummy, dummy, resident=False))
            continue
        ws = [synth.normal_f16(s, SIGMA, seed, synth.expert_stream(layer, e, i))
              for i, s in enumerate(((F, D), (F, D), (D, F)))]
        if e in wl["int4"]:
            experts.append(orc.Expert(*[orc.quantize_int4(w) for w in ws]))
        elif e in wl.get("int8", ()):
            experts.append(orc.Expert(*[orc.quantize_int8(w) for w in ws]))
        else:
            experts.append(orc.Expert(*[orc.Mat(w) for w in ws]))
    return wg, bias, experts


def parity_metrics(got, ref):
    import numpy as np
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    err = got - ref
    return {"max_err_over_max_ref": float(np.abs(err).max() / np.abs(ref).max()),
            "rel_l2": float(np.linalg.norm(err) / np.linalg.norm(ref))}


def layer_parity(wl, seed, layer, x_host, idx_dev, out_dev, tokens):
    """One step of a layer workload against the oracle on the given tokens of that step."""
    import numpy as np
    from oracle import moe_oracle as orc
    t0 = time.perf_counter()
    wg, bias, _ = host_layer(wl, seed, layer, ())
    ref_idx, ref_gate = orc.route(x_host, wg, K, bias)
    need = sorted(set(int(e) for t in tokens for e in ref_idx[t]))
    _, _, experts = host_layer(wl, seed, layer, need)
    ref, _, _ = orc.layer_forward(np.ascontiguousarray(x_host[tokens]), wg, experts, K, bias)
    res = parity_metrics(out_dev[tokens], ref)
    res.update({"routing_indices_equal": bool(np.array_equal(idx_dev, ref_idx)), "tokens_checked": len(tokens),
                "tokens_in_step": int(x_host.shape[0]), "oracle_s": round(time.perf_counter() - t0, 1)})
    return res


def cpu_baseline(wl, seed: int, n_tokens: int):
    """The oracle, as it stands, on the host cores: the first `n_tokens` tokens of the workload's token stream
    through pool layer 0.  Only the routed experts are generated on the host (set-up is not timed)."""
    from oracle import moe_oracle as orc
    from paper_2407_14417_amd import synth
    x = synth.normal_f16((n_tokens, D), 1.0, seed, synth.x_stream(0))
    wg, bias, _ = host_layer(wl, seed, 0, ())
    idx, _ = orc.route(x, wg, K, bias)
    _, _, experts = host_layer(wl, seed, 0, sorted(set(int(e) for e in idx.reshape(-1))))
    T = wl["T"]
    t0 = time.perf_counter()
    for t in range(0, n_tokens, T):
        orc.layer_forward(x[t:t + T], wg, experts, K, bias)
    dt = time.perf_counter() - t0
    return {"value": n_tokens / dt, "unit": "tokens/s", "cores": orc.max_threads(), "kind": "oracle",
            "sample": f"first {n_tokens} tokens of the workload in calls of {min(T, n_tokens)}, pool layer 0, routed "
                      f"experts only, {dt:.1f} s of oracle time; OpenMP over output rows"}


# ---------------------------------------------------------------- workloads

def run_layer_workload(args, wl, mm, workload, torch, np, headline: bool):
    T, pool = wl["T"], (args.pool or wl["pool"])
    steps = (args.steps or wl["steps"]) if headline else wl["steps"]
    warmup = (args.warmup if args.warmup is not None else wl["warmup"]) if headline else wl["warmup"]
    layers = [workload.device_layer(D, F, E, K, wl["int4"], seed=args.seed, layer=l, router=wl["router"],
                                    zipf=wl["zipf"], int8_experts=wl.get("int8", ())) for l in range(pool)]
    n_tok = steps + warmup
    x_all = workload.device_tokens(n_tok * T, D, seed=args.seed).reshape(n_tok, T, D)
    out_all = torch.empty((n_tok, T, D), dtype=torch.float16, device="cuda")
    idx_all = torch.empty((n_tok, T, K), dtype=torch.int32, device="cuda")
    ws = mm.alloc_workspace(layers[0], T)
    torch.cuda.synchronize()

    def step(i: int) -> None:
        mm.moe_layer_forward(layers[i % pool], x_all[i], out_all[i], ws, idx_all[i], None)

    stream = torch.cuda.Stream()
    replay_ms, launch = timed_replays(torch, stream, step, warmup, steps, warmup, args.no_graph)
    assert mm.moe_read_status(ws) == 0
    stat = percentiles(replay_ms, steps)

    idx = idx_all[warmup:].cpu().numpy()
    per_step_bytes = np.array([workload.stored_bytes(layers[(warmup + j) % pool], idx[j].reshape(-1))
                               for j in range(steps)], dtype=np.float64)
    flops_per_step = 2.0 * 3.0 * D * F * T * K        # 2 flops per weight of w1, w3, w2 per routed (token, expert) pair
    sec = stat["median"] * 1e-3
    GBps = float(per_step_bytes.mean() / sec / 1e9)
    TFLOPs = float(flops_per_step / sec / 1e12)
    res = {
        "workload": wl["name"], "tokens_per_step": T, "pool_layers": pool, "launch": launch,
        "steps_per_replay": steps, "replays": len(replay_ms),
        "ms_per_step": stat["median"], "ms_per_step_p10": stat["p10"], "ms_per_step_p90": stat["p90"],
        "tokens_per_s": T / sec, "bytes_per_step": float(per_step_bytes.mean()), "flops_per_step": flops_per_step,
        "effective_weight_GBps": GBps, "TFLOPs": TFLOPs,
    }
    hbm_us = per_step_bytes.mean() / (HBM_PEAK_GBPS * 1e9) * 1e6
    mfma_us = flops_per_step / (MFMA_F16_PEAK_TFLOPS * 1e12) * 1e6
    if wl["bound"] == "hbm":
        res.update({"bound": "hbm", "roofline_us": hbm_us, "frac": GBps / HBM_PEAK_GBPS})
    else:
        res.update({"bound": "mfma", "roofline_us": max(hbm_us, mfma_us), "roofline_hbm_us": hbm_us,
                    "roofline_mfma_us": mfma_us, "frac": TFLOPs / MFMA_F16_PEAK_TFLOPS,
                    "frac_of_hbm_peak_on_bytes": GBps / HBM_PEAK_GBPS})
    if T == 1:
        n_int4 = np.array([sum(int(e) in wl["int4"] for e in idx[j, 0]) for j in range(steps)])
        if not wl.get("int8"):
            res["routed_pairs"] = {name: int((n_int4 == kind).sum())
                                   for kind, name in ((0, "fp16+fp16"), (1, "fp16+int4"), (2, "int4+int4"))}
    else:
        counts = np.stack([np.bincount(idx[j].reshape(-1), minlength=E) for j in range(steps)])
        res["rows_per_expert_mean"] = [float(c) for c in counts.mean(axis=0)]
        res["active_experts_mean"] = float((counts > 0).sum(axis=1).mean())

    roof = None
    if headline:
        # ---- roofline leg: the same steps, eagerly, the kernels of every step between HIP events
        traced = {"up": mm.KERNEL_UP, "down": mm.KERNEL_DOWN}
        if T > 1:                               # one token: the gating network runs inside the up-projection launch
            traced["route"] = mm.KERNEL_ROUTE
        with torch.cuda.stream(stream):
            pairs = {n: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                         for _ in range(steps)] for n in traced}
            for n in traced:                    # torch creates the hipEvent_t lazily, on the first record
                for a, b in pairs[n]:
                    a.record(stream)
                    b.record(stream)
            for j, i in enumerate(range(warmup, n_tok)):
                for n, kid in traced.items():
                    mm.moe_trace_kernel(kid, pairs[n][j][0].cuda_event, pairs[n][j][1].cuda_event)
                step(i)
            stream.synchronize()
        for kid in traced.values():             # nothing stays armed for the captures of the next legs
            mm.moe_trace_kernel(kid, None, None)
        ms = {n: np.array([a.elapsed_time(b) for a, b in pairs[n]]) for n in traced}
        gate_bytes = E * D * 2
        # up-projection: w1 and w3 of the routed experts = 2/3 of their stored bytes; down-projection: w2 = 1/3
        up_bytes = (per_step_bytes - gate_bytes) * (2.0 / 3.0)
        down_bytes = (per_step_bytes - gate_bytes) * (1.0 / 3.0)
        up_ms, down_ms = ms["up"], ms["down"]
        up_flops, down_flops = flops_per_step * 2.0 / 3.0, flops_per_step / 3.0
        up_GBps = float(up_bytes.sum() / (up_ms.sum() * 1e-3) / 1e9)
        up_TFLOPs = float(up_flops * steps / (up_ms.sum() * 1e-3) / 1e12)
        other = {"down_projection": {"avg_launch_us": float(down_ms.mean() * 1e3),
                                     "GBps": float(down_bytes.sum() / (down_ms.sum() * 1e-3) / 1e9),
                                     "TFLOPs": float(down_flops * steps / (down_ms.sum() * 1e-3) / 1e12)},
                 "route": {"avg_launch_us": float(ms["route"].mean() * 1e3)} if "route" in ms else
                 "inside the up-projection launch (one token)"}
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
        prof = {"decode": "decode_b1_hbm_traffic.md", "batched": "batched_int4_hbm_traffic_and_counters.md",
                "prefill": "prefill_hbm_traffic_and_counters.md"}.get(args.workload, "none")
        ratio = traffic_ratio(prof, "up_projection")
        if ratio is not None:
            roof["traffic"] = ratio * float(up_bytes.mean())          # bytes per launch, like `achieved`
            roof["traffic_source"] = f"profiles/{prof} (rocprofv3 --pmc FETCH_SIZE, copy-calibrated): " \
                                     f"fetched/algorithmic = {ratio}"
        roof["algorithmic_bytes_per_launch"] = float(up_bytes.mean())
        if T == 1 and not wl.get("int8"):
            by_pair = {}
            for kind, name in ((0, "fp16+fp16"), (1, "fp16+int4"), (2, "int4+int4")):
                sel = n_int4 == kind
                if sel.any():
                    by_pair[name] = {"launches": int(sel.sum()), "avg_us": float(up_ms[sel].mean() * 1e3),
                                     "GBps": float(up_bytes[sel].sum() / (up_ms[sel].sum() * 1e-3) / 1e9),
                                     "down_avg_us": float(down_ms[sel].mean() * 1e3),
                                     "down_GBps": float(down_bytes[sel].sum() / (down_ms[sel].sum() * 1e-3) / 1e9)}
            roof["by_pair"] = by_pair
        roof["other_kernels"] = other

    if args.parity != "none":
        j = warmup                                    # the first timed step
        x_host = x_all[j].cpu().numpy()
        idx_dev = idx_all[j].cpu().numpy()
        if T <= 16:
            tokens = list(range(T))
        else:                                         # a sample that covers every expert
            tokens = sorted(set(int(np.argwhere((idx_dev == e).any(axis=1))[0, 0]) for e in range(E)
                                if (idx_dev == e).any()) | set(range(0, T, T // 8)))
        res["parity"] = layer_parity(wl, args.seed, j % pool, x_host, idx_dev, out_all[j].cpu().numpy(), tokens)
    return res, roof


def run_chain_workload(args, wl, mm, workload, torch, np, headline: bool):
    from paper_2407_14417_amd import synth
    L = wl["layers"]
    steps = (args.steps or wl["steps"]) if headline else wl["steps"]
    warmup = (args.warmup if args.warmup is not None else wl["warmup"]) if headline else wl["warmup"]
    mask = synth.precision_mask(E * L, E * L // 2, args.seed)
    layers = []
    for l in range(L):
        layers.append(workload.device_layer(D, F, E, K, tuple(e for e in range(E) if mask[l * E + e]),
                                            seed=args.seed, layer=l))
    gains = [torch.ones(D, dtype=torch.float16, device="cuda") for _ in range(L)]
    chain = mm.Chain(layers, gains)
    n_tok = steps + warmup
    h_src = workload.device_tokens(n_tok, D, seed=args.seed).reshape(n_tok, 1, D)
    h_all = torch.empty_like(h_src)
    idx_all = torch.empty((n_tok, L, 1, K), dtype=torch.int32, device="cuda")
    ws = mm.alloc_workspace(layers[0], 1)
    torch.cuda.synchronize()

    def step(i: int) -> None:
        h_all[i].copy_(h_src[i])                 # the chain updates h in place: every replay starts from the token
        mm.moe_chain_forward(chain, 1e-5, h_all[i], ws, idx_all[i])

    stream = torch.cuda.Stream()
    replay_ms, launch = timed_replays(torch, stream, step, warmup, steps, warmup, args.no_graph)
    assert mm.moe_read_status(ws) == 0
    stat = percentiles(replay_ms, steps)
    idx = idx_all[warmup:].cpu().numpy()
    per_step_bytes = np.array([sum(workload.stored_bytes(layers[l], idx[j, l, 0]) for l in range(L))
                               for j in range(steps)], dtype=np.float64)
    sec = stat["median"] * 1e-3
    GBps = float(per_step_bytes.mean() / sec / 1e9)
    res = {
        "workload": wl["name"], "tokens_per_step": 1, "layers": L,
        "resident_GB": float(sum(e.nbytes() for l in layers for e in l.experts) / 1e9), "launch": launch,
        "steps_per_replay": steps, "replays": len(replay_ms),
        "ms_per_step": stat["median"], "ms_per_step_p10": stat["p10"], "ms_per_step_p90": stat["p90"],
        "tokens_per_s": 1.0 / sec, "bytes_per_step": float(per_step_bytes.mean()),
        "flops_per_step": 2.0 * 3.0 * D * F * K * L, "effective_weight_GBps": GBps,
        "bound": "hbm", "roofline_us": per_step_bytes.mean() / (HBM_PEAK_GBPS * 1e9) * 1e6,
        "frac": GBps / HBM_PEAK_GBPS,
    }
    if args.parity != "none":
        # the first two blocks of the first timed step, run on their own, against the oracle's chain
        from oracle import moe_oracle as orc
        t0 = time.perf_counter()
        n_check = 2
        h_chk = h_src[warmup].clone()
        idx_chk = torch.empty((n_check, 1, K), dtype=torch.int32, device="cuda")
        mm.moe_chain_forward(mm.Chain(layers[:n_check], gains[:n_check]), 1e-5, h_chk, ws, idx_chk)
        h_ref = h_src[warmup].cpu().numpy()
        g = np.ones(D, dtype=np.float16)
        same = True
        for l in range(n_check):
            lw = dict(wl, int4=tuple(e for e in range(E) if mask[l * E + e]), router="normal", zipf=None)
            wg, _, _ = host_layer(lw, args.seed, l, ())
            ridx, _ = orc.route(orc.rmsnorm(h_ref, g, 1e-5), wg, K)
            _, _, experts = host_layer(lw, args.seed, l, sorted(set(int(e) for e in ridx.reshape(-1))))
            h_ref, ridx2, _, _ = orc.chain_layer(h_ref, g, 1e-5, wg, experts, K)
            same = same and bool(np.array_equal(idx_chk[l].cpu().numpy(), ridx2))
        res["parity"] = parity_metrics(h_chk.cpu().numpy(), h_ref)
        res["parity"].update({"routing_indices_equal": same, "layers_checked": n_check,
                              "oracle_s": round(time.perf_counter() - t0, 1)})
    roof = {"bound": "hbm", "kernel": "whole step (32 x gating, up-projection, down-projection)",
            "achieved": GBps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": GBps / HBM_PEAK_GBPS,
            "traffic": None, "bytes_per_step_GB": float(per_step_bytes.mean() / 1e9)} if headline else None
    return res, roof


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
    res = {
        "workload": wl["name"], "tokens_per_step": 1, "pool_layers": pool, "launch": "eager (host round trip inside)",
        "steps_per_replay": steps, "replays": 1, "ms_per_step": elapsed / steps * 1e3,
        "tokens_per_s": steps / elapsed, "mem_budget_MB": args.mem_mb, "num_e4": int(plan.num_e4),
        "resident_e4": int(plan.resident_e4), "resident_e16": int(plan.resident_e16), "swap_slots": args.slots,
        "resident_MB": plan.bytes_resident / 1e6, "expert_misses_per_token": misses / steps,
    }
    roof = {"bound": "pcie", "kernel": "host-to-device copy of missed experts", "achieved": None, "peak": None,
            "unit": "GB/s", "frac": None, "traffic": None}
    return res, roof


def stream_ceiling(mm, torch):
    """Plain streaming-read kernel (moe_stream_read) at the byte counts of the up-projection of a 4-bit pair
    (132 MB) and of a 16-bit pair (470 MB), rotating over a 4 GiB buffer so that no cache level serves it;
    median of 20 launches, each between two HIP events recorded inside the library call right around the launch
    (the same way the up-projection launches of the roofline leg are timed)."""
    import numpy as np
    total = 4 << 30
    buf = torch.empty(total, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for label, nbytes in (("132MB", 132_120_576), ("470MB", 469_762_048)):
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(24)]
            for a, b in pairs:                  # torch creates the hipEvent_t lazily, on the first record
                a.record(stream)
                b.record(stream)
            for r, (a, b) in enumerate(pairs):
                off = (r * 977 * (1 << 20)) % (total - nbytes) // 65536 * 65536
                mm.moe_trace_kernel(mm.KERNEL_STREAM_READ, a.cuda_event, b.cuda_event)
                mm.moe_stream_read(buf[off:], nbytes, sink)
            stream.synchronize()
            med = float(np.median([a.elapsed_time(b) for a, b in pairs[4:]]))
            out[label] = {"bytes": nbytes, "median_us": med * 1e3, "GBps": nbytes / (med * 1e-3) / 1e9,
                          "frac_of_8TBps": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    del buf
    torch.cuda.empty_cache()
    return out


def run_one(name, args, mm, workload, torch, np, headline):
    wl = dict(WORKLOADS[name])
    if headline and args.int4_experts is not None and "int4" in wl:       # measurement variant: another mask
        wl["int4"] = tuple(int(e) for e in args.int4_experts.split(",") if e != "")
        wl["name"] += f" [precision mask overridden: 4-bit experts {list(wl['int4'])}]"
    if name == "chain":
        res, roof = run_chain_workload(args, wl, mm, workload, torch, np, headline)
    elif name == "offload":
        res, roof = run_offload_workload(args, wl, mm, workload, torch, np)
    else:
        res, roof = run_layer_workload(args, wl, mm, workload, torch, np, headline)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return wl, res, roof


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps per replay of the headline workload (0 = default)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="decode", help="the headline workload")
    ap.add_argument("--configs", default="all",
                    help="'all', 'none' or a comma-separated subset of " + ",".join(EXTRA_CONFIGS) +
                         ": the other workloads reported under `configs` in the same line")
    ap.add_argument("--parity", choices=("sample", "none"), default="sample",
                    help="check one step of every workload against the CPU oracle")
    ap.add_argument("--pool", type=int, default=0, help="independent layers the steps rotate over (0 = default)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--cpu-tokens", type=int, default=-1, help="oracle sample size (0 = skip, -1 = default)")
    ap.add_argument("--int4-experts", default=None,
                    help="comma-separated expert indices that are 4-bit instead of the headline workload's own mask")
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
    t_start = time.perf_counter()
    wl, res, roof = run_one(args.workload, args, mm, workload, torch, np, headline=True)

    if args.configs == "all":
        extra = [c for c in EXTRA_CONFIGS if c != args.workload]
    elif args.configs == "none":
        extra = []
    else:
        extra = [c for c in args.configs.split(",") if c]
        for c in extra:
            if c not in EXTRA_CONFIGS:
                print(f"bench.py: unknown config {c!r}", file=sys.stderr)
                return 2
    configs = {}
    for c in extra:
        t0 = time.perf_counter()
        _, cres, _ = run_one(c, args, mm, workload, torch, np, headline=False)
        cres["leg_wall_s"] = round(time.perf_counter() - t0, 1)
        configs[c] = cres

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    result = {
        "metric": "MoE-layer tokens/s + effective weight HBM GB/s (% of peak), Mixtral shape",
        "value": res["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": res["steps_per_replay"],
        "warmup": args.warmup if args.warmup is not None else wl["warmup"],
        "ms_per_step": res["ms_per_step"],
        "ms_per_step_p10": res.get("ms_per_step_p10"),
        "ms_per_step_p90": res.get("ms_per_step_p90"),
        "replays": res["replays"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 (products of f16 weights and activations accumulated in f32; uint4-g64 weights expanded to f16)",
        "data": "synthetic",
        "config": {k: res[k] for k in ("workload", "tokens_per_step", "pool_layers", "layers", "launch") if k in res},
    }
    for k in ("effective_weight_GBps", "TFLOPs", "bytes_per_step", "flops_per_step", "bound", "roofline_us", "frac",
              "routed_pairs", "rows_per_expert_mean", "active_experts_mean", "parity", "expert_misses_per_token"):
        if k in res:
            result["step_level_frac_of_peak" if k == "frac" else k] = res[k]
    if "effective_weight_GBps" in res:
        result["pct_of_hbm_peak"] = res["effective_weight_GBps"] / HBM_PEAK_GBPS * 100.0
    result["roofline"] = roof
    if configs:
        result["configs"] = configs
    if args.configs != "none":
        result["stream_ceiling"] = stream_ceiling(mm, torch)
    cpu_tokens = args.cpu_tokens
    if cpu_tokens < 0:
        cpu_tokens = {"decode": 48, "decode_int4_only": 48, "decode_fp16_only": 24, "decode_int8_only": 32, "batched": 48,
                      "prefill": 64, "chain": 0, "offload": 0}[args.workload]
    if cpu_tokens > 0 and "int4" in wl:
        result["cpu_baseline"] = cpu_baseline(wl, args.seed, cpu_tokens)
    result["bench_wall_s"] = round(time.perf_counter() - t_start, 1)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
