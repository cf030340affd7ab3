#!/usr/bin/env python3
"""MoE-layer throughput of the HIP path on one MI355X, with roofline and CPU-oracle baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tokens T] [--beta B]

One step = one pass of the whole hot path (predict, horizon, prefetch, route, grouping, miss
swap-in, grouped FFN, un-permute, bookkeeping) over every layer of the workload for one batch of
T tokens.  `value` = MoE-layer tokens/s = T * layers * steps / wall time (tokens through one MoE
layer per second), inputs resident in HBM, expert store in pinned host memory, cache warmed by
the warm-up steps.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# workload name -> (config, tokens, beta tuned for stall < 5 %)
WORKLOADS = {
    "mixtral_decode": ("mixtral_decode", 64, 16.0),
    "mixtral_prefill": ("mixtral_prefill", 8192, 0.0),
    "deepseek_v2_lite": ("deepseek_v2_lite", 32, 2.0),
    "qwen15_moe": ("qwen15_moe", 640, 2.0),
    "tiny": ("tiny", 64, 0.5),
}


def cpu_baseline(cfg, T, beta, budget_tokens):
    """The oracle, as it stands, on a bounded sample of the same workload: routing of all T tokens
    of one layer plus the expert FFN of `budget_tokens` of them; tokens/s scaled to the sample."""
    import numpy as np
    import oracle
    from paper_2510_26730_amd import synth
    oracle.build()
    h = synth.hidden(cfg, 0, T)
    Wg, b = synth.gate_weight(cfg, 0), synth.gate_bias(cfg, 0)
    res = synth.residency(cfg, 0)
    n = min(budget_tokens, T)
    toks = np.arange(n)
    t0 = time.perf_counter()
    r = oracle.route(h, Wg, b, cfg.k, beta, res, renorm=cfg.renorm)
    t_route = time.perf_counter() - t0
    ids_s = np.ascontiguousarray(r["ids"][toks])
    used = sorted(set(ids_s.ravel().tolist()))
    experts = [synth.expert_weights(cfg, 0, e) if e in used else None for e in range(cfg.E)]   # untimed: input generation
    shared = synth.shared_weights(cfg, 0)
    t0 = time.perf_counter()
    sub = oracle.route_from_ids(r["p"][toks], ids_s, cfg.E, cfg.renorm)
    y = oracle.expert_ffn(np.ascontiguousarray(h[toks]), experts, ids_s, sub["perm"])
    sh = None if shared is None else oracle.dense_ffn(np.ascontiguousarray(h[toks]), *shared)
    oracle.combine(y, sub["w"], sub["inv_perm"], sh)
    t_ffn = time.perf_counter() - t0
    per_token = t_route / T + t_ffn / n
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": 1.0 / per_token, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"one layer: routing of {T} tokens ({t_route:.2f} s) + expert FFN and combine of {n} "
                      f"tokens ({t_ffn:.2f} s), fp64, OpenMP over tokens"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="mixtral_decode", choices=sorted(WORKLOADS))
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--beta", type=float, default=None)
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--all-resident", action="store_true", help="cache holds every expert (no PCIe traffic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU hot path; run with --gpus 1 "
              "(no sharding or collectives are part of it)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_26730_amd import binding as ef
    from paper_2510_26730_amd import synth
    from paper_2510_26730_amd.runner import LayerLoop
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    ef.lib()          # fail loudly if the HIP library is not built

    cfg_name, T, beta = WORKLOADS[args.workload]
    cfg = synth.CONFIGS[cfg_name]
    T = args.tokens or T
    beta = beta if args.beta is None else args.beta
    L = args.layers or cfg.n_layers
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    loop = LayerLoop(cfg, L, T, cfg.slots_per_layer, beta=beta, profile=False, all_resident=args.all_resident)
    n_in = 4                                          # distinct step inputs, cycled
    hs = [torch.from_numpy(synth.hidden_stack(cfg, L, step=s, T=T).view("int16")).cuda() for s in range(n_in)]
    torch.cuda.synchronize()

    def kernel_table(st, wall):
        out = {}
        for i, name in enumerate(ef.EF_KERNELS):
            n = st["kernel_launches"][i]
            if n:
                sec, byt = st["kernel_seconds"][i], st["kernel_bytes"][i]
                out[name] = {"launches": n, "avg_us": 1e6 * sec / n, "alg_bytes_per_launch": byt / n,
                             "GBps": byt / sec / 1e9 if sec > 0 else None, "share_of_step_time": sec / wall}
        return out

    for s in range(args.warmup):
        loop.step(hs[s % n_in], stream)
    torch.cuda.synchronize()
    # timed region: only the dominant kernel (first FFN half) is bracketed with HIP events, on the
    # stream it is launched on
    ef.ef_set_profile(loop.ctx, 1 << ef.EF_KERNELS.index("ffn_up"))
    ef.ef_reset_stats(loop.ctx)
    t0 = time.perf_counter()
    for s in range(args.steps):
        loop.step(hs[(args.warmup + s) % n_in], stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = ef.ef_get_stats(loop.ctx)
    dom = kernel_table(st, dt).get("ffn_up")

    # separate, untimed pass with every kernel bracketed: the per-kernel breakdown
    ef.ef_set_profile(loop.ctx, 0xFF)
    ef.ef_reset_stats(loop.ctx)
    t1 = time.perf_counter()
    for s in range(2):
        loop.step(hs[s % n_in], stream)
    torch.cuda.synchronize()
    kern = kernel_table(ef.ef_get_stats(loop.ctx), time.perf_counter() - t1)

    layer_tokens = T * L * args.steps
    value = layer_tokens / dt
    roof = None
    if dom:
        a = dom["GBps"]
        roof = {"bound": "hbm", "kernel": "ffn_gate_up_kernel", "achieved": a, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": a / HBM_PEAK_GBPS, "traffic": None,
                "avg_launch_us": dom["avg_us"], "alg_bytes_per_launch": dom["alg_bytes_per_launch"],
                "launches": dom["launches"], "share_of_step_time": dom["share_of_step_time"]}
    result = {
        "metric": "MoE-layer tokens/s (route+predict+FFN) at 1 GPU",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layers, d={cfg.d}, E={cfg.E}, top-{cfg.k}, F={cfg.F}, "
                               f"T={T} tokens/step, cache {'all experts' if args.all_resident else str(cfg.slots_per_layer) + ' slots/layer'}"
                               f", beta={beta}, expert store = {loop.store_layers}-layer pinned pool reused cyclically",
                   "tokens_per_step": T, "layers": L, "beta": beta},
        "us_per_layer": 1e6 * dt / (L * args.steps),
        "stall_frac": st["stall_seconds"] / dt,
        "cache": {"hits": st["hits"], "misses": st["misses"], "miss_rate": st["miss_rate"],
                  "prefetch_issued": st["prefetch_issued"], "bytes_copied": st["bytes_copied"],
                  "pcie_GBps": st["bytes_copied"] / st["copy_seconds"] / 1e9 if st["copy_seconds"] > 0 else None,
                  "horizon": st["horizon"], "bandwidth_est_GBps": st["bandwidth_Bps"] / 1e9,
                  "layer_est_us": st["layer_seconds_est"] * 1e6},
        "kernels": kern,
        "roofline": roof,
    }
    loop.close()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, T, beta, args.cpu_tokens)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
