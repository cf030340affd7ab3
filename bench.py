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
MFMA_BF16_PEAK_TFLOPS = 2500.0          # dense bf16, no structured sparsity

# workload name -> (config, tokens, beta tuned for stall < 5 %)
WORKLOADS = {
    "mixtral_decode": ("mixtral_decode", 64, 16.0),
    "mixtral_prefill": ("mixtral_prefill", 8192, 0.0),
    "deepseek_v2_lite": ("deepseek_v2_lite", 32, 6.0),
    "qwen15_moe": ("qwen15_moe", 640, 8.0),
    "tiny": ("tiny", 64, 0.5),
}


def cpu_baseline(cfg, T, beta, target_seconds):
    """The oracle, as it stands, on a bounded sample of the same workload: whole passes (routing,
    expert FFN, combine) over ONE layer of the workload at its real shape, for up to T tokens,
    repeated until about `target_seconds` of CPU time have been spent."""
    import numpy as np
    import oracle
    from paper_2510_26730_amd import synth
    oracle.build()
    n = min(T, 64)                       # tokens whose FFN is evaluated per pass
    h = synth.hidden(cfg, 0, T)
    Wg, b = synth.gate_weight(cfg, 0), synth.gate_bias(cfg, 0)
    res = synth.residency(cfg, 0)
    r0 = oracle.route(h, Wg, b, cfg.k, beta, res, renorm=cfg.renorm)
    used = sorted(set(r0["ids"][:n].ravel().tolist()))
    experts = [synth.expert_weights(cfg, 0, e) if e in used else None for e in range(cfg.E)]   # untimed: inputs
    shared = synth.shared_weights(cfg, 0)
    hs = np.ascontiguousarray(h[:n])

    def one_pass():
        t0 = time.perf_counter()
        r = oracle.route(h, Wg, b, cfg.k, beta, res, renorm=cfg.renorm)
        t_route = time.perf_counter() - t0
        t0 = time.perf_counter()
        ids_s = np.ascontiguousarray(r["ids"][:n])
        sub = oracle.route_from_ids(r["p"][:n], ids_s, cfg.E, cfg.renorm)
        y = oracle.expert_ffn(hs, experts, ids_s, sub["perm"])
        sh = None if shared is None else oracle.dense_ffn(hs, *shared)
        oracle.combine(y, sub["w"], sub["inv_perm"], sh)
        return t_route, time.perf_counter() - t0

    tr, tf = one_pass()
    reps = int(max(1, min(64, target_seconds / max(tr + tf, 1e-3))))
    tot_r, tot_f = tr, tf
    for _ in range(reps - 1):
        a, c = one_pass()
        tot_r += a
        tot_f += c
    per_token = tot_r / (reps * T) + tot_f / (reps * n)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": 1.0 / per_token, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} passes over one layer at full shape: routing of {T} tokens ({tot_r:.2f} s) + expert "
                      f"FFN and combine of {n} tokens ({tot_f:.2f} s); fp64, OpenMP over tokens"}


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
    ap.add_argument("--int4", action="store_true",
                    help="4-bit expert weights (code and bf16 scale per 128 inputs) instead of bf16: a variant "
                         "beside the headline workload, 4x fewer bytes per expert over PCIe and from HBM")
    ap.add_argument("--slots", type=int, default=None, help="cache slots per layer (default: the workload's quota)")
    ap.add_argument("--pool-slots", type=int, default=None,
                    help="one global pool of this many cache slots shared by all layers instead of a per-layer quota")
    ap.add_argument("--horizon", type=int, default=None, help="fixed look-ahead H (default: the adaptive horizon)")
    ap.add_argument("--drift-tokens", type=int, default=0,
                    help="re-draw the expert popularity ranks (gate biases) whenever the running token count "
                         "crosses a multiple of this (0 = static popularity)")
    ap.add_argument("--delta-forest", action="store_true",
                    help="measure the deviation predictor instead of the headline: activation logs of recurring "
                         "prompts -> random forest on the host -> look-ahead recall with and without its deviation, "
                         "and the layer loop's rate with the deviation path switched on")
    ap.add_argument("--prompts", type=int, default=256, help="--delta-forest: size of the pool of recurring prompts")
    ap.add_argument("--log-steps", type=int, default=24, help="--delta-forest: steps whose routing is logged for training")
    ap.add_argument("--eval-steps", type=int, default=6, help="--delta-forest: fresh steps the look-ahead is scored on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle baseline")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="MiB of a plain device-to-device copy done 4 times before the run (a kernel of known "
                         "traffic, used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
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
    if args.calib_copy > 0:
        src = torch.empty(args.calib_copy << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.delta_forest:
        from paper_2510_26730_amd import delta_bench
        L = args.layers or 8
        H = args.horizon or 3
        r = delta_bench.run(cfg, T, L, H, args.prompts, args.steps, args.warmup, args.log_steps, args.eval_steps)
        w = r["layer_loop_with_delta"]
        print(json.dumps({
            "metric": "MoE-layer tokens/s (route+predict+FFN) at 1 GPU, look-ahead refined by the host forest's deviation",
            "value": w["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": 1e-3 * w["us_per_layer"] * L, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": r["workload"], "tokens_per_step": T, "layers": L, "horizon": H},
            "delta_forest": r}))
        return

    slots = args.slots or cfg.slots_per_layer
    loop = LayerLoop(cfg, L, T, slots, pool_slots=args.pool_slots, beta=beta, profile=False,
                     all_resident=args.all_resident, q4=args.int4)
    loop.h_fixed = args.horizon
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
                flops = st["kernel_flops"][i]
                if flops > 0:
                    out[name]["alg_flops_per_launch"] = flops / n
                    out[name]["TFLOPps"] = flops / sec / 1e12 if sec > 0 else None
        return out

    # popularity drift: a new permutation of the Zipf ranks per epoch, written into the registered bias
    # buffers (E floats per layer, host arrays prepared before the timed region)
    drift = {"tokens": 0, "epoch": 0}
    n_epochs = 1 + ((args.warmup + args.steps + 2) * T) // args.drift_tokens if args.drift_tokens > 0 else 1
    bias_epochs = [[torch.from_numpy(synth.gate_bias(cfg, l, ep)).pin_memory() for l in range(L)]
                   for ep in range(1, n_epochs + 1)] if args.drift_tokens > 0 else []

    def run_step(h):
        if args.drift_tokens > 0:
            drift["tokens"] += T
            ep = drift["tokens"] // args.drift_tokens
            if ep != drift["epoch"]:
                drift["epoch"] = ep
                for l in range(L):
                    loop.gate_b[l].copy_(bias_epochs[(ep - 1) % len(bias_epochs)][l], non_blocking=True)
        loop.step(h, stream)

    for s in range(args.warmup):
        run_step(hs[s % n_in])
    torch.cuda.synchronize()
    # timed region: only the dominant kernel is bracketed with HIP events, on the stream it is launched
    # on: the weight-streaming first FFN half when experts see few tokens (decode), its matrix-core
    # tiled form when they see hundreds (prefill)
    ntile_avg = T * cfg.k / max(1, cfg.E) / 32.0
    dom_name = "ffn_up_tiled" if ntile_avg >= 8 else "ffn_up"
    ef.ef_set_profile(loop.ctx, 1 << ef.EF_KERNELS.index(dom_name))
    # every 4th launch of it (events between kernels cost the stream 2-3 us each); with fewer than 64 launches
    # in the timed region, every launch
    ef.ef_set_profile_sampling(loop.ctx, 4 if L * args.steps >= 64 else 1)
    ef.ef_reset_stats(loop.ctx)
    t0 = time.perf_counter()
    marks = []
    for s in range(args.steps):
        run_step(hs[(args.warmup + s) % n_in])
        marks.append(time.perf_counter())     # the host runs at most one layer ahead of the GPU (it waits
    torch.cuda.synchronize()                  # for every layer's counts), so these bound each step's time
    dt = time.perf_counter() - t0
    marks[-1] = t0 + dt
    per_step = sorted(1e3 * (b - a) for a, b in zip([t0] + marks[:-1], marks))
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    st = ef.ef_get_stats(loop.ctx)
    dom = kernel_table(st, dt).get(dom_name)

    # separate, untimed pass with every kernel bracketed: the per-kernel breakdown
    ef.ef_set_profile(loop.ctx, 0x3FF)
    ef.ef_set_profile_sampling(loop.ctx, 1)
    ef.ef_reset_stats(loop.ctx)
    t1 = time.perf_counter()
    tok_dist = torch.empty(T, dtype=torch.float32, device="cuda")
    dist = torch.zeros(1, dtype=torch.float64, device="cuda")
    ef.ef_token_dist(loop.ctx, hs[0][0], T, tok_dist, dist, stream)     # first call loads the kernels
    torch.cuda.synchronize()
    ef.ef_reset_stats(loop.ctx)
    t1 = time.perf_counter()
    for s in range(2):
        # the intra-batch diversity signal of the iteration's tokens (once per step, outside `value`)
        ef.ef_token_dist(loop.ctx, hs[s % n_in][0], T, tok_dist, dist, stream)
        loop.step(hs[s % n_in], stream)
    torch.cuda.synchronize()
    kern = kernel_table(ef.ef_get_stats(loop.ctx), time.perf_counter() - t1)

    layer_tokens = T * L * args.steps
    value = layer_tokens / dt
    roof = None
    if dom and dom_name == "ffn_up_tiled":
        a = dom["TFLOPps"]
        roof = {"bound": "mfma", "kernel": "ffn_gate_up_tiled_kernel", "achieved": a, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": a / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                "avg_launch_us": dom["avg_us"], "alg_flops_per_launch": dom["alg_flops_per_launch"],
                "launches": dom["launches"], "share_of_step_time": dom["share_of_step_time"]}
    elif dom:
        a = dom["GBps"]
        # HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE scaled by
        # a copy kernel), only if it was taken on this very workload; a counter run cannot happen in here
        traffic = None
        tag = f"TRAFFIC_BYTES_PER_LAUNCH ffn_gate_up_kernel {cfg.name} T={T} beta={beta} ="
        pmc = os.path.join(ROOT, "profiles", "ffn_kernels_mixtral_decode_T64_pmc_traffic.md")
        if os.path.exists(pmc) and not args.all_resident and args.pool_slots is None and not args.int4:
            for line in open(pmc):
                if line.startswith(tag):
                    traffic = float(line.split("=")[-1])
        roof = {"bound": "hbm", "kernel": "ffn_gate_up_kernel", "achieved": a, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": a / HBM_PEAK_GBPS, "traffic": traffic,
                "avg_launch_us": dom["avg_us"], "alg_bytes_per_launch": dom["alg_bytes_per_launch"],
                "launches": dom["launches"], "share_of_step_time": dom["share_of_step_time"]}
    result = {
        "metric": "MoE-layer tokens/s (route+predict+FFN) at 1 GPU",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 (4-bit expert weights dequantised to fp16, fp32 accumulation)" if args.int4 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layers, d={cfg.d}, E={cfg.E}, top-{cfg.k}, F={cfg.F}, "
                               f"T={T} tokens/step, cache {'all experts' if args.all_resident else (str(args.pool_slots) + '-slot pool' if args.pool_slots else str(slots) + ' slots/layer')}"
                               f"{', 4-bit experts' if args.int4 else ''}, beta={beta}, expert store = {loop.store_layers}-layer pinned pool reused cyclically",
                   "tokens_per_step": T, "layers": L, "beta": beta,
                   "horizon": "adaptive" if args.horizon is None else args.horizon,
                   "drift_tokens": args.drift_tokens},
        "us_per_layer": 1e6 * dt / (L * args.steps),
        "ms_per_step_p10_p50_p90": [pct(0.1), pct(0.5), pct(0.9)],
        "stall_frac": st["stall_seconds"] / dt,
        "cache": {"hits": st["hits"], "misses": st["misses"], "miss_rate": st["miss_rate"],
                  "prefetch_issued": st["prefetch_issued"], "bytes_copied": st["bytes_copied"],
                  "pcie_GBps": st["bytes_timed"] / st["copy_seconds"] / 1e9 if st["copy_seconds"] > 0 else None,
                  "horizon": st["horizon"], "bandwidth_est_GBps": st["bandwidth_Bps"] / 1e9,
                  "layer_est_us": st["layer_seconds_est"] * 1e6},
        "kernels": kern,
        "token_dist": float(dist.cpu()[0]),
        "roofline": roof,
    }
    loop.close()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, T, beta, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
