#!/usr/bin/env python3
"""MoE-layer throughput of the HIP path on one MI355X, with roofline and CPU-oracle baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tokens T] [--beta B] ...

One step = one pass of the whole hot path (predict, horizon, prefetch, route, grouping, miss
swap-in, grouped FFN, un-permute, bookkeeping) over every layer of the workload for one batch of
T tokens.  `value` = MoE-layer tokens/s = T * layers * steps / wall time (tokens through one MoE
layer per second), inputs resident in HBM, expert store in pinned host memory, cache warmed by
the warm-up steps.  Prints ONE JSON line: the top-level fields are the headline workload
(BASELINE configuration 2, the one the metric is quoted on); `workloads` carries the same
measurement for every BASELINE configuration (1-5, configuration 4 at both of its batch shapes)
plus operating points with misses and prefetches.  With --workload NAME only that one is run.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0          # dense bf16 / fp16, no structured sparsity

# name -> synth config, BASELINE configuration, tokens per step, beta (tuned for stall < 5 % unless the note says
# otherwise), options, (steps, warmup) of the default run, note
WORKLOADS = {
    "mixtral_decode": dict(cfg="mixtral_decode", baseline_config=2, T=64, beta=16.0, steps=12, warmup=4,
                           note="headline: decode batch, 2 of 8 experts per layer in HBM"),
    "tiny": dict(cfg="tiny", baseline_config=1, T=64, beta=0.5, steps=12, warmup=4, note="4 of 8 slots"),
    "mixtral_prefill": dict(cfg="mixtral_prefill", baseline_config=3, T=8192, beta=16.0, steps=3, warmup=2,
                            note="4 x 2048-token prompts, 4 of 8 experts per layer in HBM"),
    "deepseek_decode": dict(cfg="deepseek_v2_lite", baseline_config=4, T=32, beta=6.0, steps=12, warmup=4,
                            note="32 decode tokens, 16 of 64 slots per layer"),
    "deepseek_decode_beta4": dict(cfg="deepseek_v2_lite", baseline_config=4, T=32, beta=4.0, steps=12, warmup=6,
                                  note="operating point with a few misses per step (lower residency bias)"),
    "deepseek_decode_beta3": dict(cfg="deepseek_v2_lite", baseline_config=4, T=32, beta=3.0, steps=12, warmup=6,
                                  note="hit rate 97-98 %: the band in which the look-ahead issues prefetches every few "
                                       "layers and the link still has room (no-prediction and fixed horizons: DESIGN)"),
    "deepseek_mixed": dict(cfg="deepseek_v2_lite", baseline_config=4, T=1056, beta=8.0, steps=6, warmup=3,
                           note="1024 prefill + 32 decode tokens, 16 of 64 slots per layer"),
    "qwen_mixed": dict(cfg="qwen15_moe", baseline_config=5, T=640, beta=8.0, steps=8, warmup=4,
                       note="128 decode + 512 prefill tokens, 12 of 60 slots per layer, static popularity"),
    "qwen_mixed_drift": dict(cfg="qwen15_moe", baseline_config=5, T=640, beta=8.0, steps=6, warmup=3, drift_tokens=256,
                             note="popularity ranks re-drawn every 256 tokens (every step): the resident set must be "
                                  "replaced each step, the link is saturated whatever the look-ahead"),
}
DEFAULT_SET = ["mixtral_decode", "tiny", "mixtral_prefill", "deepseek_decode", "deepseek_decode_beta4", "deepseek_decode_beta3",
               "deepseek_mixed",
               "qwen_mixed", "qwen_mixed_drift"]
# kernel kind -> (what bounds it, name in the roofline object)
KIND_BOUND = {"ffn_up": ("hbm", "ffn_gate_up_kernel (weight streaming)"), "ffn_down": ("hbm", "ffn_down_kernel (weight streaming)"),
              "ffn_up_tiled": ("mfma", "ffn_gate_up_tiled_kernel"), "ffn_down_tiled": ("mfma", "ffn_down_tiled_kernel"),
              "route": ("hbm", "gate_kernel (+ second step / grouping)"), "predict": ("hbm", "gate_kernel (look-ahead gates)"),
              "group": ("hbm", "group kernels"), "pack": ("hbm", "pack_x_kernel"), "combine": ("hbm", "combine_kernel")}


def omp_threads(n):
    """Thread count of the oracle's OpenMP regions (its library has no setter of its own)."""
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def cpu_baseline(cfg, T, beta, target_seconds, n_tokens=64, threads=None):
    """The oracle, as it stands, on a bounded sample of the same workload: whole passes (routing,
    expert FFN, combine) over ONE layer of the workload at its real shape, for up to n_tokens tokens,
    repeated until about `target_seconds` of CPU time have been spent."""
    import numpy as np
    import oracle
    from paper_2510_26730_amd import synth
    oracle.build()
    all_cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    cores = all_cores if threads is None else threads
    if not omp_threads(cores):
        cores = all_cores
    n = min(T, n_tokens)                 # tokens whose FFN is evaluated per pass
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
    omp_threads(all_cores)
    per_token = tot_r / (reps * T) + tot_f / (reps * n)
    return {"value": 1.0 / per_token, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} passes over one layer at full shape: routing of {T} tokens ({tot_r:.2f} s) + expert "
                      f"FFN and combine of {n} tokens ({tot_f:.2f} s); fp64, OpenMP over tokens"}


def kernel_table(ef, st, wall, every=1):
    out = {}
    for i, name in enumerate(ef.EF_KERNELS):
        n = st["kernel_launches"][i]
        if n:
            sec, byt = st["kernel_seconds"][i], st["kernel_bytes"][i]
            out[name] = {"launches": n, "avg_us": 1e6 * sec / n, "alg_bytes_per_launch": byt / n,
                         "GBps": byt / sec / 1e9 if sec > 0 else None,
                         # bracketed launches stand for `every` launches each
                         "share_of_step_time": sec * every / wall}
            flops = st["kernel_flops"][i]
            if flops > 0:
                out[name]["alg_flops_per_launch"] = flops / n
                out[name]["TFLOPps"] = flops / sec / 1e12 if sec > 0 else None
    return out


def traffic_from_profile(kernel_tag, cfg_name, T, beta):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this very
    workload (FETCH_SIZE + WRITE_SIZE scaled by a copy kernel); counters cannot be read from inside this run."""
    import glob
    tag = f"TRAFFIC_BYTES_PER_LAUNCH {kernel_tag} {cfg_name} T={T} beta={beta} ="
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            if line.startswith(tag):
                return float(line.split("=")[-1]), os.path.relpath(path, ROOT)
    return None, None


def measured_peaks(ef, synth):
    """What this part delivers to a plain kernel (ef_measure_peak): a streaming read of 2 GiB from HBM, and a
    register-resident loop of 16-bit matrix-core instructions.  Reported beside the published peaks."""
    import torch
    cfg = synth.CONFIGS["tiny"]
    ctx = ef.ef_create(n_layers=1, d_model=cfg.d, n_experts=cfg.E, top_k=cfg.k, d_ff=cfg.F, slots_total=1, max_tokens=32)
    try:
        n = 2 << 30
        buf = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        stream = torch.cuda.current_stream()
        hbm = ef.ef_measure_peak(ctx, ef.EF_PEAK_HBM_READ, buf, n, 8, stream)
        mfma = ef.ef_measure_peak(ctx, ef.EF_PEAK_MFMA_16BIT, None, 0, 4, stream)
        del buf
        # the host link as a swap-in sees it: one pinned host-to-device copy of 256 MiB, timed with events
        m = 256 << 20
        host = torch.empty(m, dtype=torch.uint8).pin_memory()
        dev = torch.empty(m, dtype=torch.uint8, device="cuda")
        dev.copy_(host, non_blocking=True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(4):
            dev.copy_(host, non_blocking=True)
        e1.record()
        e1.synchronize()
        pcie = 4 * m / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del host, dev
        return {"hbm_read_GBps": hbm, "mfma_16bit_TFLOPps": mfma, "pcie_h2d_GBps": pcie,
                "published": {"hbm_GBps": HBM_PEAK_GBPS, "mfma_16bit_TFLOPps": MFMA_BF16_PEAK_TFLOPS, "pcie_gen5_x16_GBps": 64.0},
                "how": "ef_measure_peak: 8 streaming reads of 2 GiB (16-byte nontemporal loads); 4 launches of a "
                       "register-resident 32x32x16 bf16 MFMA loop on every SIMD; 4 pinned host-to-device copies of 256 MiB"}
    finally:
        ef.ef_destroy(ctx)


def run_workload(name, spec, args, cpu_seconds):
    import torch
    from paper_2510_26730_amd import binding as ef
    from paper_2510_26730_amd import synth
    from paper_2510_26730_amd.runner import LayerLoop

    cfg = synth.CONFIGS[spec["cfg"]]
    T, beta = spec["T"], spec["beta"]
    steps, warmup = spec["steps"], spec["warmup"]
    L = args.layers or cfg.n_layers
    drift_tokens = spec.get("drift_tokens", 0)
    slots = spec.get("slots") or cfg.slots_per_layer
    all_resident = spec.get("all_resident", False)
    pool_slots = spec.get("pool_slots")
    int4 = spec.get("int4", False)
    stream = torch.cuda.current_stream()
    extra = {} if args.tau is None else {"cum_threshold": args.tau}
    loop = LayerLoop(cfg, L, T, slots, pool_slots=pool_slots, beta=beta, profile=False, all_resident=all_resident,
                     q4=int4, **extra)
    loop.h_fixed = spec.get("horizon")
    if args.tune:
        ef.ef_set_tuning(loop.ctx, **dict((kv.split("=")[0], int(kv.split("=")[1])) for kv in args.tune))
    n_in = 4 if L * T * cfg.d <= (1 << 28) else 2     # distinct step inputs, cycled
    hs = [torch.from_numpy(synth.hidden_stack(cfg, L, step=s, T=T).view("int16")).cuda() for s in range(n_in)]
    torch.cuda.synchronize()

    # popularity drift: a new permutation of the Zipf ranks per epoch, written into the registered bias
    # buffers (E floats per layer, host arrays prepared before the timed region)
    drift = {"tokens": 0, "epoch": 0}
    n_epochs = 1 + ((warmup + steps + 4) * T) // drift_tokens if drift_tokens > 0 else 1
    bias_epochs = [[torch.from_numpy(synth.gate_bias(cfg, l, ep)).pin_memory() for l in range(L)]
                   for ep in range(1, n_epochs + 1)] if drift_tokens > 0 else []

    def run_step(h):
        if drift_tokens > 0:
            drift["tokens"] += T
            ep = drift["tokens"] // drift_tokens
            if ep != drift["epoch"]:
                drift["epoch"] = ep
                for l in range(L):
                    loop.gate_b[l].copy_(bias_epochs[(ep - 1) % len(bias_epochs)][l], non_blocking=True)
        loop.step(h, stream)

    for s in range(warmup):
        run_step(hs[s % n_in])
    torch.cuda.synchronize()

    # untimed pass with every kernel bracketed: the per-kernel breakdown, and from it the dominant kernel (the
    # kind with the largest summed time)
    ef.ef_set_profile(loop.ctx, 0x3FF)
    ef.ef_set_profile_sampling(loop.ctx, 1)
    tok_dist = torch.empty(T, dtype=torch.float32, device="cuda")
    dist = torch.zeros(1, dtype=torch.float64, device="cuda")
    ef.ef_token_dist(loop.ctx, hs[0][0], T, tok_dist, dist, stream)     # first call loads the kernels
    torch.cuda.synchronize()
    ef.ef_reset_stats(loop.ctx)
    t1 = time.perf_counter()
    n_break = 2 if steps >= 6 else 1
    for s in range(n_break):
        # the intra-batch diversity signal of the iteration's tokens (once per step, outside `value`)
        ef.ef_token_dist(loop.ctx, hs[s % n_in][0], T, tok_dist, dist, stream)
        run_step(hs[(warmup + s) % n_in])
    torch.cuda.synchronize()
    kern = kernel_table(ef, ef.ef_get_stats(loop.ctx), time.perf_counter() - t1)
    ranked = sorted((k for k in kern if k in KIND_BOUND), key=lambda k: -kern[k]["avg_us"] * kern[k]["launches"])
    dom_name = ranked[0] if ranked else "ffn_up"

    # timed region: only the dominant kernel is bracketed with HIP events, on the stream it is launched on;
    # every 4th launch of it (events between kernels cost the stream 2-3 us each); with fewer than 64 launches
    # in the timed region, every launch
    every = 4 if L * steps >= 64 else 1
    ef.ef_set_profile(loop.ctx, 1 << ef.EF_KERNELS.index(dom_name))
    ef.ef_set_profile_sampling(loop.ctx, every)
    ef.ef_reset_stats(loop.ctx)
    t0 = time.perf_counter()
    marks = []
    for s in range(steps):
        run_step(hs[(warmup + n_break + s) % n_in])
        marks.append(time.perf_counter())     # the host runs at most one layer ahead of the GPU (it waits
    torch.cuda.synchronize()                  # for every layer's counts), so these bound each step's time
    dt = time.perf_counter() - t0
    marks[-1] = t0 + dt
    per_step = sorted(1e3 * (b - a) for a, b in zip([t0] + marks[:-1], marks))
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    st = ef.ef_get_stats(loop.ctx)
    dom = kernel_table(ef, st, dt, every).get(dom_name)
    ef.ef_set_profile(loop.ctx, 0)

    # what the residency bias costs: share of (layer, token) pairs whose expert set differs from the beta = 0
    # routing of the same hidden states, with the cache as the timed region left it
    changed = None
    if beta != 0.0:
        i32 = dict(dtype=torch.int32, device="cuda")
        n = T * cfg.k
        bufs = [dict(ids=torch.empty(n, **i32), w=torch.empty(n, dtype=torch.float32, device="cuda"),
                     counts=torch.empty(cfg.E, **i32), offsets=torch.empty(cfg.E + 1, **i32), perm=torch.empty(n, **i32),
                     inv=torch.empty(n, **i32)) for _ in range(2)]
        diff = 0
        h_last = hs[(warmup + n_break + steps - 1) % n_in]
        for l in range(L):
            for bb, o in zip((beta, 0.0), bufs):
                ef.ef_route(loop.ctx, l, h_last[l], T, bb, o["ids"], o["w"], o["counts"], o["offsets"], o["perm"],
                            o["inv"], stream)
            diff += int((bufs[0]["ids"].view(T, cfg.k) != bufs[1]["ids"].view(T, cfg.k)).any(dim=1).sum())
        changed = diff / (L * T)

    layer_tokens = T * L * steps
    us_per_layer = 1e6 * dt / (L * steps)
    roof = None
    if dom:
        bound, kname = KIND_BOUND[dom_name]
        if bound == "mfma":
            a = dom["TFLOPps"]
            traffic, src = (None, None)
            if not (all_resident or pool_slots or int4 or args.layers):
                traffic, src = traffic_from_profile(kname, cfg.name, T, beta)
            roof = {"bound": "mfma", "kernel": kname, "achieved": a, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": a / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_source": src, "avg_launch_us": dom["avg_us"],
                    "alg_flops_per_launch": dom["alg_flops_per_launch"], "launches": dom["launches"],
                    "share_of_step_time": dom["share_of_step_time"]}
        else:
            a = dom["GBps"]
            traffic, src = (None, None)
            if dom_name == "ffn_up" and not (all_resident or pool_slots or int4 or args.layers):
                traffic, src = traffic_from_profile("ffn_gate_up_kernel", cfg.name, T, beta)
            roof = {"bound": "hbm", "kernel": kname, "achieved": a, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": a / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": src,
                    "avg_launch_us": dom["avg_us"], "alg_bytes_per_launch": dom["alg_bytes_per_launch"],
                    "launches": dom["launches"], "share_of_step_time": dom["share_of_step_time"]}
    uses = st["hits"] + st["misses"]
    bw = st["bandwidth_Bps"]
    cache_txt = "all experts" if all_resident else (f"{pool_slots}-slot pool" if pool_slots else f"{slots} slots/layer")
    result = {
        "name": name, "baseline_config": spec.get("baseline_config"), "note": spec.get("note"),
        "value": layer_tokens / dt, "unit": "tokens/s", "steps": steps, "warmup": warmup,
        "ms_per_step": 1e3 * dt / steps,
        "dtype": "f16 (4-bit expert weights dequantised to fp16, fp32 accumulation)" if int4 else "bf16",
        "config": {"workload": f"{cfg.name}: {L} layers, d={cfg.d}, E={cfg.E}, top-{cfg.k}, F={cfg.F}"
                               f"{', shared FFN ' + str(cfg.F_shared) if cfg.F_shared else ''}, T={T} tokens/step, cache {cache_txt}"
                               f"{', 4-bit experts' if int4 else ''}, beta={beta}, expert store = {loop.store_layers}-layer "
                               f"pinned pool reused cyclically",
                   "tokens_per_step": T, "layers": L, "beta": beta,
                   "horizon": "adaptive" if spec.get("horizon") is None else spec["horizon"], "drift_tokens": drift_tokens},
        "us_per_layer": us_per_layer,
        "ms_per_step_p10_p50_p90": [pct(0.1), pct(0.5), pct(0.9)],
        "stall_frac": st["stall_seconds"] / dt,
        "hit_rate": st["hits"] / uses if uses else None,
        "beta_changed_token_frac": changed,
        # bytes the link can move in one layer time (C_s * T_l): misses and prefetches beyond it cannot be hidden
        "link_bound_bytes_per_layer": bw * us_per_layer * 1e-6,
        "expert_bytes": loop.es,
        "cache": {"hits": st["hits"], "misses": st["misses"], "miss_rate": st["miss_rate"],
                  "prefetch_issued": st["prefetch_issued"], "prefetch_used": st["prefetch_used"],
                  "prefetch_wasted": st["prefetch_wasted"], "prefetch_redundant": st["prefetch_redundant"],
                  "evictions": st["evictions"], "bytes_copied": st["bytes_copied"],
                  "bytes_copied_per_step": st["bytes_copied"] / steps,
                  # priority copies (misses and prefetches a layer caught in the queue): request -> complete
                  "miss_copies": st["miss_copies"],
                  "miss_copy_ms": 1e3 * st["miss_copy_seconds"] / st["miss_copies"] if st["miss_copies"] else None,
                  "miss_copy_GBps": st["miss_copy_bytes"] / st["miss_copy_seconds"] / 1e9 if st["miss_copy_seconds"] > 0 else None,
                  # of the experts a layer used, the share the look-ahead of j layers earlier had named (j = 1, 2, ...)
                  "prediction_overlap_by_distance": [st["pred_overlap_hits"][j] / st["pred_overlap_total"][j]
                                                     for j in range(7) if st["pred_overlap_total"][j] > 0],
                  "bytes_copied_per_layer": st["bytes_copied"] / (L * steps),
                  "pcie_GBps": st["bytes_timed"] / st["copy_seconds"] / 1e9 if st["copy_seconds"] > 0 else None,
                  "horizon": st["horizon"], "bandwidth_est_GBps": bw / 1e9, "layer_est_us": st["layer_seconds_est"] * 1e6},
        "kernels": {k: {"avg_us": v["avg_us"], "launches": v["launches"], "GBps": v["GBps"], "TFLOPps": v.get("TFLOPps")}
                    for k, v in kern.items()},
        "token_dist": float(dist.cpu()[0]),
        "roofline": roof,
    }
    loop.close()
    del loop, hs
    torch.cuda.empty_cache()
    if cpu_seconds > 0:
        nt = 64 if cpu_seconds >= 6 else 16
        result["cpu_baseline"] = cpu_baseline(cfg, T, beta, cpu_seconds, n_tokens=nt)
        single = cpu_baseline(cfg, T, beta, cpu_seconds / 4, n_tokens=2, threads=1)
        result["cpu_baseline"]["single_thread"] = {k: single[k] for k in ("value", "unit", "cores", "sample")}
    return result


def route_sweep(args):
    """Routing and grouping alone (gate, softmax, biased top-k, per-tile counts, prefix, stable scatter) over a
    sweep of batch sizes at the Mixtral-shaped gate (d = 4096, E = 8, top-2; experts of the smallest legal size,
    none of them run): the sizes at which these kernels are bound by reading the hidden states from HBM."""
    import dataclasses
    import torch
    from paper_2510_26730_amd import binding as ef
    from paper_2510_26730_amd import synth
    cfg = dataclasses.replace(synth.CONFIGS["mixtral_prefill"], name="mixtral_gate", F=32)
    sizes = [int(t) for t in args.route_sweep.split(",")]
    Tm, E, k, d = max(sizes), cfg.E, cfg.k, cfg.d
    L = 2
    ctx = ef.ef_create(n_layers=L, d_model=d, n_experts=E, top_k=k, d_ff=cfg.F, slots_total=E, max_tokens=Tm,
                       renorm_topk=1)
    keep = []
    store = torch.zeros(E * ef.ef_expert_bytes(d, cfg.F), dtype=torch.uint8).pin_memory()
    for l in range(L):
        gw = torch.from_numpy(synth.gate_weight(cfg, l).view("int16")).cuda()
        gb = torch.from_numpy(synth.gate_bias(cfg, l)).cuda()
        ef.ef_register_layer(ctx, l, gw, gb, store, None)
        keep += [gw, gb]
    for e in range(2):
        ef.ef_cache_swap_in(ctx, 0, e, 0, 0)
    g = torch.Generator(device="cuda")
    g.manual_seed(synth.BASE_SEED)
    h_all = torch.randn(Tm, d, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    i32 = dict(dtype=torch.int32, device="cuda")
    n = Tm * k
    o = dict(ids=torch.empty(n, **i32), w=torch.empty(n, dtype=torch.float32, device="cuda"), counts=torch.empty(E, **i32),
             offsets=torch.empty(E + 1, **i32), perm=torch.empty(n, **i32), inv=torch.empty(n, **i32),
             pids=torch.empty(n, **i32), phist=torch.empty(E, **i32))
    stream = torch.cuda.current_stream()
    reps = args.steps or 20
    rows = []
    for form in (1, 0):
        ef.ef_set_tuning(ctx, gate_stream=form)
        for H in (0, 1):
            for T in sizes:
                def call():
                    if H:
                        ef.ef_route_predict(ctx, 0, h_all, T, 1.0, H, None, None, o["ids"], o["w"], o["counts"],
                                            o["offsets"], o["perm"], o["inv"], o["pids"], o["phist"], stream)
                    else:
                        ef.ef_route(ctx, 0, h_all, T, 1.0, o["ids"], o["w"], o["counts"], o["offsets"], o["perm"],
                                    o["inv"], stream)
                for _ in range(3):
                    call()
                torch.cuda.synchronize()
                ef.ef_set_profile(ctx, (1 << ef.EF_KERNELS.index("route")) | (1 << ef.EF_KERNELS.index("group")))
                ef.ef_reset_stats(ctx)
                t0 = time.perf_counter()
                for _ in range(reps):
                    call()
                torch.cuda.synchronize()
                wall = time.perf_counter() - t0
                kt = kernel_table(ef, ef.ef_get_stats(ctx), wall)
                ef.ef_set_profile(ctx, 0)
                assert int(o["counts"].sum()) == T * k
                rows.append({"T": T, "look_ahead": H, "streaming_form": bool(form), "us_per_call_wall": 1e6 * wall / reps,
                             "gate": {"avg_us": kt["route"]["avg_us"], "alg_bytes": kt["route"]["alg_bytes_per_launch"],
                                      "GBps": kt["route"]["GBps"], "frac_of_hbm_peak": kt["route"]["GBps"] / HBM_PEAK_GBPS},
                             "group": {"avg_us": kt["group"]["avg_us"], "alg_bytes": kt["group"]["alg_bytes_per_launch"],
                                       "GBps": kt["group"]["GBps"]}})
                print(f"bench.py: route sweep T={T} H={H} streaming={form}: gate {kt['route']['avg_us']:.1f} us "
                      f"{kt['route']['GBps']:.0f} GB/s, group {kt['group']['avg_us']:.1f} us", file=sys.stderr, flush=True)
    ef.ef_destroy(ctx)
    print(json.dumps({"metric": "routing kernels over batch size (gate + grouping), Mixtral-shaped gate", "unit": "GB/s",
                      "hbm_peak_GBps": HBM_PEAK_GBPS, "route_sweep": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS),
                    help="run only this workload (default: the headline and every BASELINE configuration)")
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
    ap.add_argument("--tau", type=float, default=None,
                    help="cumulative share of the predicted demand whose experts are prefetched (default: the library's 0.9)")
    ap.add_argument("--drift-tokens", type=int, default=None,
                    help="re-draw the expert popularity ranks (gate biases) whenever the running token count "
                         "crosses a multiple of this (0 = static popularity)")
    ap.add_argument("--tune", action="append", default=[], metavar="FIELD=INT",
                    help="set a field of the library's launch tuning (ef_set_tuning), e.g. --tune down_k_slices=4")
    ap.add_argument("--delta-forest", action="store_true",
                    help="measure the deviation predictor instead of the headline: activation logs of recurring "
                         "prompts -> random forest on the host -> look-ahead recall with and without its deviation, "
                         "and the layer loop's rate with the deviation path switched on")
    ap.add_argument("--prompts", type=int, default=256, help="--delta-forest: size of the pool of recurring prompts")
    ap.add_argument("--log-steps", type=int, default=24, help="--delta-forest: steps whose routing is logged for training")
    ap.add_argument("--eval-steps", type=int, default=6, help="--delta-forest: fresh steps the look-ahead is scored on")
    ap.add_argument("--route-sweep", default=None, metavar="T1,T2,...",
                    help="measure routing + grouping alone at these batch sizes (Mixtral-shaped gate, tiny experts), "
                         "e.g. 8192,32768,131072, with both forms of the gate kernel, instead of the workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="target CPU time of the headline's oracle baseline")
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
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    ef.lib()          # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if args.calib_copy > 0:
        src = torch.empty(args.calib_copy << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.route_sweep:
        route_sweep(args)
        return

    if args.delta_forest:
        from paper_2510_26730_amd import delta_bench
        cfg = synth.CONFIGS["mixtral_decode"]
        T = args.tokens or 64
        L = args.layers or 8
        H = args.horizon or 3
        steps, warmup = args.steps or 12, args.warmup if args.warmup is not None else 4
        r = delta_bench.run(cfg, T, L, H, args.prompts, steps, warmup, args.log_steps, args.eval_steps)
        w = r["layer_loop_with_delta"]
        print(json.dumps({
            "metric": "MoE-layer tokens/s (route+predict+FFN) at 1 GPU, look-ahead refined by the host forest's deviation",
            "value": w["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": 1e-3 * w["us_per_layer"] * L, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": r["workload"], "tokens_per_step": T, "layers": L, "horizon": H},
            "delta_forest": r}))
        return

    def spec_of(name):
        spec = dict(WORKLOADS[name])
        for key, val in (("T", args.tokens), ("beta", args.beta), ("steps", args.steps), ("warmup", args.warmup),
                         ("slots", args.slots), ("pool_slots", args.pool_slots), ("horizon", args.horizon),
                         ("drift_tokens", args.drift_tokens)):
            if val is not None:
                spec[key] = val
        if args.all_resident:
            spec["all_resident"] = True
        if args.int4:
            spec["int4"] = True
        return spec

    single = args.workload is not None
    names = [args.workload] if single else DEFAULT_SET
    peaks = measured_peaks(ef, synth)
    results = []
    for i, name in enumerate(names):
        # the headline gets the full oracle sample, the others a short one each (the whole default run stays
        # within a few minutes)
        cpu_s = 0.0 if args.no_cpu_baseline else (args.cpu_seconds if i == 0 else 1.5)
        t0 = time.perf_counter()
        results.append(run_workload(name, spec_of(name), args, cpu_s))
        print(f"bench.py: {name}: {results[-1]['value']:.4g} tokens/s, stall {100 * results[-1]['stall_frac']:.1f} %, "
              f"{time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    for r in results:     # what the part delivers to a plain kernel, beside the published peak the fraction is quoted on
        roof = r.get("roofline")
        if roof and peaks:
            m = peaks["mfma_16bit_TFLOPps"] if roof["bound"] == "mfma" else peaks["hbm_read_GBps"]
            roof["measured_peak"] = m
            roof["frac_of_measured_peak"] = roof["achieved"] / m if m else None
    head = results[0]
    line = {"metric": "MoE-layer tokens/s (route+predict+FFN) at 1 GPU", "value": head["value"], "unit": "tokens/s",
            "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"], "ms_per_step": head["ms_per_step"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic"}
    for key in ("config", "us_per_layer", "ms_per_step_p10_p50_p90", "stall_frac", "hit_rate", "beta_changed_token_frac",
                "link_bound_bytes_per_layer", "expert_bytes", "cache", "kernels", "token_dist", "roofline", "cpu_baseline"):
        if key in head:
            line[key] = head[key]
    if peaks:
        line["measured_peaks"] = peaks
    if not single:
        line["workloads"] = results
    print(json.dumps(line))


if __name__ == "__main__":
    main()
