"""Measurement of the deviation predictor (paper Sec. 3.2.2-3.2.5) around the GPU layer loop:
``python bench.py --delta-forest``.

Call sequencing and counting only: routing and look-ahead run in the HIP kernels (``ef_route_predict``,
``ef_layer_step``), features / forest / cache / producer in the library's host code; this module
collects activation logs from the kernels' outputs, hands them to ``ef_forest_fit``, and counts how
many of the experts a layer really used were in the look-ahead made j layers earlier, with and
without the forest's deviation.

Workload: recurring prompts (``synth.prompt_pool`` / ``prompt_draws`` / ``prompt_hidden``): each of
the T requests of a step carries one of P prompts drawn with Zipf popularity, and a prompt's hidden
states in every layer are fixed, as with a real deterministic model that sees the same prompt again.
The plain look-ahead pushes layer l's hidden state through the gate of layer l+j and so misses the
change of the hidden state in between; the forest sees the prompt's tokens and what it activated in
the layers known so far.
"""
from __future__ import annotations

import time

import numpy as np
import torch

from . import binding as ef
from . import synth
from .runner import LayerLoop


def run(cfg, T: int, L: int, H: int, P: int, steps: int, warmup: int, log_steps: int, eval_steps: int,
        n_trees: int = 8, max_depth: int = 14, gains=(0.0, 1.0, 2.0, 4.0, 8.0, 16.0), n_tok: int = 3, V: int = 1024,
        d_emb: int = 16) -> dict:
    E, k = cfg.E, cfg.k
    S = H
    stream = torch.cuda.current_stream()
    loop = LayerLoop(cfg, L, T, cfg.slots_per_layer, beta=0.0, all_resident=True, fixed_estimates=True)
    loop.h_fixed = H
    loop.tok2req = torch.arange(T, dtype=torch.int32, device="cuda")
    pool = synth.prompt_pool(cfg, P, n_tok, V)
    table = np.ascontiguousarray(synth.feature_embedding(cfg, V, d_emb))
    hid = torch.from_numpy(synth.prompt_hidden(cfg, P, L).view(np.int16)).cuda()          # [L, P, d]

    def batch(step):
        pid = synth.prompt_draws(cfg, step, T, P, cfg.zipf_s)
        return pid, hid[:, torch.from_numpy(pid).cuda().long()].contiguous()              # [L, T, d]

    def route_pass(h, delta_of_layer=None):
        """Routing + look-ahead of every layer (no FFN).  Returns actual ids [L, T, k] and the look-ahead
        ids made at each layer, a list of [he, T, k]."""
        actual, pred = [], []
        for l in range(L):
            loop.delta = None if delta_of_layer is None else delta_of_layer(l, actual)
            he = ef.ef_route_predict(loop.ctx, l, h[l], T, 0.0, H, loop.delta, loop.tok2req, loop.ids, loop.w,
                                     loop.counts, loop.offsets, loop.perm, loop.inv_perm, loop.pred_ids, loop.hist,
                                     stream)
            stream.synchronize()
            actual.append(loop.ids.cpu().numpy().reshape(T, k).copy())
            pred.append(loop.pred_ids.cpu().numpy()[:he * T * k].reshape(he, T, k).copy())
        loop.delta = None
        return np.stack(actual), pred

    def multi_hot(ids_ltk):                      # [L, T, k] -> [T, L, E] uint8
        out = np.zeros((T, L, E), dtype=np.uint8)
        for l in range(L):
            np.put_along_axis(out[:, l], ids_ltk[l], 1, axis=1)
        return out

    def recall(actual, pred):
        """hits[j-1], total[j-1]: experts used at layer l+j that the look-ahead from layer l named."""
        hits, total = np.zeros(H, dtype=np.int64), np.zeros(H, dtype=np.int64)
        for l in range(L):
            for j in range(pred[l].shape[0]):
                a, p = actual[l + 1 + j], pred[l][j]
                hits[j] += (a[:, :, None] == p[:, None, :]).any(axis=2).sum()
                total[j] += a.size
        return hits, total

    # ---- 1. activation logs from the kernels' routing of log_steps steps -----------------------------------
    def examples(pid, act, step_size):           # act [T, L, E]; one example per (request, layer), lag = step size
        X = np.empty((T * L, d_emb + 2 + L * E), dtype=np.float32)
        Y = np.empty((T * L, E), dtype=np.uint8)
        for t in range(T):
            for l in range(L):
                prev = np.zeros((L, E), dtype=np.uint8)
                known = max(0, l - step_size)
                prev[:known] = act[t, :known]
                X[t * L + l] = ef.ef_delta_features(table, pool[pid[t]], step_size, l, prev, L, E)
                Y[t * L + l] = act[t, l]
        return X, Y

    t0 = time.perf_counter()
    Xs, Ys = [], []
    for s in range(log_steps):
        pid, h = batch(s)
        actual, _ = route_pass(h)
        for step_size in range(1, H + 1):        # the step size is a feature: one set of examples per value
            X, Y = examples(pid, multi_hot(actual), step_size)
            Xs.append(X)
            Ys.append(Y)
    X, Y = np.concatenate(Xs), np.concatenate(Ys)
    t_logs = time.perf_counter() - t0

    # ---- 2. fit ---------------------------------------------------------------------------------------------
    forest = ef.ef_forest_create(X.shape[1], E, n_trees, max_depth, 1, 0)
    boot = synth.bootstrap_indices(cfg, n_trees, X.shape[0])
    t0 = time.perf_counter()
    ef.ef_forest_fit(forest, X, Y, boot)
    t_fit = time.perf_counter() - t0
    nodes = [ef.ef_forest_tree_size(forest, t) for t in range(n_trees)]

    cache = ef.ef_delta_cache_create(1 << 20, E)
    prod = ef.ef_delta_producer_create(forest, cache, table, L, E, 0)
    delta_host = torch.zeros(T, H, E, dtype=torch.float32).pin_memory()
    delta_dev = torch.zeros(T, H, E, dtype=torch.float32, device="cuda")
    tok_off = (np.arange(T + 1) * n_tok).astype(np.int32)

    # ---- 3. look-ahead quality on fresh steps: plain look-ahead against look-ahead + deviation -----------------
    base_hits = base_tot = None
    gain_hits = {g: np.zeros(H, dtype=np.int64) for g in gains}
    acc_num, acc_den = np.zeros(H + 1), np.zeros(H + 1)       # bit accuracy per step size (Sec. 3.2.5)
    seen = set(np.concatenate([synth.prompt_draws(cfg, s, T, P, cfg.zipf_s) for s in range(log_steps)]).tolist())
    n_seen = n_req = 0
    for s in range(log_steps, log_steps + eval_steps):
        pid, h = batch(s)
        toks = np.ascontiguousarray(pool[pid].reshape(-1))
        n_seen += sum(int(p) in seen for p in pid)
        n_req += T
        actual, pred = route_pass(h)
        hh, tt = recall(actual, pred)
        base_hits = hh if base_hits is None else base_hits + hh
        base_tot = tt if base_tot is None else base_tot + tt
        act = multi_hot(actual)
        for step_size in range(1, H + 1):
            Xe, Ye = examples(pid, act, step_size)
            acc_num[step_size] += ef.ef_forest_bit_accuracy(ef.ef_forest_predict(forest, Xe, E), Ye) * Ye.size
            acc_den[step_size] += Ye.size
        for g in gains:
            def delta_of_layer(l, actual_so_far, g=g):
                known = np.zeros((T, L, E), dtype=np.uint8)
                for ll in range(l):
                    np.put_along_axis(known[:, ll], actual_so_far[ll], 1, axis=1)
                for t in range(T):
                    ef.ef_delta_submit(prod, pool[pid[t]], S, l + 1, H, known[t])
                ef.ef_delta_drain(prod)
                ef.ef_delta_assemble(cache, toks, tok_off, l, S, H, L, g, E, out=delta_host.numpy())
                delta_dev.copy_(delta_host, non_blocking=True)
                return delta_dev
            a2, p2 = route_pass(h, delta_of_layer)
            assert np.array_equal(a2, actual)            # the deviation only enters the look-ahead, never the routing
            gain_hits[g] += recall(a2, p2)[0]
    best_gain = max(gains, key=lambda g: gain_hits[g].sum())

    # ---- 4. throughput of the full layer loop with and without the deviation path ---------------------------------
    ids_host = torch.zeros(L, T * k, dtype=torch.int32).pin_memory()

    def step_with_delta(s, use_delta):
        pid, h = batch(s)
        toks = np.ascontiguousarray(pool[pid].reshape(-1))
        found = 0
        for l in range(L):
            if use_delta:
                _, hits = ef.ef_delta_assemble(cache, toks, tok_off, l, S, H, L, best_gain, E, out=delta_host.numpy())
                found += hits
                delta_dev.copy_(delta_host, non_blocking=True)
                loop.delta = delta_dev
            loop.layer_separate_calls(l, h[l], stream)
            if use_delta:
                ids_host[l].copy_(loop.ids, non_blocking=True)
        loop.delta = None
        if use_delta:
            # after the step: queue this step's requests (with everything they activated) for the producer; the
            # predictions are in the cache when the prompts come back
            stream.synchronize()
            act = multi_hot(ids_host.numpy().reshape(L, T, k))
            for t in range(T):
                ef.ef_delta_submit(prod, pool[pid[t]], S, 1, L - 1, act[t])
        return found

    timing = {}
    for use_delta in (False, True):
        base = 10_000 if use_delta else 20_000
        for s in range(warmup):
            step_with_delta(base + s, use_delta)
        torch.cuda.synchronize()
        found = 0
        t0 = time.perf_counter()
        for s in range(steps):
            found += step_with_delta(base + warmup + s, use_delta)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        timing[use_delta] = {"tokens_per_s": T * L * steps / dt, "us_per_layer": 1e6 * dt / (L * steps),
                             "delta_rows_found": found / max(1, steps * L * T * H)}
    ef.ef_delta_drain(prod)

    # producer rate: forest evaluations per second through the queue
    hits0, miss0, entries0 = ef.ef_delta_cache_counts(cache)
    fresh = ef.ef_delta_cache_create(1 << 20, E)
    prod2 = ef.ef_delta_producer_create(forest, fresh, table, L, E, 0)
    rng_tok = synth.prompt_pool(cfg, 4096, n_tok, V)
    zero_act = np.zeros((L, E), dtype=np.uint8)
    t0 = time.perf_counter()
    for r in range(4096):
        ef.ef_delta_submit(prod2, rng_tok[r], S, 1, L - 1, zero_act)
    ef.ef_delta_drain(prod2)
    t_prod = time.perf_counter() - t0
    n_prod = ef.ef_delta_cache_counts(fresh)[2]
    ef.ef_delta_producer_destroy(prod2)
    ef.ef_delta_cache_destroy(fresh)

    ef.ef_delta_producer_destroy(prod)
    ef.ef_delta_cache_destroy(cache)
    ef.ef_forest_destroy(forest)
    loop.close()
    return {
        "workload": f"{cfg.name}: {L} layers, T={T} requests per step, {P} recurring prompts of {n_tok} tokens "
                    f"(Zipf {cfg.zipf_s}), look-ahead H=S={H}, all experts resident, beta=0",
        "log_steps": log_steps, "examples": int(X.shape[0]), "features": int(X.shape[1]),
        "log_collection_s": t_logs, "fit_s": t_fit, "trees": n_trees, "max_depth": max_depth, "nodes_per_tree": nodes,
        "eval_steps": eval_steps, "share_of_eval_requests_seen_in_logs": n_seen / max(1, n_req),
        "bit_accuracy_eval": float(acc_num.sum() / acc_den.sum()),
        "bit_accuracy_by_step_size": {str(ss): float(acc_num[ss] / acc_den[ss]) for ss in range(1, H + 1)},
        "lookahead_recall_plain": (base_hits / base_tot).tolist(),
        "lookahead_recall_with_delta": {str(g): (gain_hits[g] / base_tot).tolist() for g in gains},
        "best_gain": best_gain,
        "layer_loop_plain": timing[False], "layer_loop_with_delta": timing[True],
        "producer_predictions_per_s": n_prod / t_prod, "producer_threads": "all host threads",
    }
