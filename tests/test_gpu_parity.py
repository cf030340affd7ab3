"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer results bit-exact outside near-ties (oracle gap < 1e-4); float results within
max-abs 2e-2 and relative L2 1e-2 (bf16 inputs, fp32 accumulation)."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

import helpers
from helpers import LayerStack, check_route, dev_u16, float_close, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def shape(base, **kw):
    return dataclasses.replace(synth.CONFIGS[base], **kw)


SMALL_QWEN = shape("qwen15_moe", name="small_qwen", d=256, F=96, F_shared=160, T=77)
SMALL_DEEPSEEK = shape("deepseek_v2_lite", name="small_deepseek", d=192, F=64, F_shared=128, T=130)


def oracle_layer(oracle_mod, st, layer, h, beta, resident, forced_ids=None):
    c = st.cfg
    return oracle_mod.moe_layer(h, st.gates[layer], st.biases[layer], st.experts[layer], c.k, beta=beta,
                                resident=resident, renorm=c.renorm, shared=st.shared.get(layer),
                                forced_ids=forced_ids)


@pytest.mark.parametrize("beta", [0.0, 0.75])
def test_tiny_route_and_layer(oracle_mod, beta):
    cfg = synth.CONFIGS["tiny"]
    say(f"tiny layer beta={beta}")
    st = LayerStack(cfg, 3, slots_total=12, per_layer=4, max_tokens=64)
    try:
        for e in np.nonzero(synth.residency(cfg, 0))[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        assert np.array_equal(res, synth.residency(cfg, 0))
        h = synth.hidden(cfg, 0)
        hd = dev_u16(h)
        r = st.route(0, hd, cfg.T, beta)
        got = to_np(r, cfg.T, cfg.k)
        ora = oracle_mod.route(h, st.gates[0], st.biases[0], cfg.k, beta, res, renorm=cfg.renorm)
        forced, nties = check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
        out = st.ffn(0, hd, cfg.T, r)
        full = oracle_layer(oracle_mod, st, 0, h, beta, res, forced_ids=got["ids"])
        e1, e2 = float_close(out, full["out"])
        say(f"  near-ties {nties}, max abs {e1:.2e}, rel l2 {e2:.2e}")
        stats = ef.ef_get_stats(st.ctx)
        assert stats["layers_run"] == 1 and stats["tokens_run"] == cfg.T
        assert stats["hits"] + stats["misses"] == int((got["counts"] > 0).sum())
    finally:
        st.close()


def test_tiny_predict_with_delta_and_residency(oracle_mod):
    cfg = synth.CONFIGS["tiny"]
    say("tiny predict H=2")
    st = LayerStack(cfg, 3, slots_total=12, per_layer=4, max_tokens=64, expert_layers=[0])
    try:
        ef.ef_cache_swap_in(st.ctx, 1, 3, 0, 1)
        ef.ef_cache_swap_in(st.ctx, 2, 5, 0, 2)
        ef.ef_cache_swap_in(st.ctx, 2, 0, 0, 2)
        h = synth.hidden(cfg, 0)
        R, H = 3, 2
        delta = synth.delta(cfg, 0, R, H)
        t2r = synth.tok2req(cfg, cfg.T, R)
        residents = [ef.ef_cache_query(st.ctx, 1 + j, cfg.E) for j in range(H)]
        assert [int(r.sum()) for r in residents] == [1, 2]
        for beta, dl, tr in [(0.0, None, None), (0.5, delta, t2r), (0.5, delta, None)]:
            he, ids, hist = st.predict(0, dev_u16(h), cfg.T, H, beta, dl, tr)
            assert he == H
            oids, ohist, ogap, osc = oracle_mod.predict(h, st.gates[1:3], st.biases[1:3], cfg.k, beta, residents,
                                                        dl, tr, return_scores=True)
            tie = ogap < helpers.TIE_GAP
            assert np.array_equal(ids[~tie], oids[~tie])
            for j in range(H):
                helpers.check_ids_valid(ids[j], osc[j], ogap[j], cfg.k)    # inside a near-tie: a valid choice
                assert np.array_equal(hist[j], oracle_mod.histogram(ids[j], cfg.E))
                assert hist[j].sum() == cfg.T * cfg.k
            if not tie.any():
                assert np.array_equal(hist, ohist)
        # look-ahead is clamped at the last layer
        he, ids, hist = st.predict(1, dev_u16(h), cfg.T, 2, 0.0)
        assert he == 1
        assert np.array_equal(ids[0], oracle_mod.route(h, st.gates[2], st.biases[2], cfg.k)["ids"])
        he, _, _ = st.predict(2, dev_u16(h), cfg.T, 2, 0.0)
        assert he == 0
    finally:
        st.close()


@pytest.mark.parametrize("cfg,T,H", [(synth.CONFIGS["tiny"], 64, 2), (SMALL_DEEPSEEK, 130, 4), (SMALL_DEEPSEEK, 130, 6),
                                     (SMALL_QWEN, 77, 3)])
def test_fused_route_predict_equals_separate_calls(oracle_mod, cfg, T, H):
    """One pass over the hidden states gives bit-identical results to ef_route + ef_predict
    (E=64 with H>=5 needs more gate columns than one launch holds: the launch is split)."""
    say(f"fused route+predict {cfg.name} T={T} H={H}")
    L = H + 1
    st = LayerStack(cfg, L, slots_total=cfg.E, max_tokens=T, expert_layers=[0], h_max=min(H, 7))
    try:
        for l in range(L):
            for e in np.nonzero(synth.residency(cfg, l, n_resident=3, most_popular=False))[0]:
                ef.ef_cache_swap_in(st.ctx, l, int(e), 0, l)
        h = synth.hidden(cfg, 9, T)
        hd = dev_u16(h)
        R = 4
        delta, t2r = synth.delta(cfg, 0, R, H), synth.tok2req(cfg, T, R)
        dd, td = torch.from_numpy(delta).cuda(), torch.from_numpy(t2r).cuda()
        beta = 0.4
        sep = to_np(st.route(0, hd, T, beta), T, cfg.k)
        he, pids, phist = st.predict(0, hd, T, H, beta, delta, t2r)
        assert he == H
        o = st.route(0, hd, T, 0.0)     # fresh buffers, then overwritten by the fused call
        fids = torch.full((H * T * cfg.k,), -1, dtype=torch.int32, device="cuda")
        fhist = torch.full((H * cfg.E,), -1, dtype=torch.int32, device="cuda")
        he2 = ef.ef_route_predict(st.ctx, 0, hd, T, beta, H, dd, td, o["ids"], o["w"], o["counts"], o["offsets"],
                                  o["perm"], o["inv_perm"], fids, fhist, torch.cuda.current_stream())
        fused = to_np(o, T, cfg.k)
        assert he2 == H
        for name in sep:
            assert np.array_equal(sep[name], fused[name]), name
        assert np.array_equal(fids.cpu().numpy().reshape(H, T, cfg.k), pids)
        assert np.array_equal(fhist.cpu().numpy().reshape(H, cfg.E), phist)
        # and the predictions themselves against the oracle
        residents = [ef.ef_cache_query(st.ctx, 1 + j, cfg.E) for j in range(H)]
        oids, ohist, ogap, osc = oracle_mod.predict(h, st.gates[1:1 + H], st.biases[1:1 + H], cfg.k, beta, residents,
                                                    delta, t2r, return_scores=True)
        tie = ogap < helpers.TIE_GAP
        assert np.array_equal(pids[~tie], oids[~tie])
        for j in range(H):
            helpers.check_ids_valid(pids[j], osc[j], ogap[j], cfg.k)
            assert np.array_equal(phist[j], oracle_mod.histogram(pids[j], cfg.E))
    finally:
        st.close()


@pytest.mark.parametrize("cfg,T", [(synth.CONFIGS["tiny"], 1), (synth.CONFIGS["tiny"], 31),
                                   (synth.CONFIGS["tiny"], 33), (synth.CONFIGS["tiny"], 100),
                                   (SMALL_QWEN, 77), (SMALL_QWEN, 3), (SMALL_DEEPSEEK, 130),
                                   (SMALL_DEEPSEEK, 32)])
def test_ragged_shapes_full_layer(oracle_mod, cfg, T):
    say(f"ragged {cfg.name} T={T} E={cfg.E} k={cfg.k} d={cfg.d} F={cfg.F} Fs={cfg.F_shared}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=max(T, 8))
    try:
        res = synth.residency(cfg, 0, n_resident=max(1, cfg.E // 4), most_popular=False)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        h = synth.hidden(cfg, 3, T)
        hd = dev_u16(h)
        beta = 0.5
        r = st.route(0, hd, T, beta)
        got = to_np(r, T, cfg.k)
        ora = oracle_mod.route(h, st.gates[0], st.biases[0], cfg.k, beta, res, renorm=cfg.renorm)
        check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
        out = st.ffn(0, hd, T, r)               # misses are swapped in by the call itself
        full = oracle_layer(oracle_mod, st, 0, h, beta, res, forced_ids=got["ids"])
        e1, e2 = float_close(out, full["out"])
        say(f"  max abs {e1:.2e}, rel l2 {e2:.2e}")
    finally:
        st.close()


def drawn_shapes(n_cases=12):
    """Seeded draw of layer shapes and batch sizes that no named configuration has: expert counts that are
    not powers of two, top-k up to the library's maximum, hidden sizes at the smallest legal granularity,
    batches from one token to several 32-token tiles with a ragged tail."""
    g = np.random.Generator(np.random.PCG64(20251026))
    out = []
    for i in range(n_cases):
        E = int(g.choice([3, 5, 8, 12, 16, 24, 40, 60, 64]))
        k = int(g.integers(1, min(E, 8) + 1))
        d = 64 * int(g.integers(1, 7))
        F = 32 * int(g.integers(1, 10))
        Fs = 32 * int(g.integers(0, 5)) if i % 2 else 0
        T = int(g.choice([1, 2, 7, 31, 32, 33, 63, 65, 97, 128, 161, 255, 300]))
        beta = float(g.choice([0.0, 0.25, 1.0, 4.0]))
        out.append((dataclasses.replace(synth.CONFIGS["tiny"], name=f"drawn{i}", cfg_id=900 + i, d=d, E=E, k=k, F=F,
                                        F_shared=Fs, T=T, renorm=bool(i % 3), w_std=0.05), T, beta))
    return out


@pytest.mark.parametrize("cfg,T,beta", drawn_shapes(), ids=lambda v: getattr(v, "name", str(v)))
def test_drawn_shapes_full_layer(oracle_mod, cfg, T, beta):
    say(f"drawn {cfg.name} T={T} E={cfg.E} k={cfg.k} d={cfg.d} F={cfg.F} Fs={cfg.F_shared} beta={beta} "
        f"renorm={cfg.renorm}")
    n_res = max(1, cfg.E // 3)
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=max(T, 8))
    try:
        res = synth.residency(cfg, 0, n_resident=n_res, most_popular=False)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        h = synth.hidden(cfg, 5, T)
        hd = dev_u16(h)
        r = st.route(0, hd, T, beta)
        got = to_np(r, T, cfg.k)
        ora = oracle_mod.route(h, st.gates[0], st.biases[0], cfg.k, beta, res, renorm=cfg.renorm)
        _, nties = check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
        out = st.ffn(0, hd, T, r)
        full = oracle_layer(oracle_mod, st, 0, h, beta, res, forced_ids=got["ids"])
        e1, e2 = float_close(out, full["out"])
        say(f"  near-ties {nties}, max abs {e1:.2e}, rel l2 {e2:.2e}")
    finally:
        st.close()


def test_shared_ffn_tiled_beside_streamed_routed_groups(oracle_mod):
    """A batch whose shared FFN (10 token tiles, K = 1024) takes the tiled kernels with two K slices while the
    routed experts (2-4 tiles, K = 128) stream with one: the un-permute sums a different number of planes per
    expert.  Whole output against the oracle."""
    cfg = shape("tiny", name="split_slices", d=256, F=128, F_shared=1024, T=300)
    T = cfg.T
    say(f"separate slice counts: d={cfg.d} F={cfg.F} Fs={cfg.F_shared} E={cfg.E} k={cfg.k} T={T}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=T, flags=ef.EF_FLAG_PROFILE)
    try:
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        h = synth.hidden(cfg, 2, T)
        hd = dev_u16(h)
        r = st.route(0, hd, T, 0.0)
        got = to_np(r, T, cfg.k)
        ora = oracle_mod.route(h, st.gates[0], st.biases[0], cfg.k, 0.0, res, renorm=cfg.renorm)
        check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
        out = st.ffn(0, hd, T, r)
        full = oracle_layer(oracle_mod, st, 0, h, 0.0, res, forced_ids=got["ids"])
        e1, e2 = float_close(out, full["out"])
        launches = dict(zip(ef.EF_KERNELS, ef.ef_get_stats(st.ctx)["kernel_launches"]))
        say(f"  max abs {e1:.2e}, rel l2 {e2:.2e}, launches {launches}")
        assert launches["ffn_down_tiled"] >= 1 and launches["ffn_down"] == 1   # shared FFN (+ routed groups of 10+ tiles)
    finally:
        st.close()


def test_empty_batch(oracle_mod):
    cfg = synth.CONFIGS["tiny"]
    say("T=0")
    st = LayerStack(cfg, 2, slots_total=4, max_tokens=8, expert_layers=[0])
    try:
        hd = dev_u16(synth.hidden(cfg, 0, 8))
        r = st.route(0, hd, 0, 0.0)
        torch.cuda.synchronize()
        assert r["counts"].cpu().numpy().tolist() == [0] * cfg.E
        assert r["offsets"].cpu().numpy().tolist() == [0] * (cfg.E + 1)
        out = st.ffn(0, hd, 0, r)
        assert out.shape[0] == 0
        he, ids, hist = st.predict(0, hd, 0, 1, 0.0)
        assert he == 1 and hist.sum() == 0
    finally:
        st.close()


def test_outputs_do_not_depend_on_slots_or_phase_order(oracle_mod):
    """Same routing, different cache histories: experts preloaded in different slots, or missing and
    swapped in by the FFN call in several phases through a 2-slot layer: bitwise the same output."""
    cfg = synth.CONFIGS["tiny"]
    say("slot / phase invariance")
    h = synth.hidden(cfg, 5)
    outs = []
    for variant in range(3):
        st = LayerStack(cfg, 1, slots_total=8 if variant < 2 else 2, per_layer=0 if variant < 2 else 2,
                        max_tokens=64)
        try:
            order = list(range(cfg.E)) if variant == 0 else list(reversed(range(cfg.E)))
            if variant < 2:
                for e in order:
                    ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
            hd = dev_u16(h)
            r = st.route(0, hd, cfg.T, 0.0)       # beta = 0: routing is independent of residency
            outs.append((to_np(r, cfg.T, cfg.k), st.ffn(0, hd, cfg.T, r)))
            if variant == 2:
                s = ef.ef_get_stats(st.ctx)
                assert s["misses"] == int((outs[-1][0]["counts"] > 0).sum()) and s["evictions"] >= 1
        finally:
            st.close()
    for name in ("ids", "w", "perm"):
        assert np.array_equal(outs[0][0][name], outs[1][0][name]) and np.array_equal(outs[0][0][name], outs[2][0][name])
    assert np.array_equal(outs[0][1], outs[1][1]) and np.array_equal(outs[0][1], outs[2][1])


SHARED_TILED = shape("tiny", name="shared_tiled", d=256, F=128, F_shared=1024)   # shared FFN of 10 tiles at T = 300


@pytest.mark.parametrize("cfg_name,T,q4", [("tiny", 64, False), ("tiny", 7, False), ("tiny", 64, True), ("tiny", 300, True),
                                           (SHARED_TILED, 300, False), (SHARED_TILED, 40, False)])
def test_layer_step_equals_separate_calls(cfg_name, T, q4):
    """The composite entry point (host-mapped hand-over, flag polling) gives bit-identical outputs,
    the same cache decisions and the same horizon as the separate entry points."""
    from paper_2510_26730_amd.runner import LayerLoop
    cfg = synth.CONFIGS[cfg_name] if isinstance(cfg_name, str) else cfg_name
    say(f"ef_layer_step vs separate calls, {cfg.name} T={T} 4-bit experts: {q4}")
    L = 3
    loops = [LayerLoop(cfg, L, T, cfg.slots_per_layer, beta=0.5, seed=1, fixed_estimates=True, q4=q4) for _ in range(2)]
    try:
        stream = torch.cuda.current_stream()
        for step in range(3):
            hs = torch.from_numpy(synth.hidden_stack(cfg, L, step=step, T=T).view(np.int16)).cuda()
            for l in range(L):
                loops[0].layer(l, hs[l], stream)
                loops[1].layer_separate_calls(l, hs[l], stream)
                torch.cuda.synchronize()
                assert torch.equal(loops[0].out, loops[1].out), (step, l)
                assert loops[0].H == loops[1].H
                for ll in range(L):
                    assert np.array_equal(ef.ef_cache_query(loops[0].ctx, ll, cfg.E),
                                          ef.ef_cache_query(loops[1].ctx, ll, cfg.E))
        s0, s1 = ef.ef_get_stats(loops[0].ctx), ef.ef_get_stats(loops[1].ctx)
        for key in ("hits", "misses", "prefetch_issued", "evictions", "bytes_copied", "layers_run"):
            assert s0[key] == s1[key], key
        assert s0["layers_run"] == 9
        for st in (s0, s1):      # timed copies are a subset of the copies; a finished run has timed at least one
            assert 0 < st["bytes_timed"] <= st["bytes_copied"] and st["copy_seconds"] > 0
    finally:
        for lp in loops:
            lp.close()


def _sampled_layer_check(oracle_mod, st, layer, h, T, beta, res, n_sample, seed):
    cfg = st.cfg
    hd = dev_u16(h)
    r = st.route(layer, hd, T, beta)
    got = to_np(r, T, cfg.k)
    ora = oracle_mod.route(h, st.gates[layer], st.biases[layer], cfg.k, beta, res, renorm=cfg.renorm)
    forced, nties = check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
    out = st.ffn(layer, hd, T, r)
    assert np.all(np.isfinite(out))
    # a random sample plus the tokens at the first and last position of every expert's group (the last one
    # sits in the group's partially filled token tile)
    edge = [got["perm"][p] // cfg.k for e in range(cfg.E) if got["counts"][e] > 0
            for p in (got["offsets"][e], got["offsets"][e + 1] - 1)]
    toks = np.unique(np.concatenate([np.random.default_rng(seed).permutation(T)[:n_sample],
                                     np.asarray(edge, dtype=np.int64)])).astype(np.int64)
    hs = np.ascontiguousarray(h[toks])
    ids_s = np.ascontiguousarray(got["ids"][toks])
    sub = oracle_mod.route_from_ids(ora["p"][toks], ids_s, cfg.E, cfg.renorm)
    y = oracle_mod.expert_ffn(hs, st.experts[layer], ids_s, sub["perm"])
    sh = None if not cfg.F_shared else oracle_mod.dense_ffn(hs, *st.shared[layer])
    ref = oracle_mod.combine(y, sub["w"], sub["inv_perm"], sh)
    e1, e2 = float_close(out[toks], ref)
    # the same evaluation with the oracle's intermediate activation rounded to fp16, as the kernels store it:
    # what is left is summation order and the fast exponential, an order of magnitude below the rounding itself
    y_r = oracle_mod.expert_ffn(hs, st.experts[layer], ids_s, sub["perm"], round_act=2)
    sh_r = None if not cfg.F_shared else oracle_mod.dense_ffn(hs, *st.shared[layer], round_act=2)
    ref_r = oracle_mod.combine(y_r, sub["w"], sub["inv_perm"], sh_r)
    r1, r2 = float_close(out[toks], ref_r, max_abs=5e-3, rel_l2=3e-4)    # single activations that round the other way
    say(f"  near-ties {nties}, sampled {len(toks)} tokens: max abs {e1:.2e}, rel l2 {e2:.2e}; "
        f"against fp16-rounded activations: max abs {r1:.2e}, rel l2 {r2:.2e}")


def test_full_size_mixtral_decode_layer(oracle_mod):
    """Decode batches of the headline configuration at full shape: T = 1, 8 and 64.  beta = 1 leaves
    some tokens on non-resident experts (miss swap-ins inside the FFN call, groups of one tile);
    beta = 16 is the benchmark's launch configuration (every token on the two resident experts,
    groups of two tiles, K slices of the second half across workgroups)."""
    cfg = synth.CONFIGS["mixtral_decode"]
    st = LayerStack(cfg, 1, slots_total=8, per_layer=0, max_tokens=64)
    try:
        res = synth.residency(cfg, 0)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        for T, beta, n_sample in [(64, 16.0, 64), (64, 1.0, 16), (8, 1.0, 8), (1, 0.0, 1)]:
            say(f"full size: Mixtral-shaped decode layer, T={T}, beta={beta}")
            res_now = ef.ef_cache_query(st.ctx, 0, cfg.E)
            _sampled_layer_check(oracle_mod, st, 0, synth.hidden(cfg, 0, T), T, beta, res_now, n_sample, 1)
    finally:
        st.close()


@pytest.mark.parametrize("T,H", [(64, 3), (33, 1), (1, 2)])
def test_decode_gate_second_step_fused_with_grouping_equals_separate_kernels(T, H):
    """Decode-sized batches of the headline shape take the K-split gate followed by ONE workgroup that sums the
    partial logits, runs the per-token epilogue and groups the tokens; with the fusion switched off the same
    partial logits go through the separate second-step and grouping kernels.  Same arithmetic in the same
    order: every output must be bit-identical (ids, weights, counts, offsets, permutation, look-ahead ids and
    histograms), also through the layer-step hand-over to the host."""
    cfg = dataclasses.replace(synth.CONFIGS["mixtral_decode"], F=64, name="mixtral_gate")   # routing only: tiny experts
    say(f"decode gate paths: T={T} H={H}")
    L = H + 1
    outs = []
    for fused in (1, 0):
        st = LayerStack(cfg, L, slots_total=cfg.E, max_tokens=64, expert_layers=[0], h_max=H)
        try:
            ef.ef_set_tuning(st.ctx, gate_fused_finish=fused)
            for l in range(L):
                for e in np.nonzero(synth.residency(cfg, l, n_resident=2, most_popular=False))[0]:
                    ef.ef_cache_swap_in(st.ctx, l, int(e), 0, l)
            hd = dev_u16(synth.hidden(cfg, 3, T))
            R = 3
            dd = torch.from_numpy(synth.delta(cfg, 0, R, H)).cuda()
            td = torch.from_numpy(synth.tok2req(cfg, T, R)).cuda()
            o = st.route(0, hd, T, 0.0)
            fids = torch.full((H * T * cfg.k,), -1, dtype=torch.int32, device="cuda")
            fhist = torch.full((H * cfg.E,), -1, dtype=torch.int32, device="cuda")
            he = ef.ef_route_predict(st.ctx, 0, hd, T, 0.7, H, dd, td, o["ids"], o["w"], o["counts"], o["offsets"],
                                     o["perm"], o["inv_perm"], fids, fhist, torch.cuda.current_stream())
            assert he == H
            got = to_np(o, T, cfg.k)
            got["pred_ids"], got["pred_hist"] = fids.cpu().numpy(), fhist.cpu().numpy()
            assert got["pred_hist"].reshape(H, cfg.E).sum(axis=1).tolist() == [T * cfg.k] * H
            outs.append(got)
        finally:
            st.close()
    for name in outs[0]:
        assert np.array_equal(outs[0][name], outs[1][name]), name


@pytest.mark.parametrize("force_tiled", [True, False])
def test_full_size_qwen_mixed_batch(oracle_mod, force_tiled):
    """T = 640 with a shared expert of 20 token tiles: through the matrix-core tiled kernels (the
    default for groups of at least 8 tiles) and, with the library's workgroup threshold raised,
    through the weight-streaming kernels in several passes."""
    cfg = synth.CONFIGS["qwen15_moe"]
    say(f"full size: Qwen1.5-MoE-shaped layer, T=640, shared expert, tiled kernels forced: {force_tiled}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=640)
    try:
        if not force_tiled:
            ef.ef_set_tuning(st.ctx, tiled_min_up_wgs=1000000)
        res = synth.residency(cfg, 0)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        _sampled_layer_check(oracle_mod, st, 0, synth.hidden(cfg, 0, 640), 640, 0.5, res, 24, 2)
    finally:
        st.close()


@pytest.mark.parametrize("streamed_form", ["shared4", "shared4_two_per_cu", "plain4", "plain2"])
def test_full_size_deepseek_prefill(oracle_mod, streamed_form):
    """DeepSeek-V2-Lite-shaped layer at its three batch shapes: 32 decode tokens, 1024 prefill tokens and
    the mixed 1056 (shared experts through the tiled kernels from 256 tokens on, routed experts
    streamed).  The routed experts of the larger batches hold 3-7 token tiles: by default they take passes of
    four tiles through the kernels that share fragments in LDS (one workgroup per compute unit, or two with a
    shorter register ring: the form taken beside a large tiled launch); the other two forms (plain kernels with
    passes of four, or of two tiles) are forced through ef_set_tuning."""
    cfg = synth.CONFIGS["deepseek_v2_lite"]
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=1056)
    try:
        if streamed_form == "shared4_two_per_cu":
            ef.ef_set_tuning(st.ctx, lds_shared_occupancy=2)
        elif streamed_form != "shared4":
            ef.ef_set_tuning(st.ctx, lds_shared=0)
        if streamed_form == "plain2":
            ef.ef_set_tuning(st.ctx, passes_of_four=0)
        res = synth.residency(cfg, 0)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        for T, n_sample, seed in [(1056, 24, 3), (1024, 12, 5), (32, 8, 6)]:
            say(f"full size: DeepSeek-V2-Lite-shaped layer, T={T}, shared experts")
            res_now = ef.ef_cache_query(st.ctx, 0, cfg.E)
            _sampled_layer_check(oracle_mod, st, 0, synth.hidden(cfg, 0, T), T, 0.5, res_now, n_sample, seed)
        if streamed_form == "shared4":
            # which of the two LDS-sharing forms a launch takes depends on what else is in the launch (how many
            # tiled workgroups run beside it), so the two must agree bit for bit: same sums in the same order
            hd = dev_u16(synth.hidden(cfg, 0, 1056))
            r = st.route(0, hd, 1056, 0.5)
            outs = []
            for occ in (1, 2):
                ef.ef_set_tuning(st.ctx, lds_shared_occupancy=occ)
                outs.append(st.ffn(0, hd, 1056, r))
            assert np.array_equal(outs[0], outs[1])
    finally:
        st.close()


TAIL_SHARED = shape("tiny", name="tail_shared", d=1024, E=2, k=2, F=2048, F_shared=1024, slots_per_layer=2)


def test_tail_cut_of_a_tiled_second_half_can_fall_on_the_shared_ffn(oracle_mod):
    """Two routed experts that every token uses (top-2 of 2) and a shared FFN of half their hidden size at 6144
    tokens: the tiled second half is 3 x 24 token panels x 4 column panels = 288 workgroups, more than one round over
    the compute units, and the group with the least work, whose K range is cut into slices of its own, is the
    shared FFN (its planes are summed by the un-permute's shared-row path).  Against the oracle, and against the
    same layer without the cut."""
    cfg = TAIL_SHARED
    T = 6144
    say(f"tail cut on the shared FFN: {cfg.name} T={T}")
    st = LayerStack(cfg, 1, slots_total=2, max_tokens=T)
    try:
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        h = synth.hidden(cfg, 0, T)
        _sampled_layer_check(oracle_mod, st, 0, h, T, 0.0, res, 48, 9)
        hd = dev_u16(h)
        r = st.route(0, hd, T, 0.0)
        outs = {}
        for slices in (1, 0):
            ef.ef_set_tuning(st.ctx, tiled_tail_slices=slices)
            outs[slices] = st.ffn(0, hd, T, r).copy()
        diff = float(np.max(np.abs(outs[0] - outs[1])))
        say(f"  with against without the cut: max abs difference {diff:.2e}")
        assert 0.0 < diff < 1e-4
    finally:
        st.close()


def test_full_size_mixtral_prefill_layer(oracle_mod):
    cfg = synth.CONFIGS["mixtral_prefill"]
    say("full size: Mixtral-shaped prefill layer, T=8192")
    st = LayerStack(cfg, 1, slots_total=8, max_tokens=8192)
    try:
        res = synth.residency(cfg, 0)
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        h = synth.hidden(cfg, 0, 8192)
        _sampled_layer_check(oracle_mod, st, 0, h, 8192, 0.0, res, 64, 4)
        # The second half has more than one round of workgroups over the compute units, so the group with the
        # least work is cut into K slices of its own (planes summed by the un-permute).  Without the cut, and
        # with a cut in two, the same layer must agree to the rounding of a different summation order.
        hd = dev_u16(h)
        r = st.route(0, hd, 8192, 0.0)
        outs = {}
        for slices in (1, 0, 2):
            ef.ef_set_tuning(st.ctx, tiled_tail_slices=slices)
            outs[slices] = st.ffn(0, hd, 8192, r).copy()
        for slices in (0, 2):
            diff = float(np.max(np.abs(outs[slices] - outs[1])))
            say(f"  tail slices {slices} against the default: max abs difference {diff:.2e}")
            assert 0.0 < diff < 1e-4      # different planes were summed, nothing else changed
    finally:
        st.close()
