"""GPU parity of the grouped FFN with 4-bit expert weights (w = (q - 8) * s, one bf16 scale per row
and 128 inputs) against the CPU oracle, which evaluates the same codes and scales in fp64.

Tolerance: as for bf16 experts (max-abs 2e-2, relative L2 1e-2).  The kernels form (q - 8) * s in
fp16 (one rounding, relative error <= 2^-12 per weight), convert the bf16 tokens to fp16 exactly
and keep the intermediate activations in fp16 (2^-11), all with fp32 accumulation: observed
relative L2 2e-4, max-abs 2e-3 on outputs of rms 2."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

from helpers import LayerStack, check_route, dev_u16, float_close, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def q4_shape(base, **kw):
    return dataclasses.replace(synth.CONFIGS[base], F_shared=0, **kw)


def layer_check(oracle_mod, st, h, T, beta, res, toks=None):
    cfg = st.cfg
    hd = dev_u16(h)
    r = st.route(0, hd, T, beta)
    got = to_np(r, T, cfg.k)
    ora = oracle_mod.route(h, st.gates[0], st.biases[0], cfg.k, beta, res, renorm=cfg.renorm)
    forced, nties = check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
    out = st.ffn(0, hd, T, r)
    assert np.all(np.isfinite(out))
    toks = np.arange(T) if toks is None else toks
    hs = np.ascontiguousarray(h[toks])
    ids_s = np.ascontiguousarray(got["ids"][toks])
    sub = oracle_mod.route_from_ids(ora["p"][toks], ids_s, cfg.E, cfg.renorm)
    y = oracle_mod.expert_ffn_q4(hs, st.experts[0], ids_s, sub["perm"])
    shared = None
    if cfg.F_shared:        # the dense shared FFN is a 4-bit expert every token goes through with weight 1
        n = len(toks)
        shared = oracle_mod.expert_ffn_q4(hs, [st.shared[0]], np.zeros((n, 1), dtype=np.int32), np.arange(n))
    ref = oracle_mod.combine(y, sub["w"], sub["inv_perm"], shared)
    e1, e2 = float_close(out[toks], ref)
    say(f"  near-ties {nties}, {len(toks)} tokens: max abs {e1:.2e}, rel l2 {e2:.2e}, |ref| rms {np.sqrt((ref ** 2).mean()):.2f}")


@pytest.mark.parametrize("name,kw,T", [
    ("tiny", dict(d=512, F=1024), 64),           # two tiles per expert at most
    ("tiny", dict(d=512, F=1024), 1),
    ("tiny", dict(d=512, F=1024), 37),           # ragged tile
    ("tiny", dict(d=128, F=128), 5),             # one quad pair per row block, one scale group
    ("tiny", dict(d=384, F=640), 200),           # several passes of two tiles, odd quad counts per K slice
    ("tiny", dict(d=640, F=256), 70),            # K halves of five stages: one full turn of the register ring and a tail
    ("tiny", dict(d=896, F=128), 33),            # K halves of seven stages
    ("deepseek_v2_lite", dict(d=256, F=128), 130),   # 64 experts, mostly tiny groups
])
def test_q4_layer_matches_oracle(oracle_mod, name, kw, T):
    cfg = q4_shape(name, name=f"{name}_q4", **kw)
    say(f"q4 layer {name} d={cfg.d} F={cfg.F} E={cfg.E} k={cfg.k} T={T}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=max(T, 64), q4=True)
    try:
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, 0.0, res)
    finally:
        st.close()


def test_q4_misses_are_swapped_in(oracle_mod):
    """Two of eight experts resident: the others are fetched (4-bit blobs) inside the FFN call."""
    cfg = q4_shape("tiny", name="tiny_q4", d=512, F=1024)
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=64, q4=True)
    try:
        res = synth.residency(cfg, 0, n_resident=2)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, 64), 64, 0.5, res)
        stats = ef.ef_get_stats(st.ctx)
        assert stats["misses"] > 0 and stats["bytes_copied"] % ef.ef_expert_bytes_q4(cfg.d, cfg.F) == 0
    finally:
        st.close()


def test_q4_full_size_mixtral_decode(oracle_mod):
    """The headline decode shape with 4-bit experts: T = 64 on the two resident experts (the
    benchmark's launch configuration) and T = 8 spread over more experts; sampled tokens."""
    cfg = q4_shape("mixtral_decode", name="mixtral_decode_q4")
    st = LayerStack(cfg, 1, slots_total=8, max_tokens=64, q4=True)
    try:
        res = synth.residency(cfg, 0)
        for e in np.nonzero(res)[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        for T, beta, n_sample in [(64, 16.0, 4), (8, 1.0, 3)]:
            say(f"q4 full size: Mixtral-shaped decode layer, T={T}, beta={beta}")
            res_now = ef.ef_cache_query(st.ctx, 0, cfg.E)
            toks = np.sort(np.random.default_rng(T).permutation(T)[:n_sample])
            layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, beta, res_now, toks)
    finally:
        st.close()


@pytest.mark.parametrize("kw,T,tiled", [
    (dict(d=256, F=128), 1500, True),            # every expert above 8 tiles, smallest shape the tiled kernels take
    (dict(d=512, F=384), 900, True),             # popularity skew: some experts tiled, the others streamed in passes
    (dict(d=512, F=384), 900, False),            # the same batch with the tiled kernels switched off
    (dict(d=384, F=256), 1500, True),            # d not a multiple of 256: stays on the streaming kernels
])
def test_q4_large_groups_through_tiled_kernels(oracle_mod, kw, T, tiled):
    """Groups of 8 token tiles or more: the 4-bit blobs are expanded to fp16 blobs and go through the
    matrix-core tiled kernels; smaller groups of the same layer keep the streaming kernels."""
    cfg = q4_shape("tiny", name="tiny_q4_prefill", **kw)
    say(f"q4 large groups d={cfg.d} F={cfg.F} E={cfg.E} k={cfg.k} T={T} tiled={tiled}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=T, q4=True, flags=ef.EF_FLAG_PROFILE)
    try:
        if not tiled:
            ef.ef_set_tuning(st.ctx, tiled=0)
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, 0.0, res)
        launches = dict(zip(ef.EF_KERNELS, ef.ef_get_stats(st.ctx)["kernel_launches"]))
        say(f"  launches {launches}")
        expect_tiled = tiled and cfg.d % 256 == 0
        assert (launches["ffn_up_tiled"] > 0) == expect_tiled and (launches["ffn_down_tiled"] > 0) == expect_tiled
    finally:
        st.close()


def test_q4_full_size_mixtral_prefill(oracle_mod):
    """The prefill shape with 4-bit experts (T = 8192, every expert far above 8 tiles: expansion to fp16 and
    the tiled kernels, the configuration `bench.py --workload mixtral_prefill --int4 --all-resident` times);
    sampled tokens."""
    cfg = q4_shape("mixtral_prefill", name="mixtral_prefill_q4")
    T = 8192
    say(f"q4 full size: Mixtral-shaped prefill layer, T={T}")
    st = LayerStack(cfg, 1, slots_total=8, max_tokens=T, q4=True, flags=ef.EF_FLAG_PROFILE)
    try:
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        toks = np.sort(np.random.default_rng(T).permutation(T)[:4])
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, 0.0, res, toks)
        launches = dict(zip(ef.EF_KERNELS, ef.ef_get_stats(st.ctx)["kernel_launches"]))
        assert launches["ffn_up_tiled"] == 1 and launches["ffn_down_tiled"] == 1
    finally:
        st.close()


@pytest.mark.parametrize("T,tiled_shared", [(130, False), (1, False), (300, True), (515, True)])
def test_q4_shared_ffn(oracle_mod, T, tiled_shared):
    """DeepSeek-like layer whose routed experts and dense shared FFN are all 4-bit: the shared group streams
    with the routed ones while it has fewer than 8 token tiles and takes the expansion + tiled kernels above."""
    cfg = dataclasses.replace(synth.CONFIGS["deepseek_v2_lite"], name="deepseek_q4_shared", d=256, F=128, F_shared=384)
    say(f"q4 shared FFN d={cfg.d} F={cfg.F} Fs={cfg.F_shared} E={cfg.E} k={cfg.k} T={T}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=max(T, 64), q4=True, flags=ef.EF_FLAG_PROFILE)
    try:
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, 0.0, res)
        launches = dict(zip(ef.EF_KERNELS, ef.ef_get_stats(st.ctx)["kernel_launches"]))
        assert (launches["ffn_up_tiled"] > 0) == tiled_shared and (launches["ffn_down_tiled"] > 0) == tiled_shared
    finally:
        st.close()


def test_q4_full_size_qwen_mixed_batch(oracle_mod):
    """Qwen1.5-MoE-shaped layer, T = 640, 60 routed experts and the 5632-wide shared FFN all 4-bit
    (`bench.py --workload qwen15_moe --int4`): shared FFN expanded and tiled, routed experts streamed; sampled tokens."""
    cfg = dataclasses.replace(synth.CONFIGS["qwen15_moe"], name="qwen15_moe_q4")
    T = 640
    say(f"q4 full size: Qwen-shaped layer, T={T}, shared FFN {cfg.F_shared}")
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=T, q4=True, flags=ef.EF_FLAG_PROFILE)
    try:
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 0, e, 0, 0)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        toks = np.sort(np.random.default_rng(T).permutation(T)[:6])
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, 0.0, res, toks)
        launches = dict(zip(ef.EF_KERNELS, ef.ef_get_stats(st.ctx)["kernel_launches"]))
        assert launches["ffn_up_tiled"] == 1 and launches["ffn_down_tiled"] == 1 and launches["ffn_up"] == 1
    finally:
        st.close()


def test_q4_large_groups_in_phases(oracle_mod):
    """More active experts (of 8+ token tiles each) than the three cache slots: the call works in phases that
    reuse the slots and the fp16 staging copies; every phase expands its own experts before its tiled launches."""
    cfg = q4_shape("tiny", name="tiny_q4_phases", d=256, F=256)
    T = 1500
    say(f"q4 large groups in phases d={cfg.d} F={cfg.F} E={cfg.E} k={cfg.k} T={T}, 3 slots")
    st = LayerStack(cfg, 1, slots_total=3, max_tokens=T, q4=True, flags=ef.EF_FLAG_PROFILE)
    try:
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        assert res.sum() == 0
        layer_check(oracle_mod, st, synth.hidden(cfg, 0, T), T, 0.0, res)
        stats = ef.ef_get_stats(st.ctx)
        launches = dict(zip(ef.EF_KERNELS, stats["kernel_launches"]))
        say(f"  misses {stats['misses']}, launches {launches}")
        assert stats["misses"] > 3 and launches["ffn_up_tiled"] >= 2 and launches["ffn_down_tiled"] >= 2    # more experts than slots
    finally:
        st.close()


def test_q4_create_rejects_bad_shapes():
    for kw in (dict(d_model=192, d_ff=128), dict(d_model=128, d_ff=96), dict(d_model=128, d_ff=128, d_ff_shared=96)):
        args = dict(n_layers=1, d_model=128, n_experts=4, top_k=2, d_ff=128, slots_total=4, max_tokens=8,
                    weight_bits=4)
        args.update(kw)
        with pytest.raises(ef.EfError):
            ef.ef_create(**args)
