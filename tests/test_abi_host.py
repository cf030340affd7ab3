"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, packs weights
into the documented layout, validates arguments, and its cache runtime (run against the fake copy
engine and fake clock) follows the two-level LRU model, the horizon equation and the feedback loop."""
import os
import re

import numpy as np
import pytest

from paper_2510_26730_amd import binding as ef

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(ef.LIB_PATH):
        from paper_2510_26730_amd import build
        build.build()
    return ef.lib()


def test_every_declared_symbol_is_exported(built):
    hdr = open(os.path.join(ROOT, "include", "expertflow.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ef_[a-z_0-9]+)\s*\(", hdr))
    assert declared >= {"ef_predict", "ef_route", "ef_moe_ffn", "ef_cache_swap_in"}
    assert declared == set(ef.EXPORTS)
    for name in declared:
        assert hasattr(built, name), name


def test_expert_bytes_and_strerror():
    assert ef.ef_expert_bytes(4096, 14336) == 3 * 4096 * 14336 * 2 == 352321536
    assert ef.ef_expert_bytes(2048, 1408) == 17301504
    assert ef.ef_expert_bytes(100, 64) == 0 and ef.ef_expert_bytes(64, 48) == 0
    assert ef.ef_strerror(0) == "ok" and "slot" in ef.ef_strerror(ef.EF_EBUSY)


def test_pack_expert_layout():
    """The blob is the documented permutation: rebuild it here from the layout text alone."""
    d, F = 128, 96
    rng = np.random.default_rng(0)
    W1, W3 = (rng.integers(0, 65536, (F, d), dtype=np.uint16) for _ in range(2))
    # W2 leaves as fp16 numbers: bf16 patterns over the whole fp16 range (exponents down to 2^-30: the
    # smallest round to multiples of 2^-24), both signs
    W2 = (rng.integers(0, 2, (d, F)) << 15 | rng.integers(97, 143, (d, F)) << 7 | rng.integers(0, 128, (d, F))).astype(np.uint16)
    W2[0, :4] = [0x0000, 0x8000, 0x0001, 0x3F80]        # zeros, a bf16 subnormal, 1.0
    from paper_2510_26730_amd import synth
    W2h = synth.bf16_to_f32(W2).astype(np.float16).view(np.uint16)     # numpy rounds to nearest even, keeps subnormals
    big = np.abs(synth.bf16_to_f32(W2)) >= 2.0 ** -14
    assert np.array_equal(W2h.view(np.float16)[big].astype(np.float32), synth.bf16_to_f32(W2)[big])   # exact there
    blob = ef.ef_pack_expert(W1, W3, W2).view(np.uint16)
    assert blob.size == 3 * d * F
    ref = np.empty_like(blob)
    pos = 0
    for rb in range(F // 32):
        for W in (W1, W3):
            for kb in range(d // 16):
                for lane in range(64):
                    g, i = lane // 32, lane % 32
                    for t in range(8):
                        ref[pos] = W[rb * 32 + i, kb * 16 + 8 * g + t]
                        pos += 1
    assert pos == 2 * d * F
    for cb in range(d // 32):
        for kb in range(F // 16):
            for lane in range(64):
                g, i = lane // 32, lane % 32
                for t in range(8):
                    ref[pos] = W2h[cb * 32 + i, kb * 16 + 8 * (t // 4) + 4 * g + t % 4]
                    pos += 1
    assert pos == blob.size
    assert np.array_equal(blob, ref)
    assert np.array_equal(np.sort(blob), np.sort(np.concatenate([W1.ravel(), W3.ravel(), W2h.ravel()])))
    for bad in (0x7F80, 0xFF80, 0x7FC0, 0x4780, 0xC780):     # +inf, -inf, NaN, +-65536
        W2b = W2.copy()
        W2b[d - 1, F - 1] = bad
        with pytest.raises(ef.EfError) as ei:
            ef.ef_pack_expert(W1, W3, W2b)
        assert ei.value.code == ef.EF_EINVAL
    W2b = W2.copy()
    W2b[5, 7] = 0x477F                                       # 65280, the largest bf16 below 65536
    assert ef.ef_pack_expert(W1, W3, W2b).view(np.uint16).size == 3 * d * F


def fake_ctx(**kw):
    base = dict(n_layers=8, d_model=64, n_experts=8, top_k=1, d_ff=32, slots_total=4, max_tokens=64,
                flags=ef.EF_FLAG_FAKE_COPY, init_bandwidth_gbps=1.0, init_layer_us=100.0)
    base.update(kw)
    ctx = ef.ef_create(**base)
    for l in range(base["n_layers"]):
        ef.ef_register_layer(ctx, l, None, None, 1, None)
    return ctx


def test_create_rejects_bad_configs():
    for bad in (dict(n_experts=65), dict(top_k=9), dict(top_k=0), dict(d_model=100), dict(d_ff=40),
                dict(slots_total=0), dict(h_max=0), dict(h_max=8), dict(cum_threshold=0.0),
                dict(max_tokens=0)):
        with pytest.raises(ef.EfError) as ei:
            fake_ctx(**bad)
        assert ei.value.code == ef.EF_EINVAL


def test_argument_errors_and_fake_context_has_no_device():
    ctx = fake_ctx()
    try:
        with pytest.raises(ef.EfError) as ei:
            ef.ef_cache_swap_in(ctx, 99, 0)
        assert ei.value.code == ef.EF_EINVAL and "layer" in str(ei.value)
        with pytest.raises(ef.EfError):
            ef.ef_cache_swap_in(ctx, 0, 8)
        with pytest.raises(ef.EfError):
            ef.ef_cache_swap_in(ctx, 0, 0, priority=2)
        with pytest.raises(ef.EfError) as ei:
            ef.ef_route(ctx, 0, 0, 4, 0.0, 0, 0, 0, 0, 0, 0)
        assert ei.value.code == ef.EF_ENOSYS
        with pytest.raises(ef.EfError) as ei:
            ef.ef_predict(ctx, 0, 0, 4, 2, None, None, 0.0, 0, 0)
        assert ei.value.code == ef.EF_ENOSYS
        with pytest.raises(ef.EfError) as ei:      # counts must sum to T*k
            ef.ef_moe_ffn(ctx, 0, 0, 4, 0, 0, np.array([1, 1, 1, 0, 0, 0, 0, 0], np.int32), 0, 0, 0, 0)
        assert ei.value.code == ef.EF_EINVAL
    finally:
        ef.ef_destroy(ctx)
    ctx2 = ef.ef_create(n_layers=2, d_model=64, n_experts=4, top_k=2, d_ff=32, slots_total=2, max_tokens=8,
                        flags=ef.EF_FLAG_FAKE_COPY)
    with pytest.raises(ef.EfError) as ei:           # unregistered layer
        ef.ef_cache_swap_in(ctx2, 0, 0)
    assert ei.value.code == ef.EF_EINVAL
    ef.ef_destroy(ctx2)


def counts_for(experts, E=8, T=None, k=1):
    """A counts vector that uses exactly `experts` and sums to T*k."""
    T = len(experts) if T is None else T
    c = np.zeros(E, np.int32)
    tot = T * k
    for i, e in enumerate(experts):
        c[e] = tot // len(experts) + (1 if i < tot % len(experts) else 0)
    assert c.sum() == tot and c.max() <= T
    return c


def run_layer(ctx, layer, experts, T=8):
    ef.ef_moe_ffn(ctx, layer, 0, T, 0, 0, counts_for(experts, T=T), 0, 0, 0, 0)


def test_cache_runtime_follows_the_lru_model():
    """Drive ef_cache_swap_in / ef_moe_ffn and the Python model with the same scripted trace."""
    from oracle.lru_model import TwoLevelLRU
    from cache_replay import replay_layer
    rng = np.random.default_rng(5)
    for cap in (0, 2):
        ctx = fake_ctx(slots_total=6, slots_per_layer_max=cap, n_layers=6)
        model = TwoLevelLRU(6, cap, n_layers=6, top_k=1)
        try:
            for step in range(40):
                layer = step % 6
                # prefetch for the next layers
                for j in (1, 2):
                    if layer + j < 6:
                        for e in rng.permutation(8)[:2]:
                            r = model.swap_in(layer + j, int(e), due_in=j)
                            if r == "busy":
                                with pytest.raises(ef.EfError):
                                    ef.ef_cache_swap_in(ctx, layer + j, int(e), 0, j)
                            else:
                                ef.ef_cache_swap_in(ctx, layer + j, int(e), 0, j)
                # the layer itself needs two experts: resident ones are touched, the others are misses
                need = sorted(int(e) for e in rng.permutation(8)[:2])
                replay_layer(model, layer, need)
                run_layer(ctx, layer, need)
                for l in range(6):
                    got = ef.ef_cache_query(ctx, l, 8)
                    want = np.array([model.resident(l, e) for e in range(8)], np.uint8)
                    assert np.array_equal(got, want), (cap, step, l)
        finally:
            ef.ef_destroy(ctx)


def test_moe_ffn_swaps_in_misses_and_reports_busy_when_nothing_can_be_freed():
    ctx = fake_ctx(slots_total=4, slots_per_layer_max=2)
    try:
        run_layer(ctx, 0, [0, 1, 2, 3, 4])           # 5 experts through 2 slots: phases reuse the slots
        st = ef.ef_get_stats(ctx)
        assert st["misses"] == 5 and st["hits"] == 0 and st["layers_run"] == 1
        assert st["bytes_copied"] == 5 * ef.ef_expert_bytes(64, 32)
        assert st["bytes_timed"] == st["bytes_copied"] and st["copy_seconds"] > 0     # modelled copies are all timed
        assert ef.ef_cache_query(ctx, 0, 8).sum() == 2
        assert abs(st["miss_rate"] - 1.0) < 1e-12
        run_layer(ctx, 0, [int(e) for e in np.nonzero(ef.ef_cache_query(ctx, 0, 8))[0]])
        st = ef.ef_get_stats(ctx)
        assert st["hits"] == 2 and st["misses"] == 5
        assert abs(st["miss_rate"] - (1 - 2 / 7)) < 1e-12      # R_miss = 1 - N_selected / N_total
    finally:
        ef.ef_destroy(ctx)
    ctx = fake_ctx(flags=ef.EF_FLAG_FAKE_COPY | ef.EF_FLAG_STRICT_RESIDENT)
    try:
        with pytest.raises(ef.EfError) as ei:
            run_layer(ctx, 0, [3])
        assert ei.value.code == ef.EF_ENOTRESIDENT
        ef.ef_cache_swap_in(ctx, 0, 3, 1)
        run_layer(ctx, 0, [3])
    finally:
        ef.ef_destroy(ctx)


def test_fake_clock_stall_accounting_matches_swap_in_latency_formula():
    """swap-in latency = experts * size / bandwidth (paper Sec. 2.3.1): with a 1 GB/s link and
    6144-byte experts each copy takes 6.144 us on the fake clock."""
    ctx = fake_ctx(init_bandwidth_gbps=1.0)
    es = ef.ef_expert_bytes(64, 32)
    try:
        run_layer(ctx, 0, [0, 1])                     # two misses, serial on the miss queue
        st = ef.ef_get_stats(ctx)
        assert abs(st["stall_seconds"] - 2 * es / 1e9) < 1e-12
        ef.ef_cache_swap_in(ctx, 1, 4, 0, 1)          # prefetch, then enough compute time passes
        ef.ef_fake_advance_time(ctx, 1.0)
        run_layer(ctx, 1, [4])
        st2 = ef.ef_get_stats(ctx)
        assert st2["stall_seconds"] == st["stall_seconds"]      # fully hidden
        ef.ef_cache_swap_in(ctx, 2, 5, 0, 1)          # prefetch still in flight when needed
        ef.ef_fake_advance_time(ctx, es / 1e9 / 4)
        run_layer(ctx, 2, [5])
        st3 = ef.ef_get_stats(ctx)
        assert abs((st3["stall_seconds"] - st2["stall_seconds"]) - 0.75 * es / 1e9) < 1e-12
        assert st3["prefetch_issued"] == 2 and st3["hits"] == 2 and st3["misses"] == 2
    finally:
        ef.ef_destroy(ctx)


def test_choose_horizon_matches_the_step_size_equation(oracle_mod):
    E = 8
    ctx = fake_ctx(init_bandwidth_gbps=0.001, init_layer_us=2000.0, h_max=7, cum_threshold=0.8,
                   stall_thresh=1000, overfetch_thresh=1000, slots_total=16)
    es = ef.ef_expert_bytes(64, 32)
    try:
        ef.ef_cache_swap_in(ctx, 1, 2, 0, 1)
        rng = np.random.default_rng(11)
        tau = float(np.float32(0.8))          # the config field is a C float
        for _ in range(10):
            hist = rng.integers(0, 9, (3, E)).astype(np.int32)
            res1 = ef.ef_cache_query(ctx, 1, E)
            n_e, n_miss, order = oracle_mod.expected_activations(hist[0], tau, res1)
            want = oracle_mod.horizon(n_miss, es, 0.001e9, 2000e-6, 7)
            S, lst = ef.ef_choose_horizon(ctx, 0, hist, 16)
            assert S == want
            exp_list = []
            for j in range(min(3, S)):
                resj = ef.ef_cache_query(ctx, 1 + j, E)
                nj, _, oj = oracle_mod.expected_activations(hist[j], tau, resj)
                exp_list += [(j + 1, int(e)) for e in oj[:nj] if not resj[e]]
            assert lst == exp_list
            assert ef.ef_get_stats(ctx)["horizon"] == S
        S, lst = ef.ef_choose_horizon(ctx, 7, np.zeros((2, E), np.int32), 16)   # last layer: nothing ahead
        assert S == 1 and lst == []
    finally:
        ef.ef_destroy(ctx)


def test_feedback_loop_moves_the_horizon():
    """Stalls push S up by one per `stall_thresh` stalled layers, clean layers pull it down
    (paper Sec. 3.2.2)."""
    ctx = fake_ctx(stall_thresh=2, overfetch_thresh=3, h_max=5, slots_total=16, init_bandwidth_gbps=1000.0)
    hist = np.zeros((1, 8), np.int32)
    hist[0, 0] = 8
    try:
        assert ef.ef_choose_horizon(ctx, 0, hist, 8)[0] == 1
        for i in range(4):
            run_layer(ctx, 0, [i])                     # every layer misses -> stall
        assert ef.ef_choose_horizon(ctx, 0, hist, 8)[0] == 3      # 1 + 4 // 2
        for i in range(3):
            run_layer(ctx, 0, [0])                     # resident and ready -> overfetch counter
        assert ef.ef_choose_horizon(ctx, 0, hist, 8)[0] == 2
        st = ef.ef_get_stats(ctx)
        assert st["stall_counter"] == 0 and st["overfetch_counter"] == 0
    finally:
        ef.ef_destroy(ctx)


def test_pack_expert_q4_layout():
    """The 4-bit blob against an independent reading of the layout the header describes."""
    import dataclasses
    from paper_2510_26730_amd import synth
    cfg = dataclasses.replace(synth.CONFIGS["tiny"], d=256, F=384, F_shared=0)
    q1, s1, q3, s3, q2, s2 = synth.expert_weights_q4(cfg, 0, 0)
    blob = ef.ef_pack_expert_q4(q1, s1, q3, s3, q2, s2)
    d, F = cfg.d, cfg.F
    assert blob.size == ef.ef_expert_bytes_q4(d, F) == 3 * d * F // 2 + 3 * d * F // 64
    assert ef.ef_expert_bytes_q4(192, 128) == 0 and ef.ef_expert_bytes_q4(128, 96) == 0

    def codes(x):   # dword -> the eight codes t = 0..7
        return [(int(x) >> (4 * (t // 2) + 16 * (t % 2))) & 15 for t in range(8)]

    dw = blob[:d * F].view(np.uint32).reshape(F // 32, d // 64, 2, 64, 4)
    rng = np.random.default_rng(0)
    for _ in range(300):
        rb, kq, which = rng.integers(F // 32), rng.integers(d // 64), rng.integers(2)
        lane, j = rng.integers(64), rng.integers(4)
        g, i = lane >> 5, lane & 31
        c0 = (kq * 4 + j) * 16 + 8 * g
        assert codes(dw[rb, kq, which, lane, j]) == (q1, q3)[which][rb * 32 + i, c0:c0 + 8].tolist()
    dwb = blob[d * F:d * F + d * F // 2].view(np.uint32).reshape(d // 32, F // 64, 64, 4)
    for _ in range(300):
        cb, kq, lane, j = rng.integers(d // 32), rng.integers(F // 64), rng.integers(64), rng.integers(4)
        g, i = lane >> 5, lane & 31
        c0 = (kq * 4 + j) * 16
        assert codes(dwb[cb, kq, lane, j]) == [int(q2[cb * 32 + i, c0 + 8 * (t // 4) + 4 * g + t % 4]) for t in range(8)]
    off = 3 * d * F // 2
    sa = blob[off:off + d * F // 32].view(np.uint16).reshape(F // 32, d // 128, 2, 32)
    assert np.array_equal(sa[:, :, 0, :].transpose(0, 2, 1).reshape(F, d // 128), s1)
    assert np.array_equal(sa[:, :, 1, :].transpose(0, 2, 1).reshape(F, d // 128), s3)
    sb = blob[off + d * F // 32:].view(np.uint16).reshape(d // 32, F // 128, 32)
    assert np.array_equal(sb.transpose(0, 2, 1).reshape(d, F // 128), s2)


def test_tuning_defaults_and_validation():
    """The launch tuning lives in the context: defaults after ef_create, out-of-range values rejected
    without changing anything, and no environment variable steers the library."""
    ctx = fake_ctx()
    try:
        t = ef.ef_get_tuning(ctx)
        assert t["tiled"] == 1 and t["tiled_min_tiles"] == 10 and t["lds_shared_occupancy"] == 0
        assert t["up_want_waves"] == 640 and t["gate_k_split"] == 0 and t["early_pack"] == 1
        assert t["copy_chunk_mib"] == 32 and t["copy_depth"] == 2 and t["tiled_tail_slices"] == 1 and t["down_tail_split"] == 1 and t["dist_form"] == 0
        ef.ef_set_tuning(ctx, tiled=0, down_k_slices=4, up_k_slices=2)
        t2 = ef.ef_get_tuning(ctx)
        assert (t2["tiled"], t2["down_k_slices"], t2["up_k_slices"]) == (0, 4, 2)
        for bad in (dict(tiled=2), dict(tiled_min_tiles=7), dict(up_k_slices=3), dict(down_k_slices=9),
                    dict(gate_k_split=17), dict(lds_shared_occupancy=3), dict(up_want_waves=0),
                    dict(tiled_min_up_wgs=0), dict(early_pack=-1), dict(tiled_tail_slices=3), dict(down_tail_split=2), dict(dist_form=3),
                    dict(copy_chunk_mib=0), dict(copy_depth=9)):
            with pytest.raises(ef.EfError) as ei:
                ef.ef_set_tuning(ctx, **bad)
            assert ei.value.code == ef.EF_EINVAL
            assert ef.ef_get_tuning(ctx) == t2
    finally:
        ef.ef_destroy(ctx)
    src_dir = os.path.join(ROOT, "paper_2510_26730_amd", "csrc")
    for name in os.listdir(src_dir):
        assert "getenv" not in open(os.path.join(src_dir, name)).read(), name
