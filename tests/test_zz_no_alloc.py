"""ef_route_static (routing without device allocation: scratch in a static device array of the library)
against ef_route through the C ABI: every output bit-identical, on two calls in a row of which the
second has the smaller input, and no device memory taken by the calls."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

from helpers import LayerStack, check_route, dev_u16, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def shape(base, **kw):
    return dataclasses.replace(synth.CONFIGS[base], **kw)


CASES = [
    # routing only: experts of the smallest legal size
    ("mixtral_gate", shape("mixtral_decode", name="mixtral_gate", F=32), [(64, 16.0), (33, 1.0), (1, 0.0)]),
    ("deepseek_gate", shape("deepseek_v2_lite", name="deepseek_gate", F=32, F_shared=0), [(1056, 1.0), (32, 2.0)]),
    ("qwen_gate", shape("qwen15_moe", name="qwen_gate", F=32, F_shared=0), [(2500, 0.5), (640, 1.0), (7, 0.0)]),
]


def route_with(fn, st, hd, T, beta):
    c = st.cfg
    n = max(1, T * c.k)
    o = dict(ids=torch.full((n,), -1, dtype=torch.int32, device="cuda"),
             w=torch.full((n,), -1.0, dtype=torch.float32, device="cuda"),
             counts=torch.full((c.E,), -1, dtype=torch.int32, device="cuda"),
             offsets=torch.full((c.E + 1,), -1, dtype=torch.int32, device="cuda"),
             perm=torch.full((n,), -1, dtype=torch.int32, device="cuda"),
             inv_perm=torch.full((n,), -1, dtype=torch.int32, device="cuda"))
    return o, lambda: fn(st.ctx, 0, hd, T, beta, o["ids"], o["w"], o["counts"], o["offsets"], o["perm"],
                         o["inv_perm"], torch.cuda.current_stream())


@pytest.mark.parametrize("name,cfg,calls", CASES, ids=[c[0] for c in CASES])
def test_route_static_equals_route(name, cfg, calls):
    say(f"ef_route_static vs ef_route: {name}, calls {calls}")
    t_ctx = max(T for T, _ in calls)      # ef_route, the reference here, needs the context's scratch for them
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=t_ctx, expert_layers=[0])
    try:
        for e in np.nonzero(synth.residency(cfg, 0))[0]:
            ef.ef_cache_swap_in(st.ctx, 0, int(e), 0, 0)
        torch.cuda.synchronize()
        inputs = [(T, beta, dev_u16(synth.hidden(cfg, 7 + i, T))) for i, (T, beta) in enumerate(calls)]
        want = []
        for T, beta, hd in inputs:
            o, call = route_with(ef.ef_route, st, hd, T, beta)
            call()
            want.append(to_np(o, T, cfg.k))
        # the static calls, back to back on one stream (the second, smaller one finds the first one's leftovers
        # in the scratch); buffers prepared first, so that the only device work between the two memory readings
        # is the calls themselves
        outs = [route_with(ef.ef_route_static, st, hd, T, beta) for T, beta, hd in inputs]
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        for _, call in outs:
            call()
        torch.cuda.synchronize()
        free1 = torch.cuda.mem_get_info()[0]
        assert free1 == free0, ("device memory changed across the static calls", free0, free1)
        for (T, beta, _), (o, _), w in zip(inputs, outs, want):
            got = to_np(o, T, cfg.k)
            for key in w:
                assert np.array_equal(got[key], w[key]), (T, beta, key)
            assert got["counts"].sum() == T * cfg.k
    finally:
        st.close()


def test_route_static_rejects_batches_beyond_its_scratch(oracle_mod):
    cfg = shape("tiny", name="tiny_gate", F=32)
    st = LayerStack(cfg, 1, slots_total=cfg.E, max_tokens=64, expert_layers=[0])
    try:
        hd = dev_u16(synth.hidden(cfg, 0, 64))
        o, _ = route_with(ef.ef_route_static, st, hd, 64, 0.0)
        with pytest.raises(ef.EfError) as ei:
            ef.ef_route_static(st.ctx, 0, hd, 8193, 0.0, o["ids"], o["w"], o["counts"], o["offsets"], o["perm"],
                               o["inv_perm"], torch.cuda.current_stream())
        assert ei.value.code == ef.EF_EINVAL and "8192" in str(ei.value)
        # the context was created for 64 tokens; a larger batch is fine for the static call
        T = 300
        h = synth.hidden(cfg, 1, T)
        hd = dev_u16(h)
        o, call = route_with(ef.ef_route_static, st, hd, T, 0.25)
        call()
        got = to_np(o, T, cfg.k)
        res = ef.ef_cache_query(st.ctx, 0, cfg.E)
        ora = oracle_mod.route(h, st.gates[0], st.biases[0], cfg.k, 0.25, res, renorm=cfg.renorm)
        check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)
        with pytest.raises(ef.EfError):
            ef.ef_route(st.ctx, 0, hd, T, 0.25, o["ids"], o["w"], o["counts"], o["offsets"], o["perm"], o["inv_perm"],
                        torch.cuda.current_stream())
    finally:
        st.close()
