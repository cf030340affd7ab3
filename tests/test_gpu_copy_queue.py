"""The copy queue on the device (paper Sec. 3.4): expert copies go to the copy stream in chunks, a miss of the
layer being run overtakes queued prefetches at the next chunk boundary, and whatever order the chunks take the
cache slots end up holding exactly the experts' bytes (checked through the FFN output of every expert against the
oracle)."""
import dataclasses
import sys
import time

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

from helpers import LayerStack, dev_u16, float_close, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_chunked_copies_deliver_every_expert_intact(oracle_mod):
    """Experts of 3 MiB in chunks of 1 MiB, two layers: all experts of layer 1 are queued as prefetches, then
    layer 0 runs with every expert missing (priority copies that overtake them), then layer 1 runs on the
    prefetched experts.  Outputs of both layers against the oracle."""
    cfg = synth.CONFIGS["tiny"]
    T = 64
    st = LayerStack(cfg, 2, slots_total=2 * cfg.E, max_tokens=T)
    try:
        ef.ef_set_tuning(st.ctx, copy_chunk_mib=1, copy_depth=2)
        for e in range(cfg.E):
            ef.ef_cache_swap_in(st.ctx, 1, e, 0, 1)
        for layer in (0, 1):
            h = synth.hidden(cfg, 20 + layer, T)
            hd = dev_u16(h)
            res = ef.ef_cache_query(st.ctx, layer, cfg.E)
            r = st.route(layer, hd, T, 0.0)
            got = to_np(r, T, cfg.k)
            out = st.ffn(layer, hd, T, r)
            full = oracle_mod.moe_layer(h, st.gates[layer], st.biases[layer], st.experts[layer], cfg.k, beta=0.0,
                                        resident=res, renorm=cfg.renorm, forced_ids=got["ids"])
            e1, e2 = float_close(out, full["out"])
            say(f"  layer {layer}: max abs {e1:.2e}, rel l2 {e2:.2e}")
        s = ef.ef_get_stats(st.ctx)
        used = int((got["counts"] > 0).sum())
        assert s["prefetch_issued"] == cfg.E and s["prefetch_used"] == used and s["misses"] >= 1
        assert s["miss_copies"] >= s["misses"]
    finally:
        st.close()


@pytest.mark.parametrize("chunk_mib", [16, 32])
def test_a_miss_is_not_held_up_by_queued_prefetches(chunk_mib):
    """Mixtral-sized experts (336 MiB, 6 ms on the link each): six prefetches are queued, then a miss is
    requested.  The miss must complete long before the prefetches queued ahead of it would have let it (it
    waits for the chunks already handed to the link, not for 2 GiB of prefetches), and the link must stay busy
    (aggregate rate of everything copied)."""
    cfg = dataclasses.replace(synth.CONFIGS["mixtral_decode"], name="mixtral_copy")
    E, d, F = cfg.E, cfg.d, cfg.F
    es = ef.ef_expert_bytes(d, F)
    ctx = ef.ef_create(n_layers=2, d_model=d, n_experts=E, top_k=cfg.k, d_ff=F, slots_total=8, max_tokens=32)
    store = torch.zeros(E * es, dtype=torch.uint8).pin_memory()          # only the transfer matters here
    gw = torch.zeros(E, d, dtype=torch.int16, device="cuda")
    try:
        ef.ef_set_tuning(ctx, copy_chunk_mib=chunk_mib, copy_depth=2)
        for l in range(2):
            ef.ef_register_layer(ctx, l, gw, None, store, None)
        ef.ef_cache_swap_in(ctx, 0, 7, 1, 0)                              # warm the link and the worker
        ef.ef_get_stats(ctx)
        ef.ef_reset_stats(ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in range(6):
            ef.ef_cache_swap_in(ctx, 1, e, 0, 1)
        time.sleep(0.004)                                                 # the first prefetch is under way
        ef.ef_cache_swap_in(ctx, 0, 0, 1, 0)                              # the miss
        s = ef.ef_get_stats(ctx)                                          # drains the queue
        total = time.perf_counter() - t0
        miss_ms = 1e3 * s["miss_copy_seconds"] / s["miss_copies"]
        miss_gbps = s["miss_copy_bytes"] / s["miss_copy_seconds"] / 1e9
        link = s["bytes_timed"] / s["copy_seconds"] / 1e9
        say(f"  chunks of {chunk_mib} MiB: miss complete after {miss_ms:.2f} ms ({miss_gbps:.1f} GB/s from its request), "
            f"link {link:.1f} GB/s over the timed chunks, 7 experts in {1e3 * total:.1f} ms "
            f"({7 * es / total / 1e9:.1f} GB/s from the first request)")
        assert s["miss_copies"] == 1 and s["bytes_copied"] == 7 * es
        one = es / (link * 1e9)                                           # one expert on the link
        assert 1e-3 * miss_ms < 1.5 * one, "the miss waited for more than the chunks in flight"
        assert 7 * es / total / 1e9 > 0.85 * link, "the link idled between chunks"
    finally:
        ef.ef_destroy(ctx)
