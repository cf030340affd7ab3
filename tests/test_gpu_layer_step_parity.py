"""GPU parity of the composite entry point at the benchmark's shapes: several layers and steps of
ef_layer_step (device-planned token packing, host-mapped hand-over, misses swapped in inside the call,
prefetches decided by the horizon controller, residency that evolves from layer to layer) against the CPU
oracle, layer by layer:

* routing of the layer with the residency the cache reported before the call (ids bit-exact outside
  near-ties, a valid choice inside; counts, offsets, permutation teacher-forced; weights to 1e-5);
* look-ahead ids and demand histograms of the next layers, same rule;
* output rows of sampled tokens and of the first and last token of every expert group (max-abs 2e-2,
  relative L2 1e-2);
* the horizon the call returns and the residency of every layer after the call against the two-level
  LRU model driven with the same accesses and the step-size equation.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

import helpers
from cache_replay import replay_layer
from helpers import LayerStack, check_ids_valid, check_route, dev_u16, float_close

pytestmark = pytest.mark.gpu

BW_GBPS, LAYER_US = 50.0, 200.0      # fixed estimates of the contexts below


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class CacheMirror:
    """The accesses one ef_layer_step makes to the expert cache, replayed on the reference model
    (oracle/lru_model.py), and the step size from the oracle's expected-activation rule and equation."""

    def __init__(self, oracle_mod, cfg, L, slots_per_layer, expert_bytes, h_max, tau=0.9):
        from oracle.lru_model import TwoLevelLRU
        self.o, self.cfg, self.L, self.es, self.h_max = oracle_mod, cfg, L, expert_bytes, h_max
        self.tau = float(np.float32(tau))            # the configuration field is a C float
        self.model = TwoLevelLRU(L * slots_per_layer, slots_per_layer, n_layers=L, top_k=cfg.k)
        self.S = 1

    def resident(self, layer):
        return np.array([self.model.resident(layer, e) for e in range(self.cfg.E)], np.uint8)

    def run_layer(self, layer, counts):
        replay_layer(self.model, layer, [e for e in range(self.cfg.E) if counts[e] > 0])

    def choose_horizon(self, layer, hist):
        """hist [He, E]: demand of layers layer+1.. as the library's host received it."""
        He = hist.shape[0]
        if He == 0:
            return self.S
        chosen = []
        for j in range(He):
            n_e, _, order = self.o.expected_activations(hist[j], self.tau, None)
            chosen.append([int(e) for e in order[:n_e]])
        n_miss = sum(1 for e in chosen[0] if not self.model.resident(layer + 1, e))
        self.S = self.o.horizon(n_miss, self.es, BW_GBPS * 1e9, LAYER_US * 1e-6, self.h_max)
        self.model.set_S(self.S)
        todo = [(j + 1, e) for j in range(min(He, self.S)) for e in chosen[j]
                if not self.model.resident(layer + 1 + j, e)]
        for j, e in todo:
            self.model.swap_in(layer + j, e, due_in=j)      # "busy" only skips the prefetch
        return self.S


CASES = [
    # name, config, tokens, beta, steps, sampled tokens per layer
    ("mixtral_decode_beta1", "mixtral_decode", 64, 1.0, 2, 6),
    ("mixtral_decode_beta16", "mixtral_decode", 64, 16.0, 2, 12),
    ("deepseek_decode", "deepseek_v2_lite", 32, 2.0, 2, 8),
    ("deepseek_mixed_1056", "deepseek_v2_lite", 1056, 1.0, 2, 8),
    ("qwen_mixed_640", "qwen15_moe", 640, 1.0, 2, 8),
]


@pytest.mark.parametrize("name,cfg_name,T,beta,steps,n_sample", CASES, ids=[c[0] for c in CASES])
def test_layer_step_sequence_against_oracle(oracle_mod, name, cfg_name, T, beta, steps, n_sample):
    cfg = synth.CONFIGS[cfg_name]
    L, h_max = 3, 4
    slots = cfg.slots_per_layer
    say(f"layer-step sequence {name}: {L} layers x {steps} steps, T={T}, beta={beta}, {slots} slots/layer")
    st = LayerStack(cfg, L, slots_total=L * slots, per_layer=slots, max_tokens=T, expert_layers=[0], h_max=h_max,
                    flags=ef.EF_FLAG_FIXED_ESTIMATES, stall_thresh=10 ** 6, overfetch_thresh=10 ** 6,
                    init_bandwidth_gbps=BW_GBPS, init_layer_us=LAYER_US)
    mirror = CacheMirror(oracle_mod, cfg, L, slots, st.es, h_max)
    stream = torch.cuda.current_stream()
    out = torch.empty(T, cfg.d, dtype=torch.float32, device="cuda")
    try:
        for step in range(steps):
            hs = synth.hidden_stack(cfg, L, step=step, T=T)
            for l in range(L):
                say(f"  step {step} layer {l}")
                res = [ef.ef_cache_query(st.ctx, ll, cfg.E) for ll in range(L)]
                for ll in range(L):
                    assert np.array_equal(res[ll], mirror.resident(ll)), ("residency before", step, l, ll)
                He = min(mirror.S, L - 1 - l)
                h = hs[l]
                counts = np.full(cfg.E, -1, np.int32)
                out.fill_(float("nan"))
                hd = dev_u16(h)
                Hn = ef.ef_layer_step(st.ctx, l, hd, T, beta, -1, None, None, out, counts, stream)
                got = ef.ef_layer_step_fetch(st.ctx, T, cfg.k, cfg.E, stream=stream)
                got["counts"] = counts
                out_np = out.cpu().numpy()

                # routing of this layer
                ora = oracle_mod.route(h, st.gates[l], st.biases[l], cfg.k, beta, res[l], renorm=cfg.renorm)
                _, nties = check_route(got, ora, cfg.E, cfg.k, cfg.renorm, oracle_mod=oracle_mod)

                # look-ahead: the same hidden states through the next layers' gates, with their residency
                assert got["pred_ids"].shape[0] == He
                for j in range(He):
                    z = oracle_mod.gate_logits(h, st.gates[l + 1 + j], st.biases[l + 1 + j])
                    s = oracle_mod.scores(z, beta, res[l + 1 + j])
                    oids, ogap = oracle_mod.topk(s, cfg.k)
                    tie = ogap < helpers.TIE_GAP
                    assert np.array_equal(got["pred_ids"][j][~tie], oids[~tie]), ("look-ahead ids", step, l, j)
                    check_ids_valid(got["pred_ids"][j], s, ogap, cfg.k)
                    assert np.array_equal(got["pred_hist"][j], oracle_mod.histogram(got["pred_ids"][j], cfg.E))
                    nties += int(tie.sum())

                # outputs: sampled tokens and the first / last token of every expert group
                edge = [got["perm"][p] // cfg.k for e in range(cfg.E) if counts[e] > 0
                        for p in (got["offsets"][e], got["offsets"][e + 1] - 1)]
                toks = np.unique(np.concatenate([np.random.default_rng(100 * step + l).permutation(T)[:n_sample],
                                                 np.asarray(edge, dtype=np.int64)])).astype(np.int64)
                hsub = np.ascontiguousarray(h[toks])
                ids_s = np.ascontiguousarray(got["ids"][toks])
                sub = oracle_mod.route_from_ids(ora["p"][toks], ids_s, cfg.E, cfg.renorm)
                y = oracle_mod.expert_ffn(hsub, st.experts_of(l), ids_s, sub["perm"])
                sh = None if not cfg.F_shared else oracle_mod.dense_ffn(hsub, *st.shared_of(l))
                ref = oracle_mod.combine(y, sub["w"], sub["inv_perm"], sh)
                assert np.all(np.isfinite(out_np))
                e1, e2 = float_close(out_np[toks], ref)

                # cache decisions
                mirror.run_layer(l, counts)
                S = mirror.choose_horizon(l, got["pred_hist"])
                assert Hn == S, ("horizon", step, l, Hn, S)
                for ll in range(L):
                    assert np.array_equal(ef.ef_cache_query(st.ctx, ll, cfg.E), mirror.resident(ll)), \
                        ("residency after", step, l, ll)
                say(f"    experts used {int((counts > 0).sum())}, near-ties {nties}, {len(toks)} tokens: "
                    f"max abs {e1:.2e}, rel l2 {e2:.2e}, horizon -> {Hn}")
        stats = ef.ef_get_stats(st.ctx)
        say(f"  hits {stats['hits']} misses {stats['misses']} prefetches {stats['prefetch_issued']} "
            f"evictions {stats['evictions']}")
        assert stats["layers_run"] == L * steps
    finally:
        st.close()


def test_handover_words_of_an_earlier_call_are_never_taken_for_new_ones():
    """The demand histogram of look-ahead position j reaches the host in words that only calls with a
    horizon above j rewrite, each tagged with the call's sequence number modulo 255.  A long run at
    horizon 1 between two calls at horizon 3 leaves the words of positions 1 and 2 untouched; when the
    second such call comes exactly one tag period after the first, stale words would carry the right
    tag.  Every call's horizon and every layer's residency must equal those of the separate entry
    points (which copy the histograms with a stream-ordered copy) over more than two tag periods."""
    from paper_2510_26730_amd.runner import LayerLoop
    import dataclasses
    cfg = dataclasses.replace(synth.CONFIGS["tiny"], name="tiny_handover", F=64, n_layers=4)
    L, T = 4, 64
    say("hand-over tags over 530 calls with horizon changes")
    # a link estimate so low that any predicted miss asks for the largest step size: the prefetch list then
    # covers every look-ahead position the call has, and a stale histogram would change the residency
    loops = [LayerLoop(cfg, L, T, cfg.slots_per_layer, beta=0.25, seed=3, fixed_estimates=True,
                       init_bandwidth_gbps=1e-4, stall_thresh=10 ** 6, overfetch_thresh=10 ** 6) for _ in range(2)]
    try:
        stream = torch.cuda.current_stream()
        hs = [torch.from_numpy(synth.hidden_stack(cfg, 1, step=s, T=T).view(np.int16)).cuda()[0] for s in range(7)]
        wide = {1, 256, 257, 511, 512, 513, 514}        # calls (1-based) that look three layers ahead
        for call in range(1, 531):
            H = 3 if call in wide else 1
            for lp in loops:
                lp.h_fixed = H
            h = hs[call % 7]       # calls 1 and 256 (same tag) see different tokens
            loops[0].layer(0, h, stream)
            loops[1].layer_separate_calls(0, h, stream)
            torch.cuda.synchronize()
            assert loops[0].H == loops[1].H, (call, loops[0].H, loops[1].H)
            for ll in range(L):
                assert np.array_equal(ef.ef_cache_query(loops[0].ctx, ll, cfg.E),
                                      ef.ef_cache_query(loops[1].ctx, ll, cfg.E)), (call, ll)
            if call in wide:
                assert torch.equal(loops[0].out, loops[1].out), call
        s0, s1 = ef.ef_get_stats(loops[0].ctx), ef.ef_get_stats(loops[1].ctx)
        for key in ("hits", "misses", "prefetch_issued", "evictions", "bytes_copied"):
            assert s0[key] == s1[key], key
    finally:
        for lp in loops:
            lp.close()
