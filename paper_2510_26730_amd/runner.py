"""Layer loop over the C ABI: the order of calls of one decode / prefill step.

Call sequencing and buffer ownership only; all arithmetic and all cache policy
live in the library.  Per layer l:

    ef_route_predict(l)  one pass over the hidden states: the layer's own gate (softmax, biased
                         top-k, grouping) and the gates of l+1..l+H (demand histograms)
    -- counts and histograms reach the host --
    ef_choose_horizon(l) -> H for the next layer, prefetch list
    ef_cache_swap_in(...) prefetches on the copy stream
    ef_moe_ffn(l)   resident groups first, misses swapped in and run after

`layer` uses the library's composite ef_layer_step, `layer_separate_calls` spells the sequence out.

Weights for benchmarks are random bf16 written straight in packed order (a
permutation of i.i.d. draws is i.i.d.), optionally one small pool of layer
stores reused cyclically so that an 84 GiB model does not have to be
materialised on the host.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as ef
from . import synth


class LayerLoop:
    def __init__(self, cfg: synth.MoEShape, n_layers: int, T: int, slots_per_layer: int,
                 pool_slots: int | None = None, store_layers: int = 2, h_max: int = 4, beta: float = 0.0,
                 profile: bool = False, all_resident: bool = False, seed: int = 0,
                 fixed_estimates: bool = False, q4: bool = False, **create_kw):
        self.cfg, self.L, self.T, self.beta = cfg, n_layers, T, beta
        E, k, d = cfg.E, cfg.k, cfg.d
        dev = "cuda"
        slots_total = n_layers * (E if all_resident else slots_per_layer) if pool_slots is None else pool_slots
        flags = {False: 0, True: ef.EF_FLAG_PROFILE, "ffn_up": ef.EF_FLAG_PROFILE_FFN_UP}[profile]
        flags |= ef.EF_FLAG_FIXED_ESTIMATES if fixed_estimates else 0
        self.ctx = ef.ef_create(n_layers=n_layers, d_model=d, n_experts=E, top_k=k, d_ff=cfg.F,
                                d_ff_shared=cfg.F_shared, slots_total=slots_total,
                                slots_per_layer_max=0 if all_resident or pool_slots is not None else slots_per_layer,
                                max_tokens=T, h_max=h_max, renorm_topk=int(cfg.renorm), flags=flags,
                                weight_bits=4 if q4 else 0, **create_kw)
        self.q4 = q4
        self.es = ef.ef_expert_bytes_q4(d, cfg.F) if q4 else ef.ef_expert_bytes(d, cfg.F)
        g = torch.Generator(device=dev)
        g.manual_seed(synth.BASE_SEED * 100 + cfg.cfg_id * 10 + seed)
        self.store_layers = min(store_layers, n_layers)
        self.stores = []
        for _ in range(self.store_layers):
            if q4:
                # 4-bit blobs drawn directly in packed order: uniform codes (every byte of the code sections
                # holds two) and one constant scale, so that (q - 8) * s has the standard deviation w_std
                st = torch.empty(E * self.es, dtype=torch.uint8, pin_memory=True)
                ncode = 3 * d * cfg.F // 2
                scale = torch.full(((self.es - ncode) // 2,), cfg.w_std / 4.61, dtype=torch.bfloat16, device=dev)
                for e in range(E):
                    codes = torch.randint(0, 256, (ncode,), generator=g, device=dev, dtype=torch.uint8)
                    st[e * self.es:e * self.es + ncode].copy_(codes)
                    st[e * self.es + ncode:(e + 1) * self.es].copy_(scale.view(torch.uint8))
                self.stores.append(st)
                continue
            st = torch.empty(E * self.es // 2, dtype=torch.int16, pin_memory=True)
            for e in range(E):           # one expert at a time keeps the device staging buffer small
                st[e * (self.es // 2):(e + 1) * (self.es // 2)].copy_(self._random_blob(d, cfg.F, cfg.w_std, g))
            self.stores.append(st)
        self.shared = []
        if cfg.F_shared and q4:
            nb = ef.ef_expert_bytes_q4(d, cfg.F_shared)
            ncode = 3 * d * cfg.F_shared // 2
            for _ in range(self.store_layers):
                sb = torch.empty(nb, dtype=torch.uint8, device=dev)
                sb[:ncode] = torch.randint(0, 256, (ncode,), generator=g, device=dev, dtype=torch.uint8)
                sb[ncode:] = torch.full(((nb - ncode) // 2,), cfg.w_std / 4.61, dtype=torch.bfloat16,
                                        device=dev).view(torch.uint8)
                self.shared.append(sb)
        elif cfg.F_shared:
            for _ in range(self.store_layers):
                self.shared.append(self._random_blob(d, cfg.F_shared, cfg.w_std, g))
        self.gate_w, self.gate_b = [], []
        for l in range(n_layers):
            self.gate_w.append(torch.from_numpy(synth.gate_weight(cfg, l).view(np.int16)).to(dev))
            self.gate_b.append(torch.from_numpy(synth.gate_bias(cfg, l)).to(dev))
            ef.ef_register_layer(self.ctx, l, self.gate_w[l], self.gate_b[l], self.stores[l % self.store_layers],
                                 self.shared[l % self.store_layers] if cfg.F_shared else None)
        i32 = dict(dtype=torch.int32, device=dev)
        n = T * k
        self.ids = torch.empty(n, **i32)
        self.w = torch.empty(n, dtype=torch.float32, device=dev)
        # counts and the predicted histograms sit in one buffer so that one copy brings both to the host
        self.meta = torch.zeros(E + ef.EF_MAX_HORIZON * E, **i32)
        self.counts, self.hist = self.meta[:E], self.meta[E:]
        self.meta_host = torch.zeros(E + ef.EF_MAX_HORIZON * E, dtype=torch.int32, pin_memory=True)
        self.offsets = torch.empty(E + 1, **i32)
        self.perm = torch.empty(n, **i32)
        self.inv_perm = torch.empty(n, **i32)
        self.pred_ids = torch.empty(ef.EF_MAX_HORIZON * n, **i32)
        self.out = torch.empty(T, d, dtype=torch.float32, device=dev)
        self.H = 1
        self.h_fixed = None
        self.delta = None        # [R, H, E] float32 on the device: deviation added to the look-ahead logits
        self.tok2req = None      # [T] int32 on the device: request of each token (None: token t is request t)
        torch.cuda.synchronize()
        if all_resident:
            for l in range(n_layers):
                for e in range(E):
                    ef.ef_cache_swap_in(self.ctx, l, e, 0, 0)
            torch.cuda.synchronize()
            ef.ef_get_stats(self.ctx)

    @staticmethod
    def _random_blob(d, F, std, g):
        """A packed expert of i.i.d. N(0, std^2) weights rounded to bf16, drawn directly in packed order on the
        device: W1 / W3 fragments as bf16 bit patterns, the W2 section as the fp16 numbers equal to them."""
        w = torch.randn(3 * d * F, generator=g, device="cuda", dtype=torch.float32).mul_(std).to(torch.bfloat16)
        blob = torch.empty(3 * d * F, dtype=torch.int16, device="cuda")
        blob[:2 * d * F] = w[:2 * d * F].view(torch.int16)
        blob[2 * d * F:] = w[2 * d * F:].to(torch.float16).view(torch.int16)
        return blob

    def close(self):
        torch.cuda.synchronize()
        ef.ef_destroy(self.ctx)

    def layer(self, l: int, h: torch.Tensor, stream) -> None:
        """One layer through the composite entry point (the library sequences the calls)."""
        H = -1 if self.h_fixed is None else self.h_fixed
        self.H = ef.ef_layer_step(self.ctx, l, h, self.T, self.beta, H, self.delta, self.tok2req, self.out, None, stream)

    def layer_separate_calls(self, l: int, h: torch.Tensor, stream) -> None:
        """The same layer through the separate entry points (what ef_layer_step does inside)."""
        E, T = self.cfg.E, self.T
        H = self.H if self.h_fixed is None else self.h_fixed
        he = ef.ef_route_predict(self.ctx, l, h, T, self.beta, H, self.delta, self.tok2req, self.ids, self.w, self.counts,
                                 self.offsets, self.perm, self.inv_perm, self.pred_ids, self.hist, stream)
        self.meta_host.copy_(self.meta, non_blocking=True)
        stream.synchronize()
        mh = self.meta_host.numpy()
        # the FFN is enqueued first (the GPU is idle until then); the prefetch copies decided afterwards
        # overlap it
        ef.ef_moe_ffn(self.ctx, l, h, T, self.ids, self.w, mh[:E], self.offsets, self.perm, self.inv_perm,
                      self.out, stream)
        if he > 0:
            self.H, lst = ef.ef_choose_horizon(self.ctx, l, mh[E:E + he * E].reshape(he, E), T)
            for j, e in lst:
                try:
                    ef.ef_cache_swap_in(self.ctx, l + j, e, 0, j)
                except ef.EfError as err:       # a full, pinned cache is not an error for a prefetch
                    if err.code != ef.EF_EBUSY:
                        raise

    def step(self, hidden_stack: torch.Tensor, stream) -> None:
        """hidden_stack [L, T, d] bf16 on the device: the inputs of the L layers of this step."""
        for l in range(self.L):
            self.layer(l, hidden_stack[l], stream)
