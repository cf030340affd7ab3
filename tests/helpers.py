"""Shared plumbing of the GPU parity tests: builds a library context for a synthetic layer stack,
runs the hot path through the C ABI and returns numpy results.  No arithmetic of the method here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth


def dev_u16(a: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns -> device tensor (int16 storage; the library only sees the address)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


class LayerStack:
    """Weights of `n_layers` layers of one shape, on the host (row-major, for the oracle) and
    registered with a library context (gates on the device, packed experts in pinned memory)."""

    def __init__(self, cfg: synth.MoEShape, n_layers: int, slots_total: int, per_layer: int = 0,
                 max_tokens: int = 64, expert_layers=None, h_max: int = 4, q4: bool = False, **create_kw):
        self.cfg, self.n_layers, self.q4 = cfg, n_layers, q4
        self.gates = [synth.gate_weight(cfg, l) for l in range(n_layers)]
        self.biases = [synth.gate_bias(cfg, l) for l in range(n_layers)]
        self.expert_layers = list(range(n_layers)) if expert_layers is None else list(expert_layers)
        make = synth.expert_weights_q4 if q4 else synth.expert_weights
        self.experts = {l: [make(cfg, l, e) for e in range(cfg.E)] for l in self.expert_layers}
        make_shared = synth.shared_weights_q4 if q4 else synth.shared_weights
        self.shared = {l: make_shared(cfg, l) for l in self.expert_layers} if cfg.F_shared else {}
        self.ctx = ef.ef_create(n_layers=n_layers, d_model=cfg.d, n_experts=cfg.E, top_k=cfg.k, d_ff=cfg.F,
                                d_ff_shared=cfg.F_shared, slots_total=slots_total,
                                slots_per_layer_max=per_layer, max_tokens=max_tokens, h_max=h_max,
                                renorm_topk=int(cfg.renorm), weight_bits=4 if q4 else 0, **create_kw)
        self.es = ef.ef_expert_bytes_q4(cfg.d, cfg.F) if q4 else ef.ef_expert_bytes(cfg.d, cfg.F)
        pack = ef.ef_pack_expert_q4 if q4 else ef.ef_pack_expert
        self._keep = []
        packed = {}    # layers without expert weights of their own register the packed store of the first layer that has
        for l in range(n_layers):
            gw, gb = dev_u16(self.gates[l]), torch.from_numpy(self.biases[l]).cuda()
            src = l if l in self.experts else self.expert_layers[0]
            if src not in packed:
                store = torch.empty(cfg.E * self.es, dtype=torch.uint8, pin_memory=True)
                sv = store.numpy()
                for e in range(cfg.E):
                    pack(*self.experts[src][e], blob=sv[e * self.es:(e + 1) * self.es])
                sh = None
                if cfg.F_shared:
                    if q4:
                        sb = np.empty(ef.ef_expert_bytes_q4(cfg.d, cfg.F_shared), dtype=np.uint8)
                        ef.ef_pack_expert_q4(*self.shared[src], blob=sb)
                        sh = torch.from_numpy(sb).cuda()
                    else:
                        sh = torch.from_numpy(ef.ef_pack_expert(*self.shared[src])).cuda()
                packed[src] = (store, sh)
            store, sh = packed[src]
            ef.ef_register_layer(self.ctx, l, gw, gb, store, sh)
            self._keep += [gw, gb, store, sh]

    def experts_of(self, layer):
        """Row-major expert weights the oracle uses for `layer` (its own, or those of the layer it shares a store with)."""
        return self.experts[layer if layer in self.experts else self.expert_layers[0]]

    def shared_of(self, layer):
        return self.shared.get(layer if layer in self.experts else self.expert_layers[0]) if self.cfg.F_shared else None

    def close(self):
        torch.cuda.synchronize()
        ef.ef_destroy(self.ctx)
        self._keep.clear()

    # ---- calls -------------------------------------------------------------------------------
    def route(self, layer, h_dev, T, beta):
        c = self.cfg
        n = max(1, T * c.k)
        o = dict(ids=torch.full((n,), -1, dtype=torch.int32, device="cuda"),
                 w=torch.full((n,), -1.0, dtype=torch.float32, device="cuda"),
                 counts=torch.full((c.E,), -1, dtype=torch.int32, device="cuda"),
                 offsets=torch.full((c.E + 1,), -1, dtype=torch.int32, device="cuda"),
                 perm=torch.full((n,), -1, dtype=torch.int32, device="cuda"),
                 inv_perm=torch.full((n,), -1, dtype=torch.int32, device="cuda"))
        ef.ef_route(self.ctx, layer, h_dev, T, beta, o["ids"], o["w"], o["counts"], o["offsets"], o["perm"],
                    o["inv_perm"], torch.cuda.current_stream())
        return o

    def ffn(self, layer, h_dev, T, r):
        out = torch.full((max(1, T), self.cfg.d), float("nan"), dtype=torch.float32, device="cuda")
        counts_host = r["counts"].cpu().numpy()
        ef.ef_moe_ffn(self.ctx, layer, h_dev, T, r["ids"], r["w"], counts_host, r["offsets"], r["perm"],
                      r["inv_perm"], out, torch.cuda.current_stream())
        torch.cuda.synchronize()
        return out.cpu().numpy()[:T]

    def predict(self, layer, h_dev, T, H, beta, delta=None, tok2req=None):
        c = self.cfg
        ids = torch.full((max(1, H * T * c.k),), -1, dtype=torch.int32, device="cuda")
        hist = torch.full((max(1, H * c.E),), -1, dtype=torch.int32, device="cuda")
        d_dev = None if delta is None else torch.from_numpy(delta).cuda()
        t_dev = None if tok2req is None else torch.from_numpy(tok2req).cuda()
        he = ef.ef_predict(self.ctx, layer, h_dev, T, H, d_dev, t_dev, beta, ids, hist,
                           torch.cuda.current_stream())
        torch.cuda.synchronize()
        return he, ids.cpu().numpy()[:H * T * c.k].reshape(H, T, c.k), hist.cpu().numpy()[:H * c.E].reshape(H, c.E)


def to_np(r, T, k):
    torch.cuda.synchronize()
    n = T * k
    return dict(ids=r["ids"].cpu().numpy()[:n].reshape(T, k), w=r["w"].cpu().numpy()[:n].reshape(T, k),
                counts=r["counts"].cpu().numpy(), offsets=r["offsets"].cpu().numpy(),
                perm=r["perm"].cpu().numpy()[:n], inv_perm=r["inv_perm"].cpu().numpy()[:n])


TIE_GAP = 1e-4


def check_route(got, ora, E, k, renorm, routed_scale=1.0, oracle_mod=None):
    """Bit-exact ids / counts / offsets / perm outside near-ties; what follows from the ids is
    re-derived by the oracle from the library's ids (teacher forcing) and must match exactly."""
    T = ora["ids"].shape[0]
    tie = ora["gap"] < TIE_GAP
    assert np.array_equal(got["ids"][~tie], ora["ids"][~tie]), "expert ids differ outside near-ties"
    for t in np.nonzero(tie)[0]:       # a near-tie may pick either side, but must be a valid choice
        s = ora["s"][t]
        kth = np.sort(s)[::-1][k - 1]
        assert np.all(s[got["ids"][t]] >= kth - TIE_GAP)
        assert len(set(got["ids"][t].tolist())) == k and np.all(np.diff(got["ids"][t]) > 0)
    forced = oracle_mod.route_from_ids(ora["p"], got["ids"], E, renorm, routed_scale)
    for name in ("counts", "offsets", "perm", "inv_perm"):
        assert np.array_equal(got[name], forced[name]), name
    assert np.max(np.abs(got["w"] - forced["w"])) < 1e-5
    return forced, int(tie.sum())


def check_ids_valid(ids, s, gap, k):
    """Expert ids [T,k] against oracle scores s [T,E] and gaps [T]: equal to the oracle's choice outside
    near-ties (the caller checks that); inside a near-tie a valid choice: k distinct ids in ascending
    order, each scoring within the tie gap of the k-th best score."""
    for t in np.nonzero(gap < TIE_GAP)[0]:
        kth = np.sort(s[t])[::-1][k - 1]
        assert np.all(s[t][ids[t]] >= kth - TIE_GAP), t
        assert len(set(ids[t].tolist())) == k and np.all(np.diff(ids[t]) > 0), t


def float_close(got, ref, max_abs=2e-2, rel_l2=1e-2):
    err = np.abs(got.astype(np.float64) - ref)
    l2 = np.linalg.norm(got.astype(np.float64) - ref) / max(np.linalg.norm(ref), 1e-30)
    assert np.all(np.isfinite(got)), "non-finite output"
    assert err.max() <= max_abs and l2 <= rel_l2, (err.max(), l2)
    return err.max(), l2
