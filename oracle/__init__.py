"""CPU oracle (test infrastructure only): ctypes front end of ``ef_oracle.c``.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package.  It never imports the HIP package.  bf16 arrays are
``numpy.uint16`` bit patterns; everything else is int32 / float32 / float64.

Composite helpers (`route`, `predict`, `moe_layer`) chain the C steps in the
order the method states them: logits -> softmax -> selection score -> top-k ->
weights -> histogram -> permutation -> expert FFN -> combine.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ef_oracle.c")
_LIB = os.path.join(_HERE, "libef_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_step_size_raw.restype = C.c_double
        _lib.oracle_step_size_raw.argtypes = [C.c_double] * 4
        _lib.oracle_horizon.restype = C.c_int
        _lib.oracle_horizon.argtypes = [C.c_double] * 4 + [C.c_int]
        _lib.oracle_expected_activations.restype = C.c_int
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def gate_logits(h, Wg, b=None):
    h, Wg = _u16(h), _u16(Wg)
    T, d = h.shape
    E = Wg.shape[0]
    assert Wg.shape[1] == d
    b = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
    z = np.empty((T, E), dtype=np.float64)
    lib().oracle_gate_logits(_p(h, C.c_uint16), _p(Wg, C.c_uint16), _p(b, C.c_float),
                             C.c_int(T), C.c_int(d), C.c_int(E), _p(z, C.c_double))
    return z


def softmax(z):
    z = np.ascontiguousarray(z, dtype=np.float64)
    T, E = z.shape
    p = np.empty_like(z)
    lib().oracle_softmax(_p(z, C.c_double), C.c_int(T), C.c_int(E), _p(p, C.c_double))
    return p


def scores(z, beta=0.0, resident=None, delta=None, tok2req=None):
    z = np.ascontiguousarray(z, dtype=np.float64)
    T, E = z.shape
    resident = None if resident is None else np.ascontiguousarray(resident, dtype=np.uint8)
    delta = None if delta is None else np.ascontiguousarray(delta, dtype=np.float32)
    tok2req = None if tok2req is None else np.ascontiguousarray(tok2req, dtype=np.int32)
    s = np.empty_like(z)
    lib().oracle_scores(_p(z, C.c_double), C.c_int(T), C.c_int(E), C.c_double(beta),
                        _p(resident, C.c_uint8), _p(delta, C.c_float), _p(tok2req, C.c_int32),
                        _p(s, C.c_double))
    return s


def topk(s, k):
    s = np.ascontiguousarray(s, dtype=np.float64)
    T, E = s.shape
    ids = np.empty((T, k), dtype=np.int32)
    gap = np.empty(T, dtype=np.float64)
    lib().oracle_topk(_p(s, C.c_double), C.c_int(T), C.c_int(E), C.c_int(k),
                      _p(ids, C.c_int32), _p(gap, C.c_double))
    return ids, gap


def weights(p, ids, renorm, routed_scale=1.0):
    p = np.ascontiguousarray(p, dtype=np.float64)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, E = p.shape
    k = ids.shape[1]
    w = np.empty((T, k), dtype=np.float64)
    lib().oracle_weights(_p(p, C.c_double), _p(ids, C.c_int32), C.c_int(T), C.c_int(E), C.c_int(k),
                         C.c_int(int(bool(renorm))), C.c_double(routed_scale), _p(w, C.c_double))
    return w


def histogram(ids, E):
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    hist = np.empty(E, dtype=np.int32)
    lib().oracle_histogram(_p(ids, C.c_int32), C.c_int(ids.size), C.c_int(E), _p(hist, C.c_int32))
    return hist


def permute(ids, E):
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, k = ids.shape
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    perm = np.empty(T * k, dtype=np.int32)
    inv = np.empty(T * k, dtype=np.int32)
    lib().oracle_permute(_p(ids, C.c_int32), C.c_int(T), C.c_int(k), C.c_int(E),
                         _p(counts, C.c_int32), _p(offsets, C.c_int32), _p(perm, C.c_int32),
                         _p(inv, C.c_int32))
    return counts, offsets, perm, inv


def _ptr_array(ws, E):
    arr = (C.c_void_p * E)()
    keep = []
    for e in range(E):
        w = ws[e] if ws is not None and e < len(ws) else None
        if w is None:
            arr[e] = None
        else:
            w = _u16(w)
            keep.append(w)
            arr[e] = w.ctypes.data
    return arr, keep


def expert_ffn(h, experts, ids, perm, pos_begin=0, pos_end=None, round_act=False):
    """experts: sequence over expert id of (W1 [F,d], W3 [F,d], W2 [d,F]) or None.

    Returns y [(pos_end-pos_begin), d] float64 for grouped positions pos_begin..pos_end.
    round_act is a diagnostic mode of the intermediate activation: 0 / False = kept in fp64 (the
    definition), 1 / True = rounded to bf16, 2 = rounded to fp16.
    """
    h = _u16(h)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    T, d = h.shape
    k = ids.shape[1]
    E = len(experts)
    pos_end = perm.size if pos_end is None else pos_end
    F = next(w[0].shape[0] for w in experts if w is not None)
    for pos in range(pos_begin, pos_end):
        assert experts[int(ids.reshape(-1)[perm[pos]])] is not None, "missing expert weights"
    a1, k1 = _ptr_array([None if w is None else w[0] for w in experts], E)
    a3, k3 = _ptr_array([None if w is None else w[1] for w in experts], E)
    a2, k2 = _ptr_array([None if w is None else w[2] for w in experts], E)
    y = np.empty((pos_end - pos_begin, d), dtype=np.float64)
    lib().oracle_expert_ffn(_p(h, C.c_uint16), C.c_int(d), C.c_int(F), C.c_int(k), a1, a3, a2,
                            _p(ids, C.c_int32), _p(perm, C.c_int32), C.c_int(pos_begin),
                            C.c_int(pos_end), C.c_int(int(round_act)), _p(y, C.c_double))
    return y


def _ptr_array_any(ws, E, dtype):
    arr = (C.c_void_p * E)()
    keep = []
    for e in range(E):
        w = ws[e] if e < len(ws) else None
        if w is None:
            arr[e] = None
        else:
            w = np.ascontiguousarray(w)
            assert w.dtype == dtype, w.dtype
            keep.append(w)
            arr[e] = w.ctypes.data
    return arr, keep


def expert_ffn_q4(h, experts, ids, perm, pos_begin=0, pos_end=None, round_act=False):
    """As expert_ffn with 4-bit weights: experts[e] = (q1, s1, q3, s3, q2, s2) or None; q* uint8 codes
    0..15 ([F,d], [F,d], [d,F]), s* bf16 scales per row and 128 inputs; w = (q - 8) * s."""
    h = _u16(h)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    T, d = h.shape
    k = ids.shape[1]
    E = len(experts)
    pos_end = perm.size if pos_end is None else pos_end
    F = next(w[0].shape[0] for w in experts if w is not None)
    assert d % 128 == 0 and F % 128 == 0
    for pos in range(pos_begin, pos_end):
        assert experts[int(ids.reshape(-1)[perm[pos]])] is not None, "missing expert weights"
    arrs, keeps = [], []
    for j, dt in enumerate([np.uint8, np.uint16, np.uint8, np.uint16, np.uint8, np.uint16]):
        a, kp = _ptr_array_any([None if w is None else w[j] for w in experts], E, dt)
        arrs.append(a)
        keeps.append(kp)
    y = np.empty((pos_end - pos_begin, d), dtype=np.float64)
    lib().oracle_expert_ffn_q4(_p(h, C.c_uint16), C.c_int(d), C.c_int(F), C.c_int(k), *arrs,
                               _p(ids, C.c_int32), _p(perm, C.c_int32), C.c_int(pos_begin),
                               C.c_int(pos_end), C.c_int(int(round_act)), _p(y, C.c_double))
    return y


def dense_ffn(h, W1, W3, W2, round_act=False):
    h, W1, W3, W2 = _u16(h), _u16(W1), _u16(W3), _u16(W2)
    T, d = h.shape
    F = W1.shape[0]
    assert W1.shape == (F, d) and W3.shape == (F, d) and W2.shape == (d, F)
    out = np.empty((T, d), dtype=np.float64)
    lib().oracle_dense_ffn(_p(h, C.c_uint16), C.c_int(T), C.c_int(d), C.c_int(F), _p(W1, C.c_uint16),
                           _p(W3, C.c_uint16), _p(W2, C.c_uint16), C.c_int(int(round_act)),
                           _p(out, C.c_double))
    return out


def combine(y, w, inv_perm, shared=None):
    y = np.ascontiguousarray(y, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    inv_perm = np.ascontiguousarray(inv_perm, dtype=np.int32)
    T, k = w.shape
    d = y.shape[1]
    shared = None if shared is None else np.ascontiguousarray(shared, dtype=np.float64)
    out = np.empty((T, d), dtype=np.float64)
    lib().oracle_combine(_p(y, C.c_double), _p(w, C.c_double), _p(inv_perm, C.c_int32), C.c_int(T),
                         C.c_int(k), C.c_int(d), _p(shared, C.c_double), _p(out, C.c_double))
    return out


def expected_activations(hist, tau, resident=None):
    """Returns (N_e, N_miss, descending order of experts)."""
    hist = np.ascontiguousarray(hist, dtype=np.int32)
    E = hist.size
    resident = None if resident is None else np.ascontiguousarray(resident, dtype=np.uint8)
    miss = C.c_int(0)
    order = np.empty(E, dtype=np.int32)
    n = lib().oracle_expected_activations(_p(hist, C.c_int32), C.c_int(E), C.c_double(tau),
                                          _p(resident, C.c_uint8), C.byref(miss), _p(order, C.c_int32))
    return int(n), int(miss.value), order


def step_size_raw(n_e, expert_bytes, bandwidth_Bps, layer_seconds):
    return float(lib().oracle_step_size_raw(n_e, expert_bytes, bandwidth_Bps, layer_seconds))


def horizon(n_e, expert_bytes, bandwidth_Bps, layer_seconds, h_max):
    return int(lib().oracle_horizon(n_e, expert_bytes, bandwidth_Bps, layer_seconds, h_max))


def token_dist(h, js=None):
    """Per-token part of the intra-batch diversity (paper Sec. 2.2): s[j] = sum_{i<j} ||v_i - v_j||_2
    for the listed tokens js (default: all, then s.sum() is Dist(t))."""
    h = _u16(h)
    T, d = h.shape
    js_a = None if js is None else np.ascontiguousarray(js, dtype=np.int32)
    n = T if js_a is None else len(js_a)
    s = np.empty(n, dtype=np.float64)
    lib().oracle_token_dist(_p(h, C.c_uint16), C.c_int(T), C.c_int(d), _p(js_a, C.c_int32), C.c_int(n),
                            _p(s, C.c_double))
    return s


# ---------------------------------------------------------------------------
# composites, in the method's order
# ---------------------------------------------------------------------------

def route(h, Wg, b, k, beta=0.0, resident=None, delta=None, tok2req=None, renorm=True,
          routed_scale=1.0):
    """One layer's cache-aware routing.  Returns a dict of every intermediate."""
    E = Wg.shape[0]
    z = gate_logits(h, Wg, b)
    p = softmax(z)
    s = scores(z, beta, resident, delta, tok2req)
    ids, gap = topk(s, k)
    w = weights(p, ids, renorm, routed_scale)
    counts, offsets, perm, inv = permute(ids, E)
    return dict(z=z, p=p, s=s, ids=ids, gap=gap, w=w, hist=histogram(ids, E), counts=counts,
                offsets=offsets, perm=perm, inv_perm=inv)


def route_from_ids(p, ids, E, renorm=True, routed_scale=1.0):
    """Teacher forcing: weights/histogram/permutation that follow from given ids."""
    w = weights(p, ids, renorm, routed_scale)
    counts, offsets, perm, inv = permute(ids, E)
    return dict(ids=ids, w=w, hist=histogram(ids, E), counts=counts, offsets=offsets, perm=perm,
                inv_perm=inv)


def predict(h, gates, biases, k, beta=0.0, residents=None, delta=None, tok2req=None, return_scores=False):
    """Cross-layer prediction: the same h through the next H layers' gates.

    gates: list of H [E,d] arrays; biases: list of H [E] arrays (or None);
    residents: list of H [E] flags (or None); delta: [R,H,E] or None.
    Returns ids [H,T,k], hist [H,E], gap [H,T] (and the selection scores [H,T,E] on request).
    """
    H = len(gates)
    T = h.shape[0]
    E = gates[0].shape[0]
    ids = np.empty((H, T, k), dtype=np.int32)
    hist = np.empty((H, E), dtype=np.int32)
    gap = np.empty((H, T), dtype=np.float64)
    sc = np.empty((H, T, E), dtype=np.float64)
    for j in range(H):
        z = gate_logits(h, gates[j], None if biases is None else biases[j])
        dj = None if delta is None else np.ascontiguousarray(delta[:, j, :])
        s = scores(z, beta, None if residents is None else residents[j], dj, tok2req)
        ids[j], gap[j] = topk(s, k)
        hist[j] = histogram(ids[j], E)
        sc[j] = s
    if return_scores:
        return ids, hist, gap, sc
    return ids, hist, gap


def moe_layer(h, Wg, b, experts, k, beta=0.0, resident=None, renorm=True, routed_scale=1.0,
              shared=None, round_act=False, forced_ids=None):
    """Whole layer: route -> grouped expert FFN -> weighted un-permute (+ shared experts)."""
    r = route(h, Wg, b, k, beta, resident, None, None, renorm, routed_scale)
    if forced_ids is not None:
        r.update(route_from_ids(r["p"], forced_ids, Wg.shape[0], renorm, routed_scale))
    y = expert_ffn(h, experts, r["ids"], r["perm"], round_act=round_act)
    sh = None if shared is None else dense_ffn(h, *shared, round_act=round_act)
    r["y"] = y
    r["out"] = combine(y, r["w"], r["inv_perm"], sh)
    return r
