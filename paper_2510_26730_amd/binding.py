"""ctypes binding of ``libexpertflow.so``: the same entry points as ``include/expertflow.h``.

Argument marshalling only.  Device buffers are passed as torch tensors (their
``data_ptr()``) or raw integer addresses, host buffers as numpy arrays.  Every
step of the hot path runs inside the library's kernels; nothing here computes.
The library must have been built (``python -m paper_2510_26730_amd.build``);
a missing library is an error, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libexpertflow.so")

EF_OK, EF_EINVAL, EF_ENOMEM, EF_EHIP, EF_EBUSY, EF_ENOTRESIDENT, EF_ENOSYS = 0, -1, -2, -3, -4, -5, -6
EF_FLAG_FAKE_COPY = 1
EF_FLAG_STRICT_RESIDENT = 2
EF_FLAG_PROFILE = 4
EF_FLAG_FIXED_ESTIMATES = 8
EF_FLAG_PROFILE_FFN_UP = 16
EF_KERNELS = ["predict", "route", "group", "ffn_up_tiled", "pack", "ffn_up", "ffn_down", "combine", "ffn_down_tiled",
              "dist"]
EF_MAX_EXPERTS, EF_MAX_TOPK, EF_MAX_HORIZON = 64, 8, 7

EXPORTS = [
    "ef_strerror", "ef_expert_bytes", "ef_pack_expert", "ef_expert_bytes_q4", "ef_pack_expert_q4", "ef_create", "ef_destroy", "ef_last_error",
    "ef_register_layer", "ef_predict", "ef_route", "ef_route_predict", "ef_moe_ffn", "ef_layer_step", "ef_cache_swap_in", "ef_cache_query",
    "ef_choose_horizon", "ef_token_dist", "ef_get_stats", "ef_reset_stats", "ef_set_profile", "ef_set_profile_sampling",
    "ef_fake_advance_time", "ef_layer_step_fetch", "ef_get_tuning", "ef_set_tuning", "ef_route_static", "ef_measure_peak",
    "ef_forest_create", "ef_forest_destroy", "ef_delta_features", "ef_forest_fit", "ef_forest_predict",
    "ef_forest_tree_size", "ef_forest_tree_export", "ef_forest_bit_accuracy", "ef_delta_from_activation",
    "ef_delta_cache_create", "ef_delta_cache_destroy", "ef_delta_cache_put", "ef_delta_cache_get",
    "ef_delta_cache_counts", "ef_delta_producer_create", "ef_delta_producer_destroy", "ef_delta_submit",
    "ef_delta_drain", "ef_delta_assemble",
]


class ef_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_experts", C.c_int32), ("top_k", C.c_int32),
        ("d_ff", C.c_int32), ("d_ff_shared", C.c_int32), ("slots_total", C.c_int32),
        ("slots_per_layer_max", C.c_int32), ("max_tokens", C.c_int32), ("h_max", C.c_int32),
        ("renorm_topk", C.c_int32), ("routed_scale", C.c_float), ("cum_threshold", C.c_float),
        ("stall_thresh", C.c_int32), ("overfetch_thresh", C.c_int32), ("flags", C.c_uint32),
        ("init_bandwidth_gbps", C.c_float), ("init_layer_us", C.c_float), ("weight_bits", C.c_int32),
    ]


class ef_stats(C.Structure):
    _fields_ = [
        ("hits", C.c_int64), ("misses", C.c_int64), ("prefetch_issued", C.c_int64),
        ("prefetch_redundant", C.c_int64), ("evictions", C.c_int64), ("bytes_copied", C.c_int64), ("bytes_timed", C.c_int64),
        ("layers_run", C.c_int64), ("tokens_run", C.c_int64), ("copy_seconds", C.c_double),
        ("stall_seconds", C.c_double), ("layer_seconds", C.c_double), ("bandwidth_Bps", C.c_double),
        ("layer_seconds_est", C.c_double), ("miss_rate", C.c_double), ("horizon", C.c_int32),
        ("stall_counter", C.c_int32), ("overfetch_counter", C.c_int32), ("reserved_", C.c_int32),
        ("prefetch_used", C.c_int64), ("prefetch_wasted", C.c_int64), ("miss_copies", C.c_int64),
        ("miss_copy_bytes", C.c_int64), ("miss_copy_seconds", C.c_double),
        ("pred_overlap_hits", C.c_int64 * 7), ("pred_overlap_total", C.c_int64 * 7),
        ("kernel_seconds", C.c_double * 10), ("kernel_bytes", C.c_double * 10),
        ("kernel_launches", C.c_int64 * 10), ("kernel_flops", C.c_double * 10),
    ]

    def as_dict(self):
        out = {}
        for n, _ in self._fields_:
            v = getattr(self, n)
            out[n] = list(v) if hasattr(v, "__len__") else v
        return out


class ef_tuning(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "tiled", "tiled_min_tiles", "tiled_min_up_wgs", "tiled_min_down_wgs", "tiled_xcd_rotation", "overlap_tiled",
        "sort_groups", "passes_of_four", "lds_shared", "lds_shared_occupancy", "up_want_waves", "up_k_slices",
        "down_want_wgs", "down_k_slices", "down_slices_by_longest_k", "down_split_slice_counts", "gate_k_split",
        "gate_token_split", "gate_fused_finish", "gate_stream", "early_pack", "copy_chunk_mib", "copy_depth",
        "down_tail_split", "tiled_tail_slices", "dist_form")]


class ef_forest_config(C.Structure):
    _fields_ = [("n_features", C.c_int32), ("n_outputs", C.c_int32), ("n_trees", C.c_int32),
                ("max_depth", C.c_int32), ("min_samples_leaf", C.c_int32), ("n_threads", C.c_int32)]


class EfError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"expertflow error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """Load the built library; fails loudly if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run python -m paper_2510_26730_amd.build")
        L = C.CDLL(LIB_PATH)
        vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
        L.ef_strerror.restype = C.c_char_p
        L.ef_strerror.argtypes = [i32]
        L.ef_expert_bytes.restype = C.c_size_t
        L.ef_expert_bytes.argtypes = [i32, i32]
        L.ef_pack_expert.argtypes = [vp, vp, vp, i32, i32, vp]
        L.ef_expert_bytes_q4.restype = C.c_size_t
        L.ef_expert_bytes_q4.argtypes = [i32, i32]
        L.ef_pack_expert_q4.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp]
        L.ef_create.argtypes = [C.POINTER(ef_config), C.POINTER(vp)]
        L.ef_destroy.argtypes = [vp]
        L.ef_last_error.restype = C.c_char_p
        L.ef_last_error.argtypes = [vp]
        L.ef_register_layer.argtypes = [vp, i32, vp, vp, vp, vp]
        L.ef_predict.argtypes = [vp, i32, vp, i32, i32, vp, vp, f32, vp, vp, C.POINTER(i32), vp]
        L.ef_route.argtypes = [vp, i32, vp, i32, f32, vp, vp, vp, vp, vp, vp, vp]
        L.ef_route_static.argtypes = [vp, i32, vp, i32, f32, vp, vp, vp, vp, vp, vp, vp]
        L.ef_route_predict.argtypes = [vp, i32, vp, i32, f32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                       C.POINTER(i32), vp]
        L.ef_moe_ffn.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.ef_layer_step.argtypes = [vp, i32, vp, i32, f32, i32, vp, vp, vp, C.POINTER(i32), vp, vp]
        L.ef_cache_swap_in.argtypes = [vp, i32, i32, i32, i32, C.POINTER(i32)]
        L.ef_cache_query.argtypes = [vp, i32, vp]
        L.ef_choose_horizon.argtypes = [vp, i32, vp, i32, i32, C.POINTER(i32), vp, C.POINTER(i32)]
        L.ef_token_dist.argtypes = [vp, vp, i32, vp, vp, vp]
        L.ef_measure_peak.argtypes = [vp, i32, vp, C.c_size_t, i32, C.POINTER(C.c_double), vp]
        L.ef_get_stats.argtypes = [vp, C.POINTER(ef_stats)]
        L.ef_reset_stats.argtypes = [vp]
        L.ef_set_profile.argtypes = [vp, C.c_uint]
        L.ef_set_profile_sampling.argtypes = [vp, i32]
        L.ef_fake_advance_time.argtypes = [vp, C.c_double]
        L.ef_layer_step_fetch.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.POINTER(i32), C.POINTER(i32), vp]
        L.ef_get_tuning.argtypes = [vp, C.POINTER(ef_tuning)]
        L.ef_set_tuning.argtypes = [vp, C.POINTER(ef_tuning)]
        ll = C.c_longlong
        L.ef_forest_create.argtypes = [C.POINTER(ef_forest_config), C.POINTER(vp)]
        L.ef_forest_destroy.argtypes = [vp]
        L.ef_delta_features.argtypes = [vp, i32, i32, vp, i32, i32, i32, vp, i32, i32, vp]
        L.ef_forest_fit.argtypes = [vp, vp, vp, i32, vp]
        L.ef_forest_predict.argtypes = [vp, vp, i32, vp]
        L.ef_forest_tree_size.argtypes = [vp, i32]
        L.ef_forest_tree_export.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.ef_forest_bit_accuracy.argtypes = [vp, vp, i32, i32, C.POINTER(C.c_double)]
        L.ef_delta_from_activation.argtypes = [vp, i32, i32, f32, vp]
        L.ef_delta_cache_create.argtypes = [i32, i32, C.POINTER(vp)]
        L.ef_delta_cache_destroy.argtypes = [vp]
        L.ef_delta_cache_put.argtypes = [vp, vp, i32, i32, i32, vp]
        L.ef_delta_cache_get.argtypes = [vp, vp, i32, i32, i32, vp]
        L.ef_delta_cache_counts.argtypes = [vp, C.POINTER(ll), C.POINTER(ll), C.POINTER(ll)]
        L.ef_delta_producer_create.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, C.POINTER(vp)]
        L.ef_delta_producer_destroy.argtypes = [vp]
        L.ef_delta_submit.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.ef_delta_drain.argtypes = [vp]
        L.ef_delta_assemble.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, C.POINTER(i32)]
        _lib = L
    return _lib


def _ptr(x):
    """Address of a torch tensor / numpy array / raw int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        assert x.flags["C_CONTIGUOUS"]
        return x.ctypes.data
    assert x.is_contiguous()
    return x.data_ptr()


def _check(ctx, rc):
    if rc != 0:
        text = lib().ef_last_error(ctx)
        raise EfError(rc, (text or b"").decode())
    return rc


def _stream(stream):
    if stream is None:
        return None
    return stream if isinstance(stream, int) else stream.cuda_stream


# ---- utilities ------------------------------------------------------------------------------

def ef_strerror(code):
    return lib().ef_strerror(code).decode()


def ef_expert_bytes(d_model, d_ff):
    return int(lib().ef_expert_bytes(d_model, d_ff))


def ef_pack_expert(W1, W3, W2, blob=None):
    """W1, W3 [F,d], W2 [d,F] uint16 numpy arrays -> packed blob (numpy uint8, or written into `blob`)."""
    F, d = W1.shape
    assert W3.shape == (F, d) and W2.shape == (d, F)
    n = ef_expert_bytes(d, F)
    if n == 0:
        raise EfError(EF_EINVAL, "d_model must be a multiple of 64 and d_ff of 32")
    out = np.empty(n, dtype=np.uint8) if blob is None else blob
    W1, W3, W2 = (np.ascontiguousarray(w, dtype=np.uint16) for w in (W1, W3, W2))
    _check(None, lib().ef_pack_expert(_ptr(W1), _ptr(W3), _ptr(W2), d, F, _ptr(out)))
    return out


def ef_expert_bytes_q4(d, F):
    return int(lib().ef_expert_bytes_q4(d, F))


def ef_pack_expert_q4(q1, s1, q3, s3, q2, s2, blob=None):
    """Codes q1, q3 [F,d], q2 [d,F] uint8 (0..15) and bf16 scales s1, s3 [F,d/128], s2 [d,F/128] (uint16)
    -> packed 4-bit blob (numpy uint8, or written into `blob`)."""
    F, d = q1.shape
    assert q3.shape == (F, d) and q2.shape == (d, F)
    assert s1.shape == (F, d // 128) and s3.shape == (F, d // 128) and s2.shape == (d, F // 128)
    n = ef_expert_bytes_q4(d, F)
    if n == 0:
        raise EfError(EF_EINVAL, "d_model and d_ff must be multiples of 128")
    out = np.empty(n, dtype=np.uint8) if blob is None else blob
    q1, q3, q2 = (np.ascontiguousarray(q, dtype=np.uint8) for q in (q1, q3, q2))
    s1, s3, s2 = (np.ascontiguousarray(x, dtype=np.uint16) for x in (s1, s3, s2))
    _check(None, lib().ef_pack_expert_q4(_ptr(q1), _ptr(s1), _ptr(q3), _ptr(s3), _ptr(q2), _ptr(s2), d, F,
                                         _ptr(out)))
    return out


# ---- context ----------------------------------------------------------------------------------

def ef_create(**kw):
    """Keyword arguments are the fields of ef_config; returns the opaque context handle."""
    cfg = ef_config()
    defaults = dict(d_ff_shared=0, slots_per_layer_max=0, h_max=4, renorm_topk=1, routed_scale=1.0,
                    cum_threshold=0.9, stall_thresh=4, overfetch_thresh=4, flags=0,
                    init_bandwidth_gbps=50.0, init_layer_us=200.0, weight_bits=0)
    defaults.update(kw)
    for k, v in defaults.items():
        setattr(cfg, k, v)
    h = C.c_void_p()
    _check(None, lib().ef_create(C.byref(cfg), C.byref(h)))
    return h


def ef_destroy(ctx):
    return lib().ef_destroy(ctx)


def ef_last_error(ctx):
    return (lib().ef_last_error(ctx) or b"").decode()


def ef_register_layer(ctx, layer, gate_w, gate_b, experts, shared_blob=None):
    return _check(ctx, lib().ef_register_layer(ctx, layer, _ptr(gate_w), _ptr(gate_b), _ptr(experts),
                                               _ptr(shared_blob)))


# ---- hot path ---------------------------------------------------------------------------------

def ef_predict(ctx, layer, hidden, T, H, delta, tok2req, beta, topk_ids, hist, stream=None):
    """Returns the effective H (clamped at the last layer)."""
    he = C.c_int(0)
    _check(ctx, lib().ef_predict(ctx, layer, _ptr(hidden), T, H, _ptr(delta), _ptr(tok2req), beta,
                                 _ptr(topk_ids), _ptr(hist), C.byref(he), _stream(stream)))
    return he.value


def ef_route(ctx, layer, hidden, T, beta, topk_ids, topk_w, counts, offsets, perm, inv_perm, stream=None):
    return _check(ctx, lib().ef_route(ctx, layer, _ptr(hidden), T, beta, _ptr(topk_ids), _ptr(topk_w),
                                      _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv_perm),
                                      _stream(stream)))


def ef_route_static(ctx, layer, hidden, T, beta, topk_ids, topk_w, counts, offsets, perm, inv_perm, stream=None):
    return _check(ctx, lib().ef_route_static(ctx, layer, _ptr(hidden), T, beta, _ptr(topk_ids), _ptr(topk_w),
                                             _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv_perm),
                                             _stream(stream)))


def ef_route_predict(ctx, layer, hidden, T, beta, H, delta, tok2req, topk_ids, topk_w, counts, offsets, perm,
                     inv_perm, pred_ids, pred_hist, stream=None):
    """Returns the effective H."""
    he = C.c_int(0)
    _check(ctx, lib().ef_route_predict(ctx, layer, _ptr(hidden), T, beta, H, _ptr(delta), _ptr(tok2req),
                                       _ptr(topk_ids), _ptr(topk_w), _ptr(counts), _ptr(offsets), _ptr(perm),
                                       _ptr(inv_perm), _ptr(pred_ids), _ptr(pred_hist), C.byref(he),
                                       _stream(stream)))
    return he.value


def ef_moe_ffn(ctx, layer, hidden, T, topk_ids, topk_w, counts_host, offsets, perm, inv_perm, out,
               stream=None):
    counts_host = np.ascontiguousarray(counts_host, dtype=np.int32)
    return _check(ctx, lib().ef_moe_ffn(ctx, layer, _ptr(hidden), T, _ptr(topk_ids), _ptr(topk_w),
                                        _ptr(counts_host), _ptr(offsets), _ptr(perm), _ptr(inv_perm),
                                        _ptr(out), _stream(stream)))


def ef_layer_step(ctx, layer, hidden, T, beta, H, delta, tok2req, out, counts_host=None, stream=None):
    """Whole layer in one call; returns the horizon chosen for the next layer."""
    hn = C.c_int(0)
    _check(ctx, lib().ef_layer_step(ctx, layer, _ptr(hidden), T, beta, H, _ptr(delta), _ptr(tok2req), _ptr(out),
                                    C.byref(hn), _ptr(counts_host), _stream(stream)))
    return hn.value


def ef_layer_step_fetch(ctx, T, k, E, H_max=EF_MAX_HORIZON, stream=None):
    """Routing state the last ef_layer_step left in the library's buffers, as numpy arrays:
    dict(ids [T,k], w [T,k], offsets [E+1], perm, inv_perm [T*k], pred_ids [H_eff,T,k], pred_hist [H_eff,E])."""
    n = T * k
    o = dict(ids=np.empty(n, np.int32), w=np.empty(n, np.float32), offsets=np.empty(E + 1, np.int32),
             perm=np.empty(n, np.int32), inv_perm=np.empty(n, np.int32),
             pred_ids=np.empty(H_max * n, np.int32), pred_hist=np.empty(H_max * E, np.int32))
    t_out, he = C.c_int(0), C.c_int(0)
    _check(ctx, lib().ef_layer_step_fetch(ctx, _ptr(o["ids"]), _ptr(o["w"]), _ptr(o["offsets"]), _ptr(o["perm"]),
                                          _ptr(o["inv_perm"]), _ptr(o["pred_ids"]), _ptr(o["pred_hist"]),
                                          C.byref(t_out), C.byref(he), _stream(stream)))
    assert t_out.value == T, (t_out.value, T)
    H = he.value
    o["ids"], o["w"] = o["ids"].reshape(T, k), o["w"].reshape(T, k)
    o["pred_ids"] = o["pred_ids"][:H * n].reshape(H, T, k)
    o["pred_hist"] = o["pred_hist"][:H * E].reshape(H, E)
    return o


def ef_get_tuning(ctx):
    t = ef_tuning()
    _check(ctx, lib().ef_get_tuning(ctx, C.byref(t)))
    return {n: getattr(t, n) for n, _ in t._fields_}


def ef_set_tuning(ctx, **kw):
    """Change the named fields of the context's launch tuning (the others keep their values)."""
    t = ef_tuning()
    _check(ctx, lib().ef_get_tuning(ctx, C.byref(t)))
    for name, v in kw.items():
        if name not in dict(t._fields_):
            raise KeyError(name)
        setattr(t, name, int(v))
    return _check(ctx, lib().ef_set_tuning(ctx, C.byref(t)))


def ef_token_dist(ctx, hidden, T, tok_dist, dist, stream=None):
    """Dist(t) of the batch: tok_dist [T] f32 (or None) and dist [1] f64, both on the device."""
    return _check(ctx, lib().ef_token_dist(ctx, _ptr(hidden), T, _ptr(tok_dist), _ptr(dist), _stream(stream)))


EF_PEAK_HBM_READ, EF_PEAK_MFMA_16BIT = 0, 1


def ef_measure_peak(ctx, what, buf=None, nbytes=0, reps=4, stream=None):
    """Measured ceiling of the device: GB/s of a plain streaming read of `buf` (EF_PEAK_HBM_READ) or TFLOP/s of a
    register-resident matrix-core loop (EF_PEAK_MFMA_16BIT)."""
    out = C.c_double(0.0)
    _check(ctx, lib().ef_measure_peak(ctx, what, _ptr(buf), nbytes, reps, C.byref(out), _stream(stream)))
    return out.value


def ef_cache_swap_in(ctx, layer, expert, priority=0, due_in=0):
    """Returns the slot."""
    slot = C.c_int(-1)
    _check(ctx, lib().ef_cache_swap_in(ctx, layer, expert, priority, due_in, C.byref(slot)))
    return slot.value


def ef_cache_query(ctx, layer, n_experts):
    r = np.zeros(n_experts, dtype=np.uint8)
    _check(ctx, lib().ef_cache_query(ctx, layer, _ptr(r)))
    return r


def ef_choose_horizon(ctx, layer, hist_host, T):
    """hist_host [H,E] int32 numpy.  Returns (H_next, [(j, expert), ...])."""
    hist_host = np.ascontiguousarray(hist_host, dtype=np.int32)
    H, E = hist_host.shape if hist_host.ndim == 2 else (0, 0)
    lst = np.zeros(max(1, H * E), dtype=np.int32)
    hn, n = C.c_int(0), C.c_int(0)
    _check(ctx, lib().ef_choose_horizon(ctx, layer, _ptr(hist_host) if H else None, H, T, C.byref(hn),
                                        _ptr(lst), C.byref(n)))
    return hn.value, [(int(v) >> 16, int(v) & 0xFFFF) for v in lst[:n.value]]


def ef_get_stats(ctx):
    st = ef_stats()
    _check(ctx, lib().ef_get_stats(ctx, C.byref(st)))
    return st.as_dict()


def ef_reset_stats(ctx):
    return _check(ctx, lib().ef_reset_stats(ctx))


def ef_set_profile(ctx, kinds_mask):
    return _check(ctx, lib().ef_set_profile(ctx, kinds_mask))


def ef_set_profile_sampling(ctx, every):
    return _check(ctx, lib().ef_set_profile_sampling(ctx, every))


def ef_fake_advance_time(ctx, seconds):
    return _check(ctx, lib().ef_fake_advance_time(ctx, seconds))


# ---- deviation predictor (host side) ----------------------------------------------------------

def _rc(rc, what):
    if rc < 0:
        raise EfError(rc, what)
    return rc


def _np(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def ef_forest_create(n_features, n_outputs, n_trees, max_depth, min_samples_leaf=1, n_threads=0):
    cfg = ef_forest_config(n_features, n_outputs, n_trees, max_depth, min_samples_leaf, n_threads)
    out = C.c_void_p()
    _rc(lib().ef_forest_create(C.byref(cfg), C.byref(out)), "ef_forest_create")
    return out


def ef_forest_destroy(f):
    return lib().ef_forest_destroy(f)


def ef_delta_features(emb_table, token_ids, S, layer, prev_act, L, M):
    emb_table = _np(emb_table, np.float32)
    tok = _np(token_ids, np.int32)
    prev = _np(prev_act, np.uint8).reshape(-1)
    assert prev.size == L * M
    x = np.empty(emb_table.shape[1] + 2 + L * M, dtype=np.float32)
    _rc(lib().ef_delta_features(_ptr(emb_table), emb_table.shape[0], emb_table.shape[1], _ptr(tok), tok.size, S, layer,
                                _ptr(prev), L, M, _ptr(x)), "ef_delta_features")
    return x


def ef_forest_fit(f, X, Y, bootstrap=None):
    X, Y = _np(X, np.float32), _np(Y, np.uint8)
    assert X.shape[0] == Y.shape[0]
    b = None if bootstrap is None else _np(bootstrap, np.int32)
    assert b is None or b.shape[1] == X.shape[0]
    return _rc(lib().ef_forest_fit(f, _ptr(X), _ptr(Y), X.shape[0], _ptr(b)), "ef_forest_fit")


def ef_forest_predict(f, X, n_outputs):
    X = _np(X, np.float32)
    out = np.empty((X.shape[0], n_outputs), dtype=np.float64)
    _rc(lib().ef_forest_predict(f, _ptr(X), X.shape[0], _ptr(out)), "ef_forest_predict")
    return out


def ef_forest_tree_size(f, t):
    return _rc(lib().ef_forest_tree_size(f, t), "ef_forest_tree_size")


def ef_forest_tree_export(f, t, n_outputs):
    n = ef_forest_tree_size(f, t)
    tree = {"feature": np.empty(n, np.int32), "threshold": np.empty(n, np.float64), "left": np.empty(n, np.int32),
            "right": np.empty(n, np.int32), "count": np.empty(n, np.int32), "value": np.empty((n, n_outputs), np.float64)}
    _rc(lib().ef_forest_tree_export(f, t, *[_ptr(tree[k]) for k in ("feature", "threshold", "left", "right", "count",
                                                                     "value")]), "ef_forest_tree_export")
    return tree


def ef_forest_bit_accuracy(Y_hat, Y):
    Y_hat, Y = _np(Y_hat, np.float64), _np(Y, np.uint8)
    acc = C.c_double()
    _rc(lib().ef_forest_bit_accuracy(_ptr(Y_hat), _ptr(Y), Y.shape[0], Y.shape[1], C.byref(acc)), "ef_forest_bit_accuracy")
    return acc.value


def ef_delta_from_activation(Y_hat, gain):
    Y_hat = _np(Y_hat, np.float64)
    out = np.empty(Y_hat.shape, dtype=np.float32)
    M = Y_hat.shape[-1]
    _rc(lib().ef_delta_from_activation(_ptr(Y_hat), Y_hat.size // M, M, gain, _ptr(out)), "ef_delta_from_activation")
    return out


def ef_delta_cache_create(capacity, M):
    out = C.c_void_p()
    _rc(lib().ef_delta_cache_create(capacity, M, C.byref(out)), "ef_delta_cache_create")
    return out


def ef_delta_cache_destroy(c):
    return lib().ef_delta_cache_destroy(c)


def ef_delta_cache_put(c, token_ids, layer, S, y_hat):
    tok, y = _np(token_ids, np.int32), _np(y_hat, np.float64)
    return _rc(lib().ef_delta_cache_put(c, _ptr(tok), tok.size, layer, S, _ptr(y)), "ef_delta_cache_put")


def ef_delta_cache_get(c, token_ids, layer, S, M):
    """The cached prediction [M] or None."""
    tok = _np(token_ids, np.int32)
    y = np.empty(M, dtype=np.float64)
    hit = _rc(lib().ef_delta_cache_get(c, _ptr(tok), tok.size, layer, S, _ptr(y)), "ef_delta_cache_get")
    return y if hit else None


def ef_delta_cache_counts(c):
    h, m, e = C.c_longlong(), C.c_longlong(), C.c_longlong()
    _rc(lib().ef_delta_cache_counts(c, C.byref(h), C.byref(m), C.byref(e)), "ef_delta_cache_counts")
    return h.value, m.value, e.value


def ef_delta_producer_create(forest, cache, emb_table, L, M, n_threads=0):
    """emb_table must be a C-contiguous float32 array that the caller keeps alive."""
    assert emb_table.dtype == np.float32 and emb_table.flags["C_CONTIGUOUS"]
    out = C.c_void_p()
    _rc(lib().ef_delta_producer_create(forest, cache, _ptr(emb_table), emb_table.shape[0], emb_table.shape[1], L, M,
                                       n_threads, C.byref(out)), "ef_delta_producer_create")
    return out


def ef_delta_producer_destroy(p):
    return lib().ef_delta_producer_destroy(p)


def ef_delta_submit(p, token_ids, S, layer_first, n_layers, prev_act):
    tok, prev = _np(token_ids, np.int32), _np(prev_act, np.uint8).reshape(-1)
    return _rc(lib().ef_delta_submit(p, _ptr(tok), tok.size, S, layer_first, n_layers, _ptr(prev)), "ef_delta_submit")


def ef_delta_drain(p):
    return _rc(lib().ef_delta_drain(p), "ef_delta_drain")


def ef_delta_assemble(c, token_ids, tok_off, layer, S, H, L, gain, M, out=None):
    """(delta [R, H, M] float32, rows found).  `out` may be a caller-provided (e.g. pinned) array."""
    tok, off = _np(token_ids, np.int32), _np(tok_off, np.int32)
    R = off.size - 1
    delta = np.empty((R, H, M), dtype=np.float32) if out is None else out
    hits = C.c_int32()
    _rc(lib().ef_delta_assemble(c, _ptr(tok), _ptr(off), R, layer, S, H, L, gain, _ptr(delta), C.byref(hits)),
        "ef_delta_assemble")
    return delta, hits.value
