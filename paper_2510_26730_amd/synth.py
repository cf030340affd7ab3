"""Seeded synthetic inputs for the MoE-layer hot path.

This module only *draws inputs*: hidden states, gate matrices, gate biases,
expert weights, residency flags and request maps, in the shapes and
distributions of the five workload configurations.  It contains none of the
method's arithmetic (no gate product, softmax, top-k, permutation, FFN or
cache policy) and imports neither the CPU oracle nor the HIP library, so both
sides can be fed the very same arrays.

bf16 tensors are carried as ``numpy.uint16`` bit patterns (round to nearest
even from float32).  Every array is a pure function of ``(config id, stream id,
indices...)`` through ``numpy.random.SeedSequence``; large tensors are drawn in
fixed-size chunks with one child stream per chunk, so the result does not
depend on how many threads draw them.

Stream ids: 0 hidden, 1 gate W, 2 expert W, 3 inter-layer noise,
4 popularity permutation, 5 shared-expert W, 6 residency, 7 delta, 8 requests,
9 prompt pool, 10 feature embedding table, 11 bootstrap draws.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 26730
_CHUNK = 1 << 22

HIDDEN, GATE_W, EXPERT_W, NOISE, POPULARITY, SHARED_W, RESIDENCY, DELTA, REQUESTS, PROMPTS, FEATURE_EMB, BOOTSTRAP = range(12)


@dataclasses.dataclass(frozen=True)
class MoEShape:
    """One workload configuration (shapes only)."""
    name: str
    cfg_id: int
    n_layers: int
    d: int            # model dim
    E: int            # routed experts
    k: int            # top-k
    F: int            # expert FFN hidden
    F_shared: int     # hidden dim of the always-resident dense SwiGLU (0 = none)
    T: int            # default tokens per step
    slots_per_layer: int
    zipf_s: float
    renorm: bool      # renormalise combine weights over the top-k
    w_std: float = 0.02
    noise: float = 0.3

    @property
    def expert_bytes(self) -> int:
        return 3 * self.d * self.F * 2


CONFIGS = {
    "tiny": MoEShape("tiny", 1, 3, 512, 8, 2, 1024, 0, 64, 4, 1.1, True),
    "mixtral_decode": MoEShape("mixtral_decode", 2, 32, 4096, 8, 2, 14336, 0, 64, 2, 1.1, True),
    "mixtral_prefill": MoEShape("mixtral_prefill", 3, 32, 4096, 8, 2, 14336, 0, 8192, 4, 1.1, True),
    "deepseek_v2_lite": MoEShape("deepseek_v2_lite", 4, 26, 2048, 64, 6, 1408, 2816, 32, 16, 1.2, False),
    "qwen15_moe": MoEShape("qwen15_moe", 5, 24, 2048, 60, 4, 1408, 5632, 640, 12, 1.1, False),
}


def _seq(*key: int) -> np.random.SeedSequence:
    return np.random.SeedSequence([BASE_SEED, *[int(v) for v in key]])


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal_f32(n: int, key, scale: float = 1.0) -> np.ndarray:
    """n draws of N(0, scale^2) as float32; chunked, thread-count independent."""
    out = np.empty(n, dtype=np.float32)
    nchunk = (n + _CHUNK - 1) // _CHUNK
    children = _seq(*key).spawn(nchunk)

    def fill(c: int) -> None:
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        g = np.random.Generator(np.random.PCG64(children[c]))
        g.standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])
        if scale != 1.0:
            out[lo:hi] *= np.float32(scale)

    if nchunk == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, range(nchunk)))
    return out


def normal_bf16(shape, key, scale: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    x = normal_f32(n, key, scale)
    out = np.empty(n, dtype=np.uint16)
    nchunk = (n + _CHUNK - 1) // _CHUNK

    def conv(c: int) -> None:
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        out[lo:hi] = f32_to_bf16(x[lo:hi])

    if nchunk == 1:
        conv(0)
    else:
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(conv, range(nchunk)))
    return out.reshape(shape)


# ---------------------------------------------------------------------------
# per-configuration tensors
# ---------------------------------------------------------------------------

def hidden(cfg: MoEShape, step: int = 0, T: int | None = None) -> np.ndarray:
    """h_0 [T, d] bf16 ~ N(0, 1) for one step."""
    T = cfg.T if T is None else T
    return normal_bf16((T, cfg.d), (cfg.cfg_id, HIDDEN, step, T))


def next_hidden(cfg: MoEShape, h: np.ndarray, layer: int, step: int = 0) -> np.ndarray:
    """h_{l+1} = bf16(f32(h_l) + noise * N(0, 1)): the layer-to-layer correlation recipe."""
    T, d = h.shape
    n = normal_f32(T * d, (cfg.cfg_id, NOISE, step, layer, T), cfg.noise).reshape(T, d)
    return f32_to_bf16(bf16_to_f32(h) + n)


def hidden_stack(cfg: MoEShape, n_layers: int, step: int = 0, T: int | None = None) -> np.ndarray:
    """[n_layers, T, d] bf16: h_0 and its noisy successors."""
    hs = [hidden(cfg, step, T)]
    for l in range(1, n_layers):
        hs.append(next_hidden(cfg, hs[-1], l - 1, step))
    return np.stack(hs)


def gate_weight(cfg: MoEShape, layer: int) -> np.ndarray:
    """Wg [E, d] bf16 ~ N(0, w_std^2)."""
    return normal_bf16((cfg.E, cfg.d), (cfg.cfg_id, GATE_W, layer), cfg.w_std)


def popularity_ranks(cfg: MoEShape, layer: int, epoch: int = 0) -> np.ndarray:
    """Seeded permutation of 1..E: rank of each expert in the Zipf popularity order."""
    g = np.random.Generator(np.random.PCG64(_seq(cfg.cfg_id, POPULARITY, layer, epoch)))
    return (g.permutation(cfg.E) + 1).astype(np.int64)


def gate_bias(cfg: MoEShape, layer: int, epoch: int = 0) -> np.ndarray:
    """b[e] = -s * ln(rank_e): log of a Zipf(s) popularity (constant shift dropped)."""
    r = popularity_ranks(cfg, layer, epoch)
    return (-cfg.zipf_s * np.log(r.astype(np.float64))).astype(np.float32)


def expert_weights(cfg: MoEShape, layer: int, e: int):
    """(W1 [F,d], W3 [F,d], W2 [d,F]) bf16 ~ N(0, w_std^2), row-major."""
    w1 = normal_bf16((cfg.F, cfg.d), (cfg.cfg_id, EXPERT_W, layer, e, 1), cfg.w_std)
    w3 = normal_bf16((cfg.F, cfg.d), (cfg.cfg_id, EXPERT_W, layer, e, 3), cfg.w_std)
    w2 = normal_bf16((cfg.d, cfg.F), (cfg.cfg_id, EXPERT_W, layer, e, 2), cfg.w_std)
    return w1, w3, w2


def _draw_q4(cfg: MoEShape, F: int, key: tuple):
    out = []
    for which, (rows, cols) in ((1, (F, cfg.d)), (3, (F, cfg.d)), (2, (cfg.d, F))):
        n = rows * cols
        z = normal_f32(n, key + (which, 4)).reshape(rows, cols)
        q = np.clip(np.rint(z * 2.5) + 8.0, 0.0, 15.0).astype(np.uint8)
        u = normal_f32(rows * (cols // 128), key + (which, 5))
        sc = (cfg.w_std / 2.5) * (1.0 + 0.1 * np.clip(u, -3.0, 3.0))
        out += [q, f32_to_bf16(sc.reshape(rows, cols // 128))]
    return tuple(out)


def expert_weights_q4(cfg: MoEShape, layer: int, e: int):
    """4-bit form of an expert: (q1, s1, q3, s3, q2, s2); codes uint8 in 0..15 drawn as a clipped, rounded
    normal around 8, one bf16 scale per row and 128 inputs, so that (q - 8) * s ~ N(0, w_std^2) like the
    bf16 experts.  Codes and scales are drawn directly (no quantiser): they are inputs."""
    return _draw_q4(cfg, cfg.F, (cfg.cfg_id, EXPERT_W, layer, e))


def shared_weights_q4(cfg: MoEShape, layer: int):
    """4-bit form of the always-resident dense SwiGLU of hidden F_shared, drawn like a 4-bit expert."""
    if cfg.F_shared == 0:
        return None
    return _draw_q4(cfg, cfg.F_shared, (cfg.cfg_id, SHARED_W, layer))


def dequant_q4(q: np.ndarray, s: np.ndarray) -> np.ndarray:
    """(q - 8) * s as float64 [rows, cols] (what a 4-bit matrix stands for)."""
    return (q.astype(np.float64) - 8.0) * np.repeat(bf16_to_f32(s).astype(np.float64), 128, axis=1)


def shared_weights(cfg: MoEShape, layer: int):
    """Always-resident dense SwiGLU (shared experts fused into one of hidden F_shared)."""
    if cfg.F_shared == 0:
        return None
    Fs = cfg.F_shared
    w1 = normal_bf16((Fs, cfg.d), (cfg.cfg_id, SHARED_W, layer, 1), cfg.w_std)
    w3 = normal_bf16((Fs, cfg.d), (cfg.cfg_id, SHARED_W, layer, 3), cfg.w_std)
    w2 = normal_bf16((cfg.d, Fs), (cfg.cfg_id, SHARED_W, layer, 2), cfg.w_std)
    return w1, w3, w2


def residency(cfg: MoEShape, layer: int, n_resident: int | None = None, most_popular: bool = True) -> np.ndarray:
    """[E] uint8 flags with n_resident ones: the most popular experts, or a seeded random subset."""
    n = cfg.slots_per_layer if n_resident is None else n_resident
    r = np.zeros(cfg.E, dtype=np.uint8)
    if most_popular:
        r[np.argsort(popularity_ranks(cfg, layer), kind="stable")[:n]] = 1
    else:
        g = np.random.Generator(np.random.PCG64(_seq(cfg.cfg_id, RESIDENCY, layer)))
        r[g.permutation(cfg.E)[:n]] = 1
    return r


def delta(cfg: MoEShape, layer: int, R: int, H: int, scale: float = 0.5) -> np.ndarray:
    """Stand-in for the learned deviation: [R, H, E] float32 ~ N(0, scale^2)."""
    return normal_f32(R * H * cfg.E, (cfg.cfg_id, DELTA, layer, R, H), scale).reshape(R, H, cfg.E)


def tok2req(cfg: MoEShape, T: int, R: int) -> np.ndarray:
    """[T] int32: request of each token; contiguous runs of seeded random lengths."""
    g = np.random.Generator(np.random.PCG64(_seq(cfg.cfg_id, REQUESTS, T, R)))
    cuts = np.sort(g.integers(0, T + 1, size=R - 1)) if R > 1 else np.empty(0, dtype=np.int64)
    out = np.zeros(T, dtype=np.int32)
    for c in cuts:
        out[c:] += 1
    return out


# ---------------------------------------------------------------------------
# recurring prompts (stand-in for real prompts through a real, deterministic model): inputs of the
# deviation predictor's logs.  A prompt is a short token id sequence; its hidden states in every layer
# are a fixed function of the prompt, so a prompt that comes back activates the same experts again.
# ---------------------------------------------------------------------------

def prompt_pool(cfg: MoEShape, P: int, n_tok: int, V: int) -> np.ndarray:
    """[P, n_tok] int32 token ids, uniform over the vocabulary 0..V-1."""
    g = np.random.Generator(np.random.PCG64(_seq(cfg.cfg_id, PROMPTS, P, n_tok, V)))
    return g.integers(0, V, size=(P, n_tok)).astype(np.int32)


def prompt_draws(cfg: MoEShape, step: int, T: int, P: int, zipf_s: float = 1.1) -> np.ndarray:
    """[T] int32: which prompt of the pool each of the T requests of a step carries; prompt p is drawn with
    probability proportional to (p + 1)^-s."""
    g = np.random.Generator(np.random.PCG64(_seq(cfg.cfg_id, PROMPTS, 1, step, T, P)))
    w = (np.arange(1, P + 1, dtype=np.float64)) ** (-zipf_s)
    return g.choice(P, size=T, p=w / w.sum()).astype(np.int32)


def prompt_hidden(cfg: MoEShape, P: int, n_layers: int) -> np.ndarray:
    """[n_layers, P, d] bf16: per prompt h_0 ~ N(0,1) and h_{l+1} = bf16(f32(h_l) + noise * N(0,1)), fixed per
    (prompt, layer): the same recipe as hidden_stack, keyed by the prompt instead of the step."""
    hs = [normal_bf16((P, cfg.d), (cfg.cfg_id, PROMPTS, 2, P))]
    for l in range(1, n_layers):
        n = normal_f32(P * cfg.d, (cfg.cfg_id, PROMPTS, 3, P, l), cfg.noise).reshape(P, cfg.d)
        hs.append(f32_to_bf16(bf16_to_f32(hs[-1]) + n))
    return np.stack(hs)


def feature_embedding(cfg: MoEShape, V: int, d_emb: int) -> np.ndarray:
    """[V, d_emb] float32 ~ N(0,1): the fixed random embedding table of the predictor's features."""
    return normal_f32(V * d_emb, (cfg.cfg_id, FEATURE_EMB, V, d_emb)).reshape(V, d_emb)


def bootstrap_indices(cfg: MoEShape, n_trees: int, N: int) -> np.ndarray:
    """[n_trees, N] int32 uniform draws from 0..N-1 (the forest's bootstrap samples)."""
    g = np.random.Generator(np.random.PCG64(_seq(cfg.cfg_id, BOOTSTRAP, n_trees, N)))
    return g.integers(0, N, size=(n_trees, N)).astype(np.int32)
