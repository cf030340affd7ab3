"""Pins of the CPU oracle against things other than itself (CPU only).

Library routines used as references run in torch fp64 on the CPU; brute force
and closed forms cover the integer steps.  Each pin is chosen so that a
plausible slip (dropped bias, transposed operand, wrong tie-break, biased
weights, off-by-one in the prefix) makes at least one of them fail.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from paper_2510_26730_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def t_bf16(u16):
    """Decode bf16 bit patterns with torch's own bfloat16 (independent of the oracle's decoder)."""
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to(torch.float64)


def rnd_bf16(shape, seed, scale=1.0):
    g = np.random.default_rng(seed)
    return synth.f32_to_bf16((g.standard_normal(shape) * scale).astype(np.float32))


def torch_swiglu(x, w1, w3, w2):
    g = x @ w1.T
    u = x @ w3.T
    return (torch.nn.functional.silu(g) * u) @ w2.T


# ---------------------------------------------------------------- gate + softmax
def test_gate_logits_match_torch_matmul(oracle_mod):
    h = rnd_bf16((37, 96), 1)
    Wg = rnd_bf16((11, 96), 2, 0.05)
    b = np.random.default_rng(3).standard_normal(11).astype(np.float32)
    z = oracle_mod.gate_logits(h, Wg, b)
    ref = t_bf16(h) @ t_bf16(Wg).T + torch.from_numpy(b).double()
    assert np.max(np.abs(z - ref.numpy())) < 1e-12
    z0 = oracle_mod.gate_logits(h, Wg, None)
    assert np.max(np.abs(z0 - (t_bf16(h) @ t_bf16(Wg).T).numpy())) < 1e-12


def test_softmax_rows_sum_to_one_and_match_library(oracle_mod):
    z = np.random.default_rng(4).standard_normal((50, 60)) * 5.0
    z[3] += 700.0          # would overflow exp() without the max shift
    p = oracle_mod.softmax(z)
    assert np.all(p >= 0.0)
    assert np.max(np.abs(p.sum(axis=1) - 1.0)) < 1e-12
    ref = torch.softmax(torch.from_numpy(z), dim=1).numpy()
    assert np.max(np.abs(p - ref)) < 1e-14
    # closed form for two experts: p0 = 1 / (1 + exp(z1 - z0))
    z2 = np.array([[0.3, -1.2]])
    assert abs(oracle_mod.softmax(z2)[0, 0] - 1.0 / (1.0 + math.exp(-1.5))) < 1e-15


# ---------------------------------------------------------------- top-k
@pytest.mark.parametrize("E,k", [(5, 1), (6, 2), (8, 2), (8, 3), (7, 7)])
def test_topk_is_the_best_subset_by_brute_force(oracle_mod, E, k):
    s = np.random.default_rng(10 * E + k).standard_normal((40, E))
    ids, gap = oracle_mod.topk(s, k)
    for t in range(s.shape[0]):
        best = max(itertools.combinations(range(E), k), key=lambda c: s[t, list(c)].sum())
        assert tuple(ids[t]) == best                      # ascending ids == combinations order
        srt = np.sort(s[t])[::-1]
        if k < E:
            assert abs(gap[t] - (srt[k - 1] - srt[k])) < 1e-15
        else:
            assert np.isinf(gap[t])


def test_topk_ties_go_to_the_lower_id(oracle_mod):
    s = np.array([[1.0, 2.0, 2.0, 2.0, 0.0],
                  [5.0, 5.0, 5.0, 5.0, 5.0],
                  [0.0, 1.0, 0.0, 1.0, 1.0]])
    ids, gap = oracle_mod.topk(s, 2)
    assert ids.tolist() == [[1, 2], [0, 1], [1, 3]]
    assert gap.tolist() == [0.0, 0.0, 0.0]


def test_zero_bias_zero_delta_is_plain_topk(oracle_mod):
    z = np.random.default_rng(5).standard_normal((64, 60))
    s = oracle_mod.scores(z, 0.0, np.ones(60, np.uint8), None, None)
    assert np.array_equal(s, z)
    s = oracle_mod.scores(z, 3.0, np.zeros(60, np.uint8), np.zeros((2, 60), np.float32),
                          np.zeros(64, np.int32))
    assert np.array_equal(s, z)
    ids, _ = oracle_mod.topk(z, 4)
    ref = torch.topk(torch.from_numpy(z), 4, dim=1).indices.sort(dim=1).values.numpy()
    assert np.array_equal(ids, ref)


def test_residency_bias_and_delta_enter_the_score_only(oracle_mod):
    rng = np.random.default_rng(6)
    z = rng.standard_normal((32, 16))
    res = np.zeros(16, np.uint8)
    res[[2, 5, 11]] = 1
    delta = rng.standard_normal((3, 16)).astype(np.float32)
    t2r = rng.integers(0, 3, 32).astype(np.int32)
    s = oracle_mod.scores(z, 1.5, res, delta, t2r)
    ref = z + 1.5 * res[None, :].astype(np.float64) + delta[t2r].astype(np.float64)
    assert np.max(np.abs(s - ref)) == 0.0
    # a large bias with >= k resident experts routes everything to resident experts
    ids, _ = oracle_mod.topk(oracle_mod.scores(z, 100.0, res, None, None), 3)
    assert np.all(np.isin(ids, [2, 5, 11]))
    # weights come from the unbiased distribution whatever beta is
    p = oracle_mod.softmax(z)
    w = oracle_mod.weights(p, ids, False)
    assert np.max(np.abs(w - np.take_along_axis(p, ids.astype(np.int64), axis=1))) == 0.0
    wn = oracle_mod.weights(p, ids, True, 2.5)
    assert np.max(np.abs(wn.sum(axis=1) - 2.5)) < 1e-14
    assert np.max(np.abs(wn / wn.sum(axis=1, keepdims=True) - w / w.sum(axis=1, keepdims=True))) < 1e-14


# ---------------------------------------------------------------- histogram + permutation
@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (64, 2, 8), (33, 6, 64), (640, 4, 60)])
def test_histogram_and_permutation_invariants(oracle_mod, T, k, E):
    rng = np.random.default_rng(T + k + E)
    ids = np.stack([np.sort(rng.permutation(E)[:k]) for _ in range(T)]).astype(np.int32)
    hist = oracle_mod.histogram(ids, E)
    counts, offsets, perm, inv = oracle_mod.permute(ids, E)
    n = T * k
    assert hist.sum() == n and np.array_equal(hist, counts)
    assert np.array_equal(hist, np.bincount(ids.ravel(), minlength=E))
    assert counts.max() <= T
    assert offsets[0] == 0 and offsets[E] == n
    assert np.array_equal(np.diff(offsets), counts)
    assert np.array_equal(perm[inv], np.arange(n)) and np.array_equal(inv[perm], np.arange(n))
    flat = ids.ravel()
    assert np.all(np.diff(flat[perm]) >= 0)
    # the stable order is the library's stable argsort of the expert ids
    assert np.array_equal(perm, np.argsort(flat, kind="stable").astype(np.int32))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


# ---------------------------------------------------------------- FFN + combine
def test_single_expert_is_a_plain_swiglu_mlp(oracle_mod):
    d, F, T = 48, 80, 9
    h = rnd_bf16((T, d), 20)
    w1, w3, w2 = rnd_bf16((F, d), 21, 0.2), rnd_bf16((F, d), 22, 0.2), rnd_bf16((d, F), 23, 0.2)
    r = oracle_mod.moe_layer(h, rnd_bf16((1, d), 24), None, [(w1, w3, w2)], 1, renorm=False)
    ref = torch_swiglu(t_bf16(h), t_bf16(w1), t_bf16(w3), t_bf16(w2)).numpy()
    assert np.all(r["ids"] == 0) and np.max(np.abs(r["w"] - 1.0)) == 0.0
    assert np.max(np.abs(r["out"] - ref)) < 1e-12 * max(1.0, np.abs(ref).max())
    dense = oracle_mod.dense_ffn(h, w1, w3, w2)
    assert np.max(np.abs(dense - ref)) < 1e-12 * max(1.0, np.abs(ref).max())


def test_k_equals_E_is_the_dense_mixture(oracle_mod):
    d, F, T, E = 32, 40, 12, 5
    h = rnd_bf16((T, d), 30)
    Wg = rnd_bf16((E, d), 31, 0.3)
    b = np.random.default_rng(32).standard_normal(E).astype(np.float32)
    ex = [(rnd_bf16((F, d), 33 + 3 * e, 0.2), rnd_bf16((F, d), 34 + 3 * e, 0.2),
           rnd_bf16((d, F), 35 + 3 * e, 0.2)) for e in range(E)]
    r = oracle_mod.moe_layer(h, Wg, b, ex, E, renorm=False)
    x = t_bf16(h)
    p = torch.softmax(x @ t_bf16(Wg).T + torch.from_numpy(b).double(), dim=1)
    ref = sum(p[:, e:e + 1] * torch_swiglu(x, *(t_bf16(w) for w in ex[e])) for e in range(E)).numpy()
    assert np.max(np.abs(r["out"] - ref)) < 1e-12 * max(1.0, np.abs(ref).max())


def test_tiny_config_layer_against_dense_masked_evaluation(oracle_mod):
    cfg = synth.CONFIGS["tiny"]
    T = 16
    h = synth.hidden(cfg, 0, T)
    Wg, b = synth.gate_weight(cfg, 0), synth.gate_bias(cfg, 0)
    ex = [synth.expert_weights(cfg, 0, e) for e in range(cfg.E)]
    res = synth.residency(cfg, 0)
    beta = 0.75
    r = oracle_mod.moe_layer(h, Wg, b, ex, cfg.k, beta=beta, resident=res, renorm=True)
    x = t_bf16(h)
    z = x @ t_bf16(Wg).T + torch.from_numpy(b).double()
    p = torch.softmax(z, dim=1)
    s = z + beta * torch.from_numpy(res.astype(np.float64))
    top = torch.topk(s, cfg.k, dim=1).indices
    mask = torch.zeros_like(p).scatter_(1, top, 1.0)
    wfull = p * mask
    wfull = wfull / wfull.sum(dim=1, keepdim=True)
    ref = sum(wfull[:, e:e + 1] * torch_swiglu(x, *(t_bf16(w) for w in ex[e])) for e in range(cfg.E)).numpy()
    assert np.array_equal(r["ids"], top.sort(dim=1).values.numpy())
    assert np.max(np.abs(r["out"] - ref)) < 1e-11


def test_shared_expert_is_added_with_weight_one(oracle_mod):
    d, F, Fs, T, E, k = 32, 24, 40, 7, 4, 2
    h = rnd_bf16((T, d), 40)
    Wg = rnd_bf16((E, d), 41, 0.3)
    ex = [(rnd_bf16((F, d), 42 + 3 * e, 0.2), rnd_bf16((F, d), 43 + 3 * e, 0.2),
           rnd_bf16((d, F), 44 + 3 * e, 0.2)) for e in range(E)]
    sh = (rnd_bf16((Fs, d), 60, 0.2), rnd_bf16((Fs, d), 61, 0.2), rnd_bf16((d, Fs), 62, 0.2))
    a = oracle_mod.moe_layer(h, Wg, None, ex, k, renorm=False)
    c = oracle_mod.moe_layer(h, Wg, None, ex, k, renorm=False, shared=sh)
    ref = torch_swiglu(t_bf16(h), *(t_bf16(w) for w in sh)).numpy()
    assert np.max(np.abs((c["out"] - a["out"]) - ref)) < 1e-12


def test_round_act_mode_rounds_like_bfloat16(oracle_mod):
    d, F, T = 16, 24, 5
    h = rnd_bf16((T, d), 50)
    w1, w3, w2 = rnd_bf16((F, d), 51, 0.4), rnd_bf16((F, d), 52, 0.4), rnd_bf16((d, F), 53, 0.4)
    out = oracle_mod.dense_ffn(h, w1, w3, w2, round_act=True)
    x = t_bf16(h)
    act = torch.nn.functional.silu(x @ t_bf16(w1).T) * (x @ t_bf16(w3).T)
    act = act.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    assert np.max(np.abs(out - (act @ t_bf16(w2).T).numpy())) < 1e-12


def test_round_act_mode_2_rounds_like_float16(oracle_mod):
    """The diagnostic mode that mirrors an fp16 scratch between the FFN halves, against torch's own
    float16 rounding; scaled inputs put activations below the fp16 normal range and above its maximum."""
    d, F, T = 16, 24, 5
    w1, w3, w2 = rnd_bf16((F, d), 51, 0.4), rnd_bf16((F, d), 52, 0.4), rnd_bf16((d, F), 53, 0.4)
    for scale in (1.0, 0.004, 300.0):
        h = rnd_bf16((T, d), 50, scale)
        out = oracle_mod.dense_ffn(h, w1, w3, w2, round_act=2)
        x = t_bf16(h)
        act = torch.nn.functional.silu(x @ t_bf16(w1).T) * (x @ t_bf16(w3).T)
        if scale == 0.004:
            assert (act.abs() < 2.0 ** -14).any()
        if scale == 300.0:
            assert (act.abs() > 65504).any()
        act = act.clamp(-65504.0, 65504.0).to(torch.float16).to(torch.float64)
        ref = (act @ t_bf16(w2).T).numpy()
        assert np.max(np.abs(out - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


# ---------------------------------------------------------------- predictor
def test_predict_with_own_gate_equals_route_and_identical_gates_agree(oracle_mod):
    cfg = synth.CONFIGS["tiny"]
    h = synth.hidden(cfg, 1, 32)
    Wg, b = synth.gate_weight(cfg, 0), synth.gate_bias(cfg, 0)
    res = synth.residency(cfg, 0)
    r = oracle_mod.route(h, Wg, b, cfg.k, beta=0.5, resident=res)
    ids, hist, gap = oracle_mod.predict(h, [Wg, Wg, Wg], [b, b, b], cfg.k, 0.5, [res, res, res])
    for j in range(3):
        assert np.array_equal(ids[j], r["ids"]) and np.array_equal(hist[j], r["hist"])
        assert np.array_equal(gap[j], r["gap"])
    assert hist.sum(axis=1).tolist() == [32 * cfg.k] * 3


def test_prediction_overlap_decays_with_lookahead(oracle_mod):
    """Pre-gating on the synthetic recurrence: further ahead = less overlap (paper Sec. 4.3 trend)."""
    cfg = synth.CONFIGS["tiny"]
    hs = synth.hidden_stack(cfg, 5, step=7, T=256)
    Wg, b = synth.gate_weight(cfg, 0), synth.gate_bias(cfg, 0)
    base = oracle_mod.route(hs[0], Wg, b, cfg.k)["ids"]
    overlap = []
    for j in range(5):
        actual = oracle_mod.route(hs[j], Wg, b, cfg.k)["ids"]
        overlap.append(np.mean([len(set(a) & set(p)) / cfg.k for a, p in zip(actual, base)]))
    assert overlap[0] == 1.0
    assert all(overlap[j] >= overlap[j + 1] - 0.02 for j in range(4))
    assert overlap[4] < overlap[1]


# ---------------------------------------------------------------- horizon
def test_step_size_equation_hand_values(oracle_mod):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "step_size_cases.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 8
    for n_e, es, cs, tl, hmax, s_raw, hor in rows:
        raw = oracle_mod.step_size_raw(float(n_e), float(es), float(cs), float(tl))
        assert abs(raw - float(s_raw)) <= 6e-4 * max(1.0, float(s_raw)), (n_e, es, cs, tl)
        assert oracle_mod.horizon(float(n_e), float(es), float(cs), float(tl), int(hmax)) == int(hor)


def test_step_size_monotone(oracle_mod):
    f = oracle_mod.step_size_raw
    assert f(4, 1e6, 1e9, 1e-3) > f(2, 1e6, 1e9, 1e-3)
    assert f(2, 2e6, 1e9, 1e-3) > f(2, 1e6, 1e9, 1e-3)
    assert f(2, 1e6, 2e9, 1e-3) < f(2, 1e6, 1e9, 1e-3)
    assert f(2, 1e6, 1e9, 2e-3) < f(2, 1e6, 1e9, 1e-3)


@pytest.mark.parametrize("tau", [0.05, 0.5, 0.9, 1.0])
def test_expected_activations_by_brute_force(oracle_mod, tau):
    rng = np.random.default_rng(int(tau * 100))
    for _ in range(20):
        E = int(rng.integers(1, 9))
        hist = rng.integers(0, 6, E).astype(np.int32)
        res = rng.integers(0, 2, E).astype(np.uint8)
        n, miss, order = oracle_mod.expected_activations(hist, tau, res)
        tot = int(hist.sum())
        srt = sorted(range(E), key=lambda e: (-int(hist[e]), e))
        assert order.tolist() == srt
        if tot == 0:
            assert n == 0 and miss == 0
            continue
        want = next(m for m in range(1, E + 1) if sum(int(hist[e]) for e in srt[:m]) / tot >= tau)
        assert n == want
        assert miss == sum(1 for e in srt[:want] if not res[e])
        if tau == 1.0:
            assert n == int(np.count_nonzero(hist))
    assert oracle_mod.expected_activations(np.array([5, 1, 9, 0], np.int32), 1e-9)[0] == 1


# ---------------------------------------------------------------------------
# intra-batch diversity Dist(t) (paper Sec. 2.2)
# ---------------------------------------------------------------------------

def test_token_dist_matches_scipy_pdist(oracle_mod):
    """Library routine: the sum of scipy's condensed pairwise Euclidean distances (fp64)."""
    from scipy.spatial.distance import pdist, squareform
    rng = np.random.default_rng(11)
    h = synth.f32_to_bf16(rng.standard_normal((37, 96)).astype(np.float32))
    v = synth.bf16_to_f32(h).astype(np.float64)
    s = oracle_mod.token_dist(h)
    assert s.shape == (37,)
    assert abs(s.sum() - pdist(v, "euclidean").sum()) < 1e-9 * s.sum()
    full = squareform(pdist(v, "euclidean"))
    ref = np.array([full[j, :j].sum() for j in range(37)])       # earlier tokens only
    np.testing.assert_allclose(s, ref, rtol=1e-12, atol=1e-12)
    js = np.array([36, 0, 5], dtype=np.int32)                     # sampled form, any order
    np.testing.assert_allclose(oracle_mod.token_dist(h, js), ref[js], rtol=1e-12, atol=1e-12)


def test_token_dist_closed_forms(oracle_mod):
    """Scaled basis vectors: ||a_i e_i - a_j e_j|| = sqrt(a_i^2 + a_j^2); duplicates add nothing;
    one token has no pair; a translation of all tokens changes nothing (values exact in bf16)."""
    a = np.array([1.0, 2.0, 0.5, 4.0, 3.0])
    v = np.zeros((5, 8), dtype=np.float32)
    v[np.arange(5), np.arange(5)] = a
    h = synth.f32_to_bf16(v)
    s = oracle_mod.token_dist(h)
    ref = np.array([sum(np.hypot(a[i], a[j]) for i in range(j)) for j in range(5)])
    np.testing.assert_allclose(s, ref, rtol=1e-14)
    dup = synth.f32_to_bf16(np.tile(v[3], (6, 1)))
    assert np.all(oracle_mod.token_dist(dup) == 0.0)
    assert oracle_mod.token_dist(h[:1]).tolist() == [0.0]
    shifted = synth.f32_to_bf16(v + 8.0)                          # small integers and halves stay exact
    np.testing.assert_allclose(oracle_mod.token_dist(shifted), ref, rtol=1e-14)
    # a plausible mistake (squared distances, or all pairs counted twice) fails these values
    assert abs(s.sum() - sum(np.hypot(a[i], a[j]) for j in range(5) for i in range(j))) < 1e-12


# ---------------------------------------------------------------------------
# 4-bit expert weights: w = (q - 8) * s, one scale per row and 128 inputs
# ---------------------------------------------------------------------------

def _q4_cfg():
    import dataclasses as dc
    return dc.replace(synth.CONFIGS["tiny"], name="tiny_q4", d=256, F=384, E=4, k=2)


def test_q4_expert_ffn_matches_torch_on_dequantised_weights(oracle_mod):
    """Library routine: torch fp64 matmul / silu with the dequantised matrices, grouped by expert."""
    cfg = _q4_cfg()
    T = 9
    h = synth.hidden(cfg, 0, T)
    experts = [synth.expert_weights_q4(cfg, 0, e) for e in range(cfg.E)]
    rng = np.random.default_rng(3)
    ids = np.stack([np.sort(rng.choice(cfg.E, cfg.k, replace=False)) for _ in range(T)]).astype(np.int32)
    perm = oracle_mod.permute(ids, cfg.E)[2]
    y = oracle_mod.expert_ffn_q4(h, experts, ids, perm)
    x = torch.from_numpy(synth.bf16_to_f32(h).astype(np.float64))
    for pos, a in enumerate(perm):
        e = int(ids.reshape(-1)[a])
        q1, s1, q3, s3, q2, s2 = experts[e]
        W1 = torch.from_numpy(synth.dequant_q4(q1, s1))
        W3 = torch.from_numpy(synth.dequant_q4(q3, s3))
        W2 = torch.from_numpy(synth.dequant_q4(q2, s2))
        xt = x[a // cfg.k]
        ref = W2 @ (torch.nn.functional.silu(W1 @ xt) * (W3 @ xt))
        np.testing.assert_allclose(y[pos], ref.numpy(), rtol=1e-10, atol=1e-12)


def test_q4_special_codes(oracle_mod):
    """Code 8 is zero; with all scales 1 and codes 9 the matrices are all-ones: closed form."""
    import dataclasses as dc
    cfg = dc.replace(synth.CONFIGS["tiny"], name="q4s", d=128, F=128, E=1, k=1)
    h = synth.f32_to_bf16(np.full((2, 128), 0.5, dtype=np.float32))
    one = synth.f32_to_bf16(np.ones((128, 1), dtype=np.float32))
    ids = np.zeros((2, 1), dtype=np.int32)
    perm = np.arange(2, dtype=np.int32)
    q9 = np.full((128, 128), 9, dtype=np.uint8)
    q8 = np.full((128, 128), 8, dtype=np.uint8)
    y = oracle_mod.expert_ffn_q4(h, [(q9, one, q9, one, q9, one)], ids, perm)
    g = 64.0                                           # 128 inputs of 0.5 through a row of ones
    np.testing.assert_allclose(y, 128 * (g / (1 + np.exp(-g)) * g), rtol=1e-12)
    y0 = oracle_mod.expert_ffn_q4(h, [(q9, one, q9, one, q8, one)], ids, perm)
    assert np.all(y0 == 0.0)
    # the scale belongs to the row and the 128-input group: doubling one W2 row doubles that output
    two = one.copy()
    two[5] = synth.f32_to_bf16(np.array([2.0], dtype=np.float32))
    y2 = oracle_mod.expert_ffn_q4(h, [(q9, one, q9, one, q9, two)], ids, perm)
    np.testing.assert_allclose(y2[:, 5], 2 * y[:, 5], rtol=1e-12)
    np.testing.assert_allclose(np.delete(y2, 5, axis=1), np.delete(y, 5, axis=1), rtol=1e-12)
